"""Model Profiler for stages of this library on one MI355X (Profiling Engine, "Model Profiler").

Synthetic microbatches are run through a stage on a grid of input sizes; the measured throughput
(model FLOPs per second, forward + backward) and the memory the stage needs become the grids that
`mllm_interp`, `mllm_item_durations` and `mllm_optimize_parallelism` read.  As in the paper the
encoder is profiled against its effective batch size (images per microbatch) and the LLM against
the sequence length, attention and the linear operations separately ("Throughput Profiling").
Only TP degree 1 can be measured on one GPU.

The caller supplies the microbatches: `make_images(b)` builds a microbatch of b images,
`make_partition(total, n)` one of `total` packed tokens cut into n equal samples.  A microbatch is
any object with the fields of mllm_batch_t (img / seq packs with cu_seqlens and mask_kind).

FLOP convention: 2mnk per GEMM, backward = 2 x forward, causal attention at half the square, no
credit for recomputation.
"""
from __future__ import annotations

from typing import Callable, List, Sequence, Tuple

import numpy as np

from . import binding as B

# values of the C ABI's enums (mllm_stage.h)
LAYER_VIT, LAYER_DECODER, LAYER_PROJECTOR = 0, 1, 2
MASK_CAUSAL = 1

BYTES_PER_PARAM_STATE = 18.0   # bf16 weight + fp32 gradient + fp32 master copy and two Adam moments


def visible_pairs(pack) -> float:
    lens = np.diff(pack.cu_seqlens).astype(np.float64)
    w = np.where(pack.mask_kind == MASK_CAUSAL, 0.5, 1.0)
    return float(np.sum(w * lens * lens))


def stage_fwd_flops(layers, batch) -> Tuple[float, float]:
    """(linear, attention) forward model FLOPs of a stage over a microbatch."""
    lin = attn = 0.0
    for L in layers:
        if L.kind == LAYER_PROJECTOR:
            lin += 2.0 * batch.img.total_tokens * L.d_model * L.d_out
            continue
        pack = batch.img if L.kind == LAYER_VIT else batch.seq
        T = pack.total_tokens
        nqkv = (L.n_q_heads + 2 * L.n_kv_heads) * L.head_dim
        fup = L.d_ff if L.kind == LAYER_VIT else 2 * L.d_ff
        lin += 2.0 * T * L.d_model * (nqkv + L.d_model + fup) + 2.0 * T * L.d_ff * L.d_model
        attn += 4.0 * visible_pairs(pack) * L.n_q_heads * L.head_dim
    return lin, attn


class StageRunner:
    """Parameters of a stage allocated once; times forward+backward on any microbatch."""

    def __init__(self, layers):
        import torch
        self.torch, self.layers = torch, layers
        B.lib()
        self.dev = torch.device("cuda:0")
        self.h = B.mllm_stage_create(layers)
        infos = [B.mllm_stage_param_info(self.h, i) for i in range(B.mllm_stage_param_count(self.h))]
        self.gen = torch.Generator(device=self.dev)
        self.gen.manual_seed(99)
        self.params = [self.randn(r, c, 0.02, 1.0 if name.endswith("_g") else 0.0) for name, _, r, c in infos]
        self.dparams = [torch.zeros(r, c, dtype=torch.float32, device=self.dev) for _, _, r, c in infos]

    def randn(self, r, c, scale=1.0, shift=0.0):
        t = self.torch
        return (t.randn(r, c, generator=self.gen, device=self.dev, dtype=t.float32) * scale + shift).to(t.bfloat16)

    def _buffers(self, batch):
        t, layers = self.torch, self.layers
        kinds = [l.kind for l in layers]
        uses_img = kinds[0] in (LAYER_VIT, LAYER_PROJECTOR)
        uses_seq = LAYER_DECODER in kinds or LAYER_PROJECTOR in kinds
        x_img = self.randn(batch.img.total_tokens, layers[0].d_model) if uses_img else None
        d_seq = next((l.d_out if l.kind == LAYER_PROJECTOR else l.d_model) for l in layers
                     if l.kind != LAYER_VIT) if uses_seq else 0
        x_seq = self.randn(batch.seq.total_tokens, d_seq) if uses_seq else None
        last = layers[-1]
        rows = batch.img.total_tokens if last.kind == LAYER_VIT else batch.seq.total_tokens
        cols = last.d_out if last.kind == LAYER_PROJECTOR else last.d_model
        dy = self.randn(rows, cols)
        y = t.empty(rows, cols, dtype=t.bfloat16, device=self.dev)
        sb, wb = B.mllm_stage_sizes(self.h, batch)
        saved = t.empty(sb, dtype=t.uint8, device=self.dev)
        ws = t.empty(wb, dtype=t.uint8, device=self.dev)
        return x_img, x_seq, dy, y, saved, ws

    def _step(self, batch, bufs):
        x_img, x_seq, dy, y, saved, ws = bufs
        B.mllm_stage_fwd(self.h, batch, self.params, x_img, x_seq, y, saved, ws)
        B.mllm_stage_bwd(self.h, batch, self.params, dy, saved, None, None, self.dparams, 0, ws)

    def time(self, batch, steps=None, warmup=1) -> float:
        """Milliseconds per forward+backward step (HIP events on the launch stream): the faster of
        two timed runs (clock ramps and other tenants of the host show up as slow outliers).
        Without a step count, short steps are repeated until about 80 ms are timed (2 to 16 steps)."""
        t = self.torch
        bufs = self._buffers(batch)

        def timed(n):
            e0, e1 = t.cuda.Event(enable_timing=True), t.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(n):
                self._step(batch, bufs)
            e1.record()
            t.cuda.synchronize()
            return e0.elapsed_time(e1) / n

        for _ in range(warmup):
            self._step(batch, bufs)
        if steps is None:
            steps = int(min(16, max(2, round(80.0 / max(timed(1), 1e-3)))))
        return min(timed(steps), timed(steps))

    def time_split(self, batch, steps=None, warmup=1) -> Tuple[float, float]:
        """(ms per step, ms of it inside the attention kernels).  The step is timed without
        per-launch records; the attention kernels' own durations come from one recorded step."""
        total = self.time(batch, steps, warmup)
        bufs = self._buffers(batch)
        self.torch.cuda.synchronize()
        B.mllm_profile_begin(64 * len(self.layers) + 64)
        self._step(batch, bufs)
        self.torch.cuda.synchronize()
        prof, _ = B.mllm_profile_end()
        attn = prof["attn_fwd"][1] + prof["attn_bwd"][1]
        return total, min(attn, total)

    def close(self):
        B.mllm_stage_destroy(self.h)


def profile_encoder(runner: StageRunner, image_counts: Sequence[int], make_images: Callable[[int], object]):
    """E_thr over the effective batch size: (x, FLOP/s, ms per step)."""
    thr, ms = [], []
    for b in image_counts:
        batch = make_images(int(b))
        lin, attn = stage_fwd_flops(runner.layers, batch)
        t = runner.time(batch)
        ms.append(t)
        thr.append(3.0 * (lin + attn) / (t * 1e-3))
    return np.array(image_counts, dtype=np.float64), np.array(thr), np.array(ms)


def profile_llm(runner: StageRunner, seq_lens: Sequence[int], make_partition: Callable[[int, int], object],
                packed_tokens: int = 16384):
    """L_lin_thr and L_attn_thr over the sequence length ("Throughput Profiling": the two are
    measured independently).  Linear operations see only the packed length, so their throughput at
    s comes from one sequence of s tokens (step time minus the attention kernels' time).
    Attention handles every sample on its own, but its kernels run all samples of a microbatch in
    one launch: its throughput at sample length s is measured on `packed_tokens` tokens cut into
    equal samples of s (one sample when s is longer), the occupancy it will have in training.
    Returns (x, linear FLOP/s, attention FLOP/s, ms per step of the lone sequence, ms of it inside
    attention, attention ms of the packed partition)."""
    lin_thr, attn_thr, ms, ms_attn, ms_attn_packed = [], [], [], [], []
    for s in seq_lens:
        lone = make_partition(int(s), 1)
        lin, _ = stage_fwd_flops(runner.layers, lone)
        total, t_attn = runner.time_split(lone)
        ms.append(total)
        ms_attn.append(t_attn)
        lin_thr.append(3.0 * lin / ((total - t_attn) * 1e-3))
        n_seg = max(1, packed_tokens // int(s))
        packed = make_partition(int(s) * n_seg, n_seg)
        _, attn = stage_fwd_flops(runner.layers, packed)
        _, t_attn_p = runner.time_split(packed) if n_seg > 1 else (total, t_attn)
        ms_attn_packed.append(t_attn_p)
        attn_thr.append(3.0 * attn / (t_attn_p * 1e-3))
    return (np.array(seq_lens, dtype=np.float64), np.array(lin_thr), np.array(attn_thr), np.array(ms),
            np.array(ms_attn), np.array(ms_attn_packed))


def memory_tables(make_layers: Callable[[int], List], make_batch: Callable[[float], object],
                  grid: Sequence[float], layer_counts: Tuple[int, int] = (2, 4)):
    """Model states and activation states at two small layer counts ("Memory Profiling"), from the
    library's own size queries (no GPU work): model_state[2] bytes, act_state[2][len(grid)] bytes.
    Activation state = what the forward pass keeps for the backward pass."""
    model_state, act_state = [], []
    for n in layer_counts:
        h = B.mllm_stage_create(make_layers(n))
        n_param = sum(r * c for _, _, r, c in (B.mllm_stage_param_info(h, i) for i in range(B.mllm_stage_param_count(h))))
        model_state.append(BYTES_PER_PARAM_STATE * n_param)
        act_state.append([float(B.mllm_stage_sizes(h, make_batch(x))[0]) for x in grid])
        B.mllm_stage_destroy(h)
    return model_state, act_state
