"""Seeded synthetic microbatches and parameters for the pipeline-stage path.

This module only *draws inputs*: sample-length mixes, packed-sequence index
arrays, random tensors and layer descriptors.  It holds none of the stage's
arithmetic, so both the fp64 CPU oracle's tests and the HIP path's tests and
benchmark can feed the very same seeded data to the two implementations.

The length mixes stand in for the paper's dataset mix (Evaluation, Table 3:
single-image, multi-image and video items): every item contributes a variable
number of fixed-size groups of visual tokens plus a variable number of text
tokens (Data Profiler, Section 3.2), and the items of a microbatch are packed
along the sequence dimension (Model Profiler, "Memory Profiling").

All tensors are drawn in fp32 with NumPy's PCG64 generator and then rounded
once, round-to-nearest-even, to the bf16 grid; both implementations consume
the rounded values.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

# ---- enums shared by name with the C header (values are part of the interface) ----
LAYER_VIT, LAYER_DECODER, LAYER_PROJECTOR = 0, 1, 2
ACT_GELU_ERF, ACT_GELU_TANH, ACT_SWIGLU = 0, 1, 2
MASK_BIDIR, MASK_CAUSAL = 0, 1

IMG_TOKENS = 576  # 24 x 24 patches of a 336-pixel image at patch size 14


# ---------------------------------------------------------------------------
# bf16 grid helpers (input preparation only)
# ---------------------------------------------------------------------------
def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns (uint16), round to nearest even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def from_bf16_bits(b: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> fp32."""
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_round(x: np.ndarray) -> np.ndarray:
    """Round an fp32 array onto the bf16 grid and return it as fp32."""
    return from_bf16_bits(to_bf16_bits(x)).reshape(np.shape(x))


# ---------------------------------------------------------------------------
# descriptors
# ---------------------------------------------------------------------------
@dataclass
class LayerDesc:
    kind: int
    d_model: int            # input width (projector: input width)
    n_q_heads: int = 0
    n_kv_heads: int = 0
    head_dim: int = 0
    d_ff: int = 0
    d_out: int = 0          # projector output width
    act: int = ACT_GELU_ERF
    has_bias: int = 0
    norm_eps: float = 1e-5
    rope_base: float = 10000.0
    pool: int = 0           # projector: average-pool this many consecutive encoder tokens first (0/1: none)
    merge: int = 0          # projector: concatenate this many consecutive encoder tokens into one row (0/1: none)
    qk_norm: int = 0        # ViT / decoder: RMS-normalise the q rows and the k rows (all heads together) before attention


def vit_layer(d, heads, head_dim, d_ff, eps=1e-5, act=ACT_GELU_ERF, qk_norm=0) -> LayerDesc:
    """qk_norm = 1: the query rows and the key rows (all heads of a token together) pass through an
    RMSNorm with a gain of their own before attention (the InternViT kind of QK normalisation)."""
    return LayerDesc(LAYER_VIT, d, heads, heads, head_dim, d_ff, 0, act, 1, eps, 0.0, qk_norm=qk_norm)


def decoder_layer(d, hq, hkv, head_dim, d_ff, rope_base, eps=1e-5, qkv_bias=0, qk_norm=0) -> LayerDesc:
    """has_bias = 1 on a decoder layer: the QKV projection (and only it) has a bias.  qk_norm = 1:
    as for vit_layer, applied before the rotary embedding."""
    return LayerDesc(LAYER_DECODER, d, hq, hkv, head_dim, d_ff, 0, ACT_SWIGLU, qkv_bias, eps, rope_base,
                     qk_norm=qk_norm)


def projector_layer(d_in, d_out, d_hidden=0, act=ACT_GELU_ERF, pool=0, merge=0) -> LayerDesc:
    """d_hidden = 0: one biased linear map; otherwise a two-layer MLP d_in -> d_hidden -> d_out
    with a GELU in between (d_ff carries d_hidden).  pool > 1: every `pool` consecutive encoder
    tokens of a segment are averaged first, so fewer tokens reach the LLM; merge > 1: every `merge`
    consecutive encoder tokens are concatenated into one row of width merge * d_in instead (token
    merging of the pixel-shuffle kind: the caller orders the patches so that those to be merged
    are adjacent)."""
    return LayerDesc(LAYER_PROJECTOR, d_in, 0, 0, 0, d_hidden, d_out, act if d_hidden else 0, 1, 0.0, 0.0, pool, merge)


def param_specs(layer: LayerDesc) -> List[Tuple[str, int, int]]:
    """(name, rows, cols) of every parameter tensor of a layer, in interface order.

    Matrices are row-major [in, out]; vectors are [1, n].  The QKV matrix is
    [Wq | Wk | Wv] along columns, the decoder's MLP-up matrix is [W_gate | W_up].
    """
    d = layer.d_model
    if layer.kind == LAYER_VIT:
        nqkv = (layer.n_q_heads + 2 * layer.n_kv_heads) * layer.head_dim
        no = layer.n_q_heads * layer.head_dim
        f = layer.d_ff
        qkn = [("qkn_q_g", 1, no), ("qkn_k_g", 1, layer.n_kv_heads * layer.head_dim)] if layer.qk_norm else []
        return [("ln1_g", 1, d), ("ln1_b", 1, d), ("w_qkv", d, nqkv), ("b_qkv", 1, nqkv),
                ("w_o", no, d), ("b_o", 1, d), ("ln2_g", 1, d), ("ln2_b", 1, d),
                ("w_1", d, f), ("b_1", 1, f), ("w_2", f, d), ("b_2", 1, d)] + qkn
    if layer.kind == LAYER_DECODER:
        nqkv = (layer.n_q_heads + 2 * layer.n_kv_heads) * layer.head_dim
        no = layer.n_q_heads * layer.head_dim
        f = layer.d_ff
        qkv = [("w_qkv", d, nqkv), ("b_qkv", 1, nqkv)] if layer.has_bias else [("w_qkv", d, nqkv)]
        qkn = [("qkn_q_g", 1, no), ("qkn_k_g", 1, layer.n_kv_heads * layer.head_dim)] if layer.qk_norm else []
        return [("rms1_g", 1, d)] + qkv + [("w_o", no, d), ("rms2_g", 1, d), ("w_gu", d, 2 * f), ("w_d", f, d)] + qkn
    if layer.kind == LAYER_PROJECTOR:
        d_in = d * max(1, layer.merge)
        if layer.d_ff:
            return [("w_p1", d_in, layer.d_ff), ("b_p1", 1, layer.d_ff), ("w_p2", layer.d_ff, layer.d_out),
                    ("b_p2", 1, layer.d_out)]
        return [("w_p", d_in, layer.d_out), ("b_p", 1, layer.d_out)]
    raise ValueError("unknown layer kind")


def draw_params(layers: Sequence[LayerDesc], seed: int) -> List[np.ndarray]:
    """All parameter tensors of a stage, flattened in interface order.

    Matrices ~ N(0, 0.02); biases and LayerNorm shifts ~ N(0, 0.02); norm gains
    ~ 1 + N(0, 0.02), so that every gradient path sees non-trivial values.
    Layer li uses generator seed `seed * 1000 + li`.  Values lie on the bf16 grid.
    """
    out: List[np.ndarray] = []
    for li, layer in enumerate(layers):
        rng = np.random.default_rng(seed * 1000 + li)
        for name, r, c in param_specs(layer):
            w = rng.standard_normal((r, c), dtype=np.float32) * np.float32(0.02)
            if name.endswith("_g"):
                w = w + np.float32(1.0)
            out.append(bf16_round(w))
    return out


# ---------------------------------------------------------------------------
# packed microbatch
# ---------------------------------------------------------------------------
@dataclass
class Pack:
    cu_seqlens: np.ndarray       # int32 [S+1]
    mask_kind: np.ndarray        # uint8 [S]

    @property
    def total_tokens(self) -> int:
        return int(self.cu_seqlens[-1])

    @property
    def n_segments(self) -> int:
        return len(self.mask_kind)

    @property
    def max_seqlen(self) -> int:
        if self.n_segments == 0:
            return 0
        return int(np.max(np.diff(self.cu_seqlens)))


def make_pack(lengths: Sequence[int], kind: int) -> Pack:
    cu = np.zeros(len(lengths) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(np.asarray(lengths, dtype=np.int64))
    return Pack(cu, np.full(len(lengths), kind, dtype=np.uint8))


@dataclass
class Batch:
    img: Optional[Pack] = None                 # segments = images (bidirectional)
    seq: Optional[Pack] = None                 # segments = samples (causal)
    img_to_seq_row: Optional[np.ndarray] = None  # int32 [T_img]
    samples: List[Tuple[int, int]] = field(default_factory=list)  # (n_images, n_text)


def batch_from_samples(samples: Sequence[Tuple[int, int]], img_tokens: int = IMG_TOKENS,
                       with_images: bool = True, pool: int = 1) -> Batch:
    """Pack samples of (n_images, n_text_tokens): image tokens first (image-major), then text.
    With a pooling connector every image (or audio clip) of `img_tokens` encoder tokens takes
    ceil(img_tokens / pool) rows of the LLM sequence."""
    llm_tokens = -(-img_tokens // max(pool, 1))
    seq_lens = [k * llm_tokens + t for k, t in samples]
    seq = make_pack(seq_lens, MASK_CAUSAL)
    n_img = sum(k for k, _ in samples)
    img = make_pack([img_tokens] * n_img, MASK_BIDIR)
    rows = []
    for s, (k, _t) in enumerate(samples):
        base = int(seq.cu_seqlens[s])
        rows.append(np.arange(base, base + k * llm_tokens, dtype=np.int32))
    i2s = np.concatenate(rows) if rows else np.zeros(0, dtype=np.int32)
    i2s = i2s.astype(np.int32)
    if not with_images:
        return Batch(None, seq, None, list(samples))
    return Batch(img, seq, i2s, list(samples))


def _fill_budget(budget: int, draw, img_tokens: int = IMG_TOKENS) -> List[Tuple[int, int]]:
    """Draw samples in order and clip each to what still fits, images kept whole,
    until the token budget is met exactly."""
    samples: List[Tuple[int, int]] = []
    rem = budget
    while rem > 0:
        k, t = draw()
        k = min(k, rem // img_tokens)
        t = min(t, rem - k * img_tokens)
        if k * img_tokens + t == 0:
            continue
        samples.append((k, t))
        rem -= k * img_tokens + t
    return samples


def _lognormal_len(rng, median: float, sigma: float, cap: int) -> int:
    v = rng.lognormal(mean=math.log(median), sigma=sigma)
    return int(min(max(int(round(v)), 1), cap))


def draw_samples_mix7b(seed: int, budget: int = 8192) -> List[Tuple[int, int]]:
    """Image count uniform in {0..4}; text lognormal(median 200, sigma 0.8), cap 2048."""
    rng = np.random.default_rng(seed)
    return _fill_budget(budget, lambda: (int(rng.integers(0, 5)),
                                         _lognormal_len(rng, 200.0, 0.8, 2048)))


def draw_samples_mix8b(seed: int, budget: int = 32768) -> List[Tuple[int, int]]:
    """Long-tailed mix: image count min(16, G-1), G ~ geometric(0.3);
    text lognormal(median 300, sigma 1.0), cap 4096."""
    rng = np.random.default_rng(seed)
    return _fill_budget(budget, lambda: (min(16, int(rng.geometric(0.3)) - 1),
                                         _lognormal_len(rng, 300.0, 1.0, 4096)))


def draw_images_vit(seed: int, n_samples: int = 16) -> List[int]:
    """Images per sample uniform in {1..4}."""
    rng = np.random.default_rng(seed)
    return [int(rng.integers(1, 5)) for _ in range(n_samples)]


def draw_tensor(seed: int, rows: int, cols: int, chunk_rows: int = 4096) -> np.ndarray:
    """N(0,1) rows on the bf16 grid (fp32 array); drawn in row chunks to bound memory."""
    rng = np.random.default_rng(seed)
    out = np.empty((rows, cols), dtype=np.float32)
    for r0 in range(0, rows, chunk_rows):
        r1 = min(rows, r0 + chunk_rows)
        out[r0:r1] = bf16_round(rng.standard_normal((r1 - r0, cols), dtype=np.float32))
    return out


# ---------------------------------------------------------------------------
# the named workloads
# ---------------------------------------------------------------------------
@dataclass
class Workload:
    name: str
    layers: List[LayerDesc]
    batch: Batch
    params: List[np.ndarray]
    x_img: Optional[np.ndarray]
    x_seq: Optional[np.ndarray]
    dy: np.ndarray


def _stage_io_shapes(layers: Sequence[LayerDesc], batch: Batch):
    kinds = [l.kind for l in layers]
    uses_img = kinds[0] in (LAYER_VIT, LAYER_PROJECTOR)
    uses_seq = LAYER_DECODER in kinds or LAYER_PROJECTOR in kinds
    last = layers[-1]
    if last.kind == LAYER_VIT:
        out_rows, out_cols = batch.img.total_tokens, last.d_model
    elif last.kind == LAYER_PROJECTOR:
        out_rows, out_cols = batch.seq.total_tokens, last.d_out
    else:
        out_rows, out_cols = batch.seq.total_tokens, last.d_model
    d_img = layers[0].d_model if uses_img else 0
    d_seq = 0
    for l in layers:
        if l.kind == LAYER_PROJECTOR:
            d_seq = l.d_out
            break
        if l.kind == LAYER_DECODER:
            d_seq = l.d_model
            break
    return uses_img, uses_seq, d_img, d_seq, out_rows, out_cols


def make_workload(name: str, layers: List[LayerDesc], batch: Batch, seed: int,
                  with_data: bool = True) -> Workload:
    uses_img, uses_seq, d_img, d_seq, out_rows, out_cols = _stage_io_shapes(layers, batch)
    params = draw_params(layers, seed) if with_data else []
    x_img = x_seq = None
    dy = None
    if with_data:
        if uses_img:
            x_img = draw_tensor(seed * 7919 + 1, batch.img.total_tokens, d_img)
        if uses_seq:
            x_seq = draw_tensor(seed * 7919 + 2, batch.seq.total_tokens, d_seq)
        dy = draw_tensor(seed * 7919 + 3, out_rows, out_cols)
    return Workload(name, layers, batch, params, x_img, x_seq, dy)


def tiny_stage_layers() -> List[LayerDesc]:
    return [vit_layer(192, 3, 64, 768), projector_layer(192, 256),
            decoder_layer(256, 4, 4, 64, 1024, 10000.0)]


def tiny_variant_layers() -> List[LayerDesc]:
    """The tiny stage with the variants of the models the paper evaluates: tanh-GELU encoder,
    two-layer MLP connector, grouped-query decoder with a QKV bias."""
    return [vit_layer(192, 3, 64, 768, act=ACT_GELU_TANH), projector_layer(192, 256, d_hidden=320),
            decoder_layer(256, 4, 2, 64, 1024, 10000.0, qkv_bias=1)]


def workload_tiny_variant(seed: int) -> Workload:
    rng = np.random.default_rng(seed)
    samples = [(1, int(rng.integers(32, 97))) for _ in range(2)]
    batch = batch_from_samples(samples, img_tokens=64)
    return make_workload("tiny_variant", tiny_variant_layers(), batch, seed)


def tiny_qknorm_layers() -> List[LayerDesc]:
    """The tiny stage with QK normalisation in the encoder layer and in a grouped-query decoder layer."""
    return [vit_layer(192, 3, 64, 768, qk_norm=1), projector_layer(192, 256),
            decoder_layer(256, 4, 2, 64, 1024, 10000.0, qk_norm=1)]


def workload_tiny_qknorm(seed: int) -> Workload:
    rng = np.random.default_rng(seed)
    samples = [(1, int(rng.integers(32, 97))) for _ in range(2)]
    batch = batch_from_samples(samples, img_tokens=64)
    return make_workload("tiny_qknorm", tiny_qknorm_layers(), batch, seed)


def tiny_pooled_layers() -> List[LayerDesc]:
    """Encoder layer, a connector that averages 3 consecutive encoder tokens before its linear map
    (the audio-language setting of the paper's evaluation), decoder layer."""
    return [vit_layer(192, 3, 64, 768), projector_layer(192, 256, pool=3),
            decoder_layer(256, 4, 4, 64, 1024, 10000.0)]


def workload_tiny_pooled(seed: int) -> Workload:
    """2 samples x (one clip of 50 encoder tokens -> 17 LLM rows, the last window holds 2) + text."""
    rng = np.random.default_rng(seed)
    samples = [(1, int(rng.integers(32, 97))) for _ in range(2)]
    batch = batch_from_samples(samples, img_tokens=50, pool=3)
    return make_workload("tiny_pooled", tiny_pooled_layers(), batch, seed)


def tiny_merged_layers() -> List[LayerDesc]:
    """Encoder layer, an MLP connector over rows that concatenate 4 consecutive encoder tokens
    (192 -> 768 wide), decoder layer."""
    return [vit_layer(192, 3, 64, 768), projector_layer(192, 256, d_hidden=256, merge=4),
            decoder_layer(256, 4, 4, 64, 1024, 10000.0)]


def workload_tiny_merged(seed: int) -> Workload:
    """2 samples x (one image of 64 encoder tokens -> 16 LLM rows) + text."""
    rng = np.random.default_rng(seed)
    samples = [(1, int(rng.integers(32, 97))) for _ in range(2)]
    batch = batch_from_samples(samples, img_tokens=64, pool=4)
    return make_workload("tiny_merged", tiny_merged_layers(), batch, seed)


def workload_tiny(seed: int) -> Workload:
    """2 samples x (64 image tokens + text uniform in 32..96); 1 ViT layer (d=192),
    projector 192->256, 1 decoder layer (d=256)."""
    rng = np.random.default_rng(seed)
    samples = [(1, int(rng.integers(32, 97))) for _ in range(2)]
    batch = batch_from_samples(samples, img_tokens=64)
    return make_workload("tiny", tiny_stage_layers(), batch, seed)


def vit_l_layer() -> LayerDesc:
    return vit_layer(1024, 16, 64, 4096)


def dec7b_layer() -> LayerDesc:
    return decoder_layer(4096, 32, 32, 128, 11008, 10000.0)


def dec8b_layer() -> LayerDesc:
    return decoder_layer(4096, 32, 8, 128, 14336, 500000.0)


def dec_qkvbias_7b_layer() -> LayerDesc:
    """Decoder layer shaped like the 7B LLM of the paper's evaluation (Table 4): d = 3584, 28 query
    heads over 4 KV heads of 128, SwiGLU 18944, QKV bias, RoPE base 1e6."""
    return decoder_layer(3584, 28, 4, 128, 18944, 1000000.0, eps=1e-6, qkv_bias=1)


def internvit_6b_layer() -> LayerDesc:
    """Encoder layer with the attention and MLP shape of the large InternViT of the evaluated
    InternVL model (Table 4): d = 3200, 25 heads of 128, MLP 12800, QK normalisation."""
    return vit_layer(3200, 25, 128, 12800, eps=1e-6, qk_norm=1)


INTERNVIT_TILE_TOKENS = 1025      # a 448 x 448 tile in 14 x 14 patches plus the class token


def workload_internvit_6b(seed: int, budget: int = 24576, with_data=True) -> Workload:
    """One such layer on a microbatch of dynamic-resolution images: every image is cut into 1..12
    tiles plus a thumbnail tile (each tile a bidirectional segment of 1025 tokens), images are
    drawn until the token budget is reached."""
    rng = np.random.default_rng(seed)
    tiles, total = [], 0
    while True:
        n = int(rng.integers(1, 13)) + 1
        if total + n * INTERNVIT_TILE_TOKENS > budget:
            n = (budget - total) // INTERNVIT_TILE_TOKENS
        if n <= 0:
            break
        tiles.append(n)
        total += n * INTERNVIT_TILE_TOKENS
    batch = Batch(make_pack([INTERNVIT_TILE_TOKENS] * sum(tiles), MASK_BIDIR), None, None, [])
    return make_workload("internvit_6b", [internvit_6b_layer()], batch, seed, with_data)


def workload_vit_l(seed: int, n_images: Optional[int] = None, with_data=True) -> Workload:
    n = n_images if n_images is not None else sum(draw_images_vit(seed))
    batch = Batch(make_pack([IMG_TOKENS] * n, MASK_BIDIR), None, None, [])
    return make_workload("vit_l", [vit_l_layer()], batch, seed, with_data)


def workload_dec7b(seed: int, budget: int = 8192, with_data=True) -> Workload:
    batch = batch_from_samples(draw_samples_mix7b(seed, budget), with_images=False)
    return make_workload("dec7b", [dec7b_layer()], batch, seed, with_data)


def workload_dec8b(seed: int, budget: int = 32768, with_data=True) -> Workload:
    batch = batch_from_samples(draw_samples_mix8b(seed, budget), with_images=False)
    return make_workload("dec8b", [dec8b_layer()], batch, seed, with_data)


def full_stage_layers(n_vit: int = 24, n_dec: int = 8) -> List[LayerDesc]:
    return ([vit_l_layer() for _ in range(n_vit)] + [projector_layer(1024, 4096)]
            + [dec8b_layer() for _ in range(n_dec)])


def workload_full_stage(seed: int, budget: int, mix: str, n_vit: int = 24, n_dec: int = 8,
                        with_data=True) -> Workload:
    samples = (draw_samples_mix7b if mix == "7b" else draw_samples_mix8b)(seed, budget)
    if sum(k for k, _ in samples) == 0:          # a stage slice needs at least one image
        k0, t0 = samples[0]
        if t0 > IMG_TOKENS:
            samples[0] = (1, t0 - IMG_TOKENS)
    batch = batch_from_samples(samples)
    return make_workload("full_stage", full_stage_layers(n_vit, n_dec), batch, seed, with_data)


def workload_dec_qkvbias_7b(seed: int, budget: int = 32768, with_data=True) -> Workload:
    batch = batch_from_samples(draw_samples_mix8b(seed, budget), with_images=False)
    return make_workload("dec_qkvbias_7b", [dec_qkvbias_7b_layer()], batch, seed, with_data)


def workload_variant_stage(seed: int, budget: int = 4096, with_data=True) -> Workload:
    """One tanh-GELU ViT-L layer, a two-layer MLP connector 1024 -> 3584 -> 3584 and one
    QKV-bias decoder layer of the 7B shape, on a `budget`-token microbatch of the narrow mix."""
    samples = draw_samples_mix7b(seed, budget)
    if sum(k for k, _ in samples) == 0:
        k0, t0 = samples[0]
        if t0 > IMG_TOKENS:
            samples[0] = (1, t0 - IMG_TOKENS)
    layers = [vit_layer(1024, 16, 64, 4096, eps=1e-6, act=ACT_GELU_TANH),
              projector_layer(1024, 3584, d_hidden=3584), dec_qkvbias_7b_layer()]
    return make_workload("variant_stage", layers, batch_from_samples(samples), seed, with_data)


def workload_audio_stage(seed: int, n_clips: int = 16, with_data=True) -> Workload:
    """Audio-language stand-in (Evaluation, audio modality): 4 encoder layers of width 1280 (20 heads
    of 64, GELU MLP 5120) over clips of 1500 encoder tokens, a connector that average-pools pairs of
    tokens and maps 1280 -> 3584, and 2 QKV-bias decoder layers of the 7B shape.  One clip plus
    lognormal(median 200, sigma 0.8) text tokens per sample."""
    rng = np.random.default_rng(seed)
    samples = [(1, int(min(max(int(round(rng.lognormal(np.log(200.0), 0.8))), 1), 2048))) for _ in range(n_clips)]
    layers = ([vit_layer(1280, 20, 64, 5120) for _ in range(4)] + [projector_layer(1280, 3584, pool=2)]
              + [dec_qkvbias_7b_layer() for _ in range(2)])
    return make_workload("audio_stage", layers, batch_from_samples(samples, img_tokens=1500, pool=2), seed, with_data)


def full_stage_sweep() -> List[Tuple[int, int, str]]:
    """The 16 (seed, budget, mix) microbatches: 4 budgets x 2 mixes x 2 seeds."""
    out = []
    seed = 400
    for budget in (4096, 8192, 16384, 32768):
        for mix in ("7b", "8b"):
            for _ in range(2):
                out.append((seed, budget, mix))
                seed += 1
    return out


def equal_partition_batch(total: int, n_segments: int) -> Batch:
    """Synthetic equal-length causal partition of `total` tokens (length-mix sensitivity)."""
    return Batch(None, make_pack([total // n_segments] * n_segments, MASK_CAUSAL), None, [])
