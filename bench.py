#!/usr/bin/env python3
"""Benchmark: packed tokens/s of one pipeline stage forward+backward (bf16) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

A step is one mllm_stage_fwd + mllm_stage_bwd over one synthetic packed microbatch whose
inputs, parameters and gradient buffers already live in HBM.  The default workload is the full
stage slice (24 ViT-L layers + connector + 8 8B-GQA decoder layers) on a 32768-token microbatch
drawn with the long-tailed length mix; other named workloads time one layer.

Prints ONE JSON line (see the keys below): throughput, the model-FLOP fraction of the bf16 MFMA
peak, a `roofline` object for the dominant kernel (per-launch durations from HIP events recorded
inside the timed region on the launch stream), a `cpu_baseline` object (the fp64 oracle timed on
the host cores on a bounded sample of the same workload) and a per-class time breakdown.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import workloads as W  # noqa: E402

MFMA_BF16_PEAK = 2.5e15   # dense, FLOP/s
HBM_PEAK = 8.0e12         # B/s


TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "hbm_traffic_full_stage_32k.md")
TRAFFIC_KERNELS = {"gemm_fwd": "gemm4_kernel<4, false, true, false>", "gemm_dx": "gemm4_kernel<4, false, false, false>",
                   "gemm_dw": "gemm4_kernel<4, true, true, true>"}


def gemm_source_digest():
    """First 16 hex digits of the SHA-256 of the GEMM kernel sources."""
    import hashlib
    h = hashlib.sha256()
    for f in ("gemm.hip", "gemm_common.h"):
        with open(os.path.join(ROOT, "paper_2603_25120_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def recorded_traffic(gemm_cls, workload):
    """L2 <-> fabric bytes per launch of the class's kernel, read from the committed summary of the two
    `rocprofv3 --pmc` runs (FETCH_SIZE, WRITE_SIZE) of this command.  The summary names the digest of the
    kernel sources it was taken with; when the sources have changed since, the figure is withheld (None)."""
    import re
    if workload != "full_stage_32k":
        return None, "counters were collected on the default workload only"
    try:
        text = open(TRAFFIC_PROFILE).read()
    except OSError:
        return None, "profiles/hbm_traffic_full_stage_32k.md is missing"
    m = re.search(r"GEMM kernel sources digest: ([0-9a-f]{16})", text)
    if not m:
        return None, "the summary names no kernel source digest"
    if m.group(1) != gemm_source_digest():
        return None, "stale: the summary was taken with kernel sources %s, these are %s" % (m.group(1), gemm_source_digest())
    row = re.search(r"\| `%s` \| \d+ \| (\d+) \| (\d+) \|" % re.escape(TRAFFIC_KERNELS[gemm_cls]), text)
    if not row:
        return None, "the summary has no row for %s" % TRAFFIC_KERNELS[gemm_cls]
    fetch_kib, write_kib = float(row.group(1)), float(row.group(2))
    return (fetch_kib * 2.0 + write_kib) * 1024.0, "profiles/hbm_traffic_full_stage_32k.md (kernel sources %s)" % m.group(1)


def stage_fwd_flops(layers, batch):
    from paper_2603_25120_amd.profiler import stage_fwd_flops as f
    return f(layers, batch)


def build_workload(name: str):
    if name == "full_stage_32k":
        wl = W.workload_full_stage(414, 32768, "8b", with_data=False)
        desc = "24 ViT-L layers + connector 1024->4096 + 8 8B-GQA decoder layers, 32768-token microbatch, long-tailed mix, seed 414"
    elif name == "full_stage_4k":
        wl = W.workload_full_stage(402, 4096, "8b", with_data=False)
        desc = "24 ViT-L + connector + 8 8B-GQA decoder layers, 4096-token microbatch, seed 402"
    elif name == "dec8b":
        wl = W.workload_dec8b(300, with_data=False)
        desc = "one 8B-GQA decoder layer, 32768-token microbatch, long-tailed mix, seed 300"
    elif name == "dec7b":
        wl = W.workload_dec7b(200, with_data=False)
        desc = "one 7B decoder layer, 8192-token microbatch, seed 200"
    elif name == "dec_qkvbias_7b":
        wl = W.workload_dec_qkvbias_7b(300, with_data=False)
        desc = "one QKV-bias decoder layer of the 7B shape (d 3584, 28/4 heads, SwiGLU 18944), 32768-token microbatch, long-tailed mix, seed 300"
    elif name == "variant_stage_16k":
        wl = W.workload_variant_stage(410, 16384, with_data=False)
        desc = "tanh-GELU ViT-L layer + MLP connector 1024->3584->3584 + QKV-bias 7B-shaped decoder layer, 16384-token microbatch, seed 410"
    elif name == "audio_stage":
        wl = W.workload_audio_stage(600, with_data=False)
        desc = "audio-language stand-in: 4 encoder layers (d 1280, 20 heads, MLP 5120) on 16 clips of 1500 tokens + pooling connector (pairs, 1280->3584) + 2 QKV-bias 7B-shaped decoder layers"
    elif name == "vit_l":
        wl = W.workload_vit_l(100, with_data=False)
        desc = "one ViT-L/14-336 layer, 16 samples x 1..4 images of 576 tokens, seed 100"
    elif name == "internvit_6b":
        wl = W.workload_internvit_6b(700, with_data=False)
        desc = "one QK-normalised encoder layer of the large InternViT shape (d 3200, 25 heads of 128, MLP 12800), 23 tiles of 1025 tokens, seed 700"
    else:
        raise SystemExit("unknown workload %r" % name)
    return wl, desc


def sample_clocks(step, torch, min_seconds=1.5):
    """Median shader clock (MHz) while `step` repeats for at least `min_seconds`, read from the
    driver's sysfs table (pp_dpm_sclk, the current level carries a '*'); None when the file is not
    there or not readable.  No other program is started for this."""
    import glob
    import re
    import threading
    paths = sorted(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk"))
    sclk, stop = [], threading.Event()

    def poll():
        while not stop.is_set():
            best = None
            for path in paths:
                try:
                    with open(path) as f:
                        for line in f:
                            m = re.search(r"(\d+)\s*Mhz\s*\*", line)
                            if m:
                                best = max(best or 0.0, float(m.group(1)))   # the busy GPU is the fastest one
                except OSError:
                    pass
            if best is not None:
                sclk.append(best)
            stop.wait(0.05)

    th = threading.Thread(target=poll, daemon=True)
    th.start()
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < min_seconds:
        step()
        torch.cuda.synchronize()
    stop.set()
    th.join(timeout=5)
    return {"sclk_mhz_under_load": float(np.median(sclk)) if sclk else None, "samples": len(sclk),
            "source": "pp_dpm_sclk"}


def run_gpu(args, wl):
    import torch
    from paper_2603_25120_amd import binding as B

    B.lib()  # raises if the HIP library is missing: there is no fallback
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    h = B.mllm_stage_create(wl.layers)
    infos = [B.mllm_stage_param_info(h, i) for i in range(B.mllm_stage_param_count(h))]
    gen = torch.Generator(device=dev)
    gen.manual_seed(1234)

    def randn(r, c, scale=1.0, shift=0.0):
        return (torch.randn(r, c, generator=gen, device=dev, dtype=torch.float32) * scale + shift).to(torch.bfloat16)

    params = [randn(r, c, 0.02, 1.0 if name.endswith("_g") else 0.0) for name, _, r, c in infos]
    dparams = [torch.zeros(r, c, dtype=torch.float32, device=dev) for _, _, r, c in infos]
    kinds = [l.kind for l in wl.layers]
    uses_img = kinds[0] in (W.LAYER_VIT, W.LAYER_PROJECTOR)
    uses_seq = W.LAYER_DECODER in kinds or W.LAYER_PROJECTOR in kinds
    x_img = randn(wl.batch.img.total_tokens, wl.layers[0].d_model) if uses_img else None
    d_seq = next((l.d_out if l.kind == W.LAYER_PROJECTOR else l.d_model) for l in wl.layers
                 if l.kind != W.LAYER_VIT) if uses_seq else 0
    x_seq = randn(wl.batch.seq.total_tokens, d_seq) if uses_seq else None
    last = wl.layers[-1]
    out_rows = wl.batch.img.total_tokens if last.kind == W.LAYER_VIT else wl.batch.seq.total_tokens
    out_cols = last.d_out if last.kind == W.LAYER_PROJECTOR else last.d_model
    dy = randn(out_rows, out_cols)
    y = torch.empty(out_rows, out_cols, dtype=torch.bfloat16, device=dev)
    dx_img = torch.empty_like(x_img) if uses_img else None
    dx_seq = torch.empty_like(x_seq) if uses_seq else None
    sb, wb = B.mllm_stage_sizes(h, wl.batch)
    saved = torch.empty(sb, dtype=torch.uint8, device=dev)
    ws = torch.empty(wb, dtype=torch.uint8, device=dev)

    def step(accumulate):
        B.mllm_stage_fwd(h, wl.batch, params, x_img, x_seq, y, saved, ws)
        B.mllm_stage_bwd(h, wl.batch, params, dy, saved, dx_img, dx_seq, dparams, accumulate, ws)

    for _ in range(args.warmup):
        step(0)
    torch.cuda.synchronize()
    # timed region: K steps; per-launch event pairs are recorded inside it on the launch stream
    n_launch_guess = 64 * len(wl.layers) * args.steps + 64
    B.mllm_profile_begin(n_launch_guess)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record()
    for i in range(args.steps):
        step(1 if i else 0)        # microbatches of one optimizer step accumulate their gradients
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    gpu_ms = e0.elapsed_time(e1)
    prof, dropped = B.mllm_profile_end()

    # shader clock and power under this load, sampled in a separate untimed pass
    clocks = sample_clocks(lambda: step(1), torch, min_seconds=1.5)

    # forward-only timing (for the forward : backward ratio)
    f0, f1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    f0.record()
    for _ in range(max(1, args.steps // 2)):
        B.mllm_stage_fwd(h, wl.batch, params, x_img, x_seq, y, saved, ws)
    f1.record()
    torch.cuda.synchronize()
    fwd_ms = f0.elapsed_time(f1) / max(1, args.steps // 2)
    finite = bool(torch.isfinite(y.float()).all().item())
    B.mllm_stage_destroy(h)
    props = torch.cuda.get_device_properties(0)
    return dict(gpu_ms=gpu_ms, wall_ms=wall_ms, prof=prof, dropped=dropped, fwd_ms=fwd_ms, finite=finite,
                saved_gib=sb / 2 ** 30, workspace_gib=wb / 2 ** 30, device=props.name,
                cus=props.multi_processor_count, clock_mhz=getattr(props, 'clock_rate', 0) / 1e3, clocks=clocks)


def cpu_baseline(sample_tokens: int = 6912):
    """Time the fp64 oracle on a bounded sample of the default workload: a microbatch drawn with the
    same long-tailed mix at a `sample_tokens` budget, through ONE ViT-L layer, the connector and ONE
    8B-GQA decoder layer, forward+backward.  The whole-stage rate follows by scaling to 24 and 8
    layers (the oracle's layers are identical in cost)."""
    from oracle import stage_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    samples = W.draw_samples_mix8b(414, sample_tokens)
    if sum(k for k, _ in samples) == 0:
        samples = [(1, sample_tokens - W.IMG_TOKENS)]
    batch = W.batch_from_samples(samples)
    vit = W.make_workload("vit", [W.vit_l_layer()], batch, 1)
    dec = W.make_workload("dec", [W.projector_layer(1024, 4096), W.dec8b_layer()], batch, 2)

    def timed(wl):
        t0 = time.perf_counter()
        y, caches = O.stage_fwd(wl.layers, wl.params, wl.batch, wl.x_img, wl.x_seq)
        O.stage_bwd(wl.layers, wl.params, wl.batch, caches, wl.dy.astype(np.float64))
        return time.perf_counter() - t0

    t_vit, t_dec = timed(vit), timed(dec)
    stage_s = 24 * t_vit + 8 * t_dec
    return {"value": batch.seq.total_tokens / stage_s, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": "%d-token microbatch (%d image tokens) of the same mix through 1 ViT-L layer (%.2f s) and "
                      "connector + 1 8B-GQA decoder layer (%.2f s), fp64 NumPy; scaled to 24 + 8 layers"
                      % (batch.seq.total_tokens, batch.img.total_tokens, t_vit, t_dec)}


def gemm_microbench(args):
    """One GEMM of the library on its own (the kernel the stage spends four fifths of its time in):
    `--gemm M N K A_LAYOUT B_LAYOUT OUT_FP32`, normally distributed bf16 operands, timed with HIP
    events over `--steps` back-to-back launches after `--warmup`.  Prints one JSON line."""
    import torch
    from paper_2603_25120_amd import binding as B
    B.lib()
    m, n, k, al, bl, f32 = args.gemm
    dev = torch.device("cuda:0")
    a = torch.randn((k, m) if al else (m, k), device=dev).to(torch.bfloat16)
    b = torch.randn((n, k) if bl else (k, n), device=dev).to(torch.bfloat16)
    c = torch.empty(m, n, device=dev, dtype=torch.float32 if f32 else torch.bfloat16)
    for _ in range(max(1, args.warmup)):
        B.mllm_op_gemm(a, b, c, m, n, k, al, bl, f32, 0)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.steps):
        B.mllm_op_gemm(a, b, c, m, n, k, al, bl, f32, 0)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    tf = 2.0 * m * n * k / (ms * 1e-3) / 1e12
    print(json.dumps({"gemm": {"m": m, "n": n, "k": k, "a_layout": al, "b_layout": bl, "out_fp32": f32},
                      "launches": args.steps, "ms_per_launch": ms, "TFLOP/s": tf, "mfma_peak_frac": tf / 2500.0}))


def sweep(args):
    """Stage time versus microbatch shape: the 16 seeded full-stage microbatches (4 token budgets x
    2 length mixes x 2 seeds) and, for one 8B-GQA decoder layer at 32768 tokens, equal-length
    partitions from 256 x 128 to 1 x 32768.  Prints a markdown table (not the one-line JSON)."""
    print("| workload | tokens | image tokens | samples | longest | sum L^2 / 1e6 | ms/step | tokens/s | % MFMA peak |")
    print("|---|---|---|---|---|---|---|---|---|")
    cases = []
    for seed, budget, mix in W.full_stage_sweep():
        wl = W.workload_full_stage(seed, budget, mix, with_data=False)
        cases.append(("full stage, mix %s, seed %d" % (mix, seed), wl))
    for nseg in (256, 64, 16, 4, 1):
        batch = W.equal_partition_batch(32768, nseg)
        cases.append(("8B-GQA layer, %d x %d" % (nseg, 32768 // nseg),
                      W.make_workload("eq", [W.dec8b_layer()], batch, 1, with_data=False)))
    for seed in (300, 301, 302, 303):
        cases.append(("8B-GQA layer, long-tailed mix, seed %d" % seed, W.workload_dec8b(seed, with_data=False)))
    for name, wl in cases:
        lin_f, attn_f = stage_fwd_flops(wl.layers, wl.batch)
        r = run_gpu(args, wl)
        ms = r["gpu_ms"] / args.steps
        seq = wl.batch.seq
        lens = np.diff(seq.cu_seqlens).astype(np.float64)
        print("| %s | %d | %d | %d | %d | %.1f | %.2f | %.0f | %.1f |" % (
            name, seq.total_tokens, wl.batch.img.total_tokens if wl.batch.img is not None else 0, seq.n_segments,
            seq.max_seqlen, float(np.sum(lens * lens)) / 1e6, ms, seq.total_tokens / (ms * 1e-3),
            100 * 3.0 * (lin_f + attn_f) / (ms * 1e-3) / MFMA_BF16_PEAK), flush=True)


def schedule_experiment(args):
    """Online microbatch scheduling on measured stage times (Online Microbatch Scheduler): a global
    batch of N items is cut into m buckets at random, by LPT and by the node-limited exact search;
    every bucket's encoder stage (24 ViT-L layers + connector) and LLM stage (8 8B-GQA layers) is
    then timed on the GPU.  Per-item durations come from three constants measured in the same run:
    encoder time per image, LLM time per token and LLM time per (sample length)^2."""
    from paper_2603_25120_amd import binding as B
    from paper_2603_25120_amd.profiler import StageRunner
    N, m = args.sched_items, args.sched_buckets
    rng = np.random.default_rng(2048)
    items = []
    while len(items) < N:
        k = min(16, int(rng.geometric(0.3)) - 1)
        t = int(min(max(int(round(rng.lognormal(np.log(300.0), 1.0))), 1), 4096))
        items.append((k, t))
    enc = StageRunner([W.vit_l_layer() for _ in range(24)] + [W.projector_layer(1024, 4096)])
    llm = StageRunner([W.dec8b_layer() for _ in range(8)])

    # duration model
    def enc_batch(samples):
        return W.batch_from_samples(samples)
    t_a = enc.time(enc_batch([(8, 1)]))
    t_b = enc.time(enc_batch([(8, 1)] * 4))
    c_img = (t_b - t_a) / 24.0                                   # ms per image
    t_1 = llm.time(W.equal_partition_batch(16384, 128))          # sum L^2 = 16384 * 128
    t_2 = llm.time(W.equal_partition_batch(16384, 4))            # sum L^2 = 16384 * 4096
    c_sq = (t_2 - t_1) / (16384.0 * (4096 - 128))
    c_tok = (t_1 - c_sq * 16384.0 * 128) / 16384.0
    e_dur = np.array([c_img * k for k, _ in items])
    l_dur = np.array([c_tok * (576 * k + t) + c_sq * (576 * k + t) ** 2 for k, t in items])
    print("duration model: encoder %.4f ms/image; LLM %.5f ms/token + %.3e ms/token^2" % (c_img, c_tok, c_sq))

    policies = []
    for seed in range(3):
        policies.append(("random, seed %d" % seed, np.random.default_rng(seed).integers(0, m, N)))
    policies.append(("round-robin in arrival order", np.arange(N) % m))
    t0 = time.perf_counter()
    lpt = B.mllm_schedule_lpt(e_dur, l_dur, m)
    t_lpt = time.perf_counter() - t0
    policies.append(("LPT", lpt))
    t0 = time.perf_counter()
    exact, cmax_exact, optimal = B.mllm_schedule(e_dur, l_dur, m, node_limit=args.sched_nodes)
    t_exact = time.perf_counter() - t0
    policies.append(("exact search, %d nodes%s" % (args.sched_nodes, "" if not optimal else " (proven optimal)"), exact))
    lb = max(e_dur.sum() / m, l_dur.sum() / m, max(e_dur.max(), l_dur.max()))
    print("\n| policy | predicted C_max ms | measured max E_j ms | measured max L_j ms | measured C_max ms | measured sum of stage times ms |")
    print("|---|---|---|---|---|---|")
    for name, assign in policies:
        E = [0.0] * m
        L = [0.0] * m
        pe = np.zeros(m)
        pl = np.zeros(m)
        for j in range(m):
            idx = [i for i in range(N) if assign[i] == j]
            pe[j], pl[j] = e_dur[idx].sum(), l_dur[idx].sum()
            samples = [items[i] for i in idx]
            if not samples:
                continue
            batch = W.batch_from_samples(samples)
            if batch.img.total_tokens > 0:
                E[j] = enc.time(batch)
            L[j] = llm.time(W.Batch(None, batch.seq, None, samples))
        print("| %s | %.1f | %.1f | %.1f | %.1f | %.1f |" % (name, max(pe.max(), pl.max()), max(E), max(L),
                                                          max(max(E), max(L)), sum(E) + sum(L)), flush=True)
    print("\nlower bound on C_max from the duration model: %.1f ms; scheduler time on the host: LPT %.3f ms, exact search %.1f ms"
          % (lb, t_lpt * 1e3, t_exact * 1e3))
    # scheduler latency and LPT's distance from the lower bound at a global batch of 2048 items
    big = []
    while len(big) < 2048:
        k = min(16, int(rng.geometric(0.3)) - 1)
        t = int(min(max(int(round(rng.lognormal(np.log(300.0), 1.0))), 1), 4096))
        big.append((k, t))
    e2 = np.array([c_img * k for k, _ in big])
    l2 = np.array([c_tok * (576 * k + t) + c_sq * (576 * k + t) ** 2 for k, t in big])
    for m2 in (16, 64):
        t0 = time.perf_counter()
        a2 = B.mllm_schedule_lpt(e2, l2, m2)
        dt = time.perf_counter() - t0
        Ej = np.bincount(a2, weights=e2, minlength=m2)
        Lj = np.bincount(a2, weights=l2, minlength=m2)
        c = max(Ej.max(), Lj.max())
        lb2 = max(e2.sum() / m2, l2.sum() / m2, max(e2.max(), l2.max()))
        t0 = time.perf_counter()
        _, c3, opt3 = B.mllm_schedule(e2, l2, m2, node_limit=args.sched_nodes)
        dt3 = time.perf_counter() - t0
        print("2048 items, %d buckets: LPT C_max %.1f ms, %.2f %% above the lower bound %.1f ms, %.2f ms on the host; "
              "exact search (%d nodes, %s) C_max %.1f ms in %.0f ms"
              % (m2, c, 100 * (c / lb2 - 1), lb2, dt * 1e3, args.sched_nodes, "optimal" if opt3 else "limit hit", c3, dt3 * 1e3))
    enc.close()
    llm.close()


def draw_items(rng, n):
    """Items of the long-tailed mix: (images, text tokens)."""
    items = []
    while len(items) < n:
        k = min(16, int(rng.geometric(0.3)) - 1)
        t = int(min(max(int(round(rng.lognormal(np.log(300.0), 1.0))), 1), 4096))
        items.append((k, t))
    return items


def plan_experiment(args):
    """Model Profiler + Data Profiler + Algorithm 1 on this GPU's measurements.

    1. Throughput profiling: the encoder stage (24 ViT-L layers + connector) over the number of
       images, the LLM stage (8 8B-GQA layers) over the length of one sample with attention and
       linear operations separated.
    2. Held-out check: stage times of the 16 seeded full-stage microbatches predicted from the
       curves (the per-item rule of the paper, and a variant that reads the linear curve at the
       packed length) against the measured times.
    3. Memory tables from the library's size queries at 2 and 4 layers; Algorithm 1 on a 24-layer
       encoder + 32-layer LLM for several cluster sizes (TP fixed at 1: the only degree one GPU can
       profile), with its search time."""
    from paper_2603_25120_amd import binding as B
    from paper_2603_25120_amd import profiler as MP
    enc_layers = [W.vit_l_layer() for _ in range(24)] + [W.projector_layer(1024, 4096)]
    llm_layers = [W.dec8b_layer() for _ in range(8)]
    enc, llm = MP.StageRunner(enc_layers), MP.StageRunner(llm_layers)
    b_grid = [1, 2, 4, 8, 16, 32, 56]
    s_grid = [128, 256, 512, 1024, 2048, 4096, 8192, 16384, 32768]
    bx, e_thr, e_ms = MP.profile_encoder(enc, b_grid, lambda b: W.batch_from_samples([(b, 1)]))
    sx, lin_thr, attn_thr, l_ms, l_attn_ms, l_attn_packed_ms = MP.profile_llm(llm, s_grid, W.equal_partition_batch)
    print("## Throughput profiling (forward + backward, model FLOPs)\n")
    print("| images | encoder stage ms | E_thr TFLOP/s |\n|---|---|---|")
    for b, ms, thr in zip(b_grid, e_ms, e_thr):
        print("| %d | %.2f | %.0f |" % (b, ms, thr / 1e12))
    print("\n| sample length | LLM stage ms, one sample | of it attention ms | L_lin_thr TFLOP/s | attention ms, 16384 tokens of such samples | L_attn_thr TFLOP/s |\n|---|---|---|---|---|---|")
    for sl, ms, ma, a, mp, c in zip(s_grid, l_ms, l_attn_ms, lin_thr, l_attn_packed_ms, attn_thr):
        print("| %d | %.2f | %.2f | %.0f | %.2f | %.0f |" % (sl, ms, ma, a / 1e12, mp, c / 1e12), flush=True)

    # held-out microbatches
    print("\n## Held-out check on the 16 seeded full-stage microbatches\n")
    print("| microbatch | tokens | items | E measured ms | E predicted ms | L measured ms | L per-item rule ms | L packed-length rule ms |")
    print("|---|---|---|---|---|---|---|---|")
    err_e, err_item, err_packed = [], [], []
    one_img = W.batch_from_samples([(1, 1)])
    e_lin1, e_attn1 = MP.stage_fwd_flops(enc_layers, one_img)
    e_flop_img = 3.0 * (e_lin1 + e_attn1)
    tok = W.equal_partition_batch(1, 1)
    l_lin_tok = 3.0 * MP.stage_fwd_flops(llm_layers, tok)[0]
    l_attn_sq = 3.0 * MP.stage_fwd_flops(llm_layers, tok)[1]            # per (sample length)^2
    for seed, budget, mix in W.full_stage_sweep():
        wl = W.workload_full_stage(seed, budget, mix, with_data=False)
        samples = wl.batch.samples
        b = np.array([k for k, _ in samples], dtype=np.float64)
        sl = np.array([W.IMG_TOKENS * k + t for k, t in samples], dtype=np.float64)
        e_dur, l_dur = B.mllm_item_durations(b, sl, e_flop_img * b, l_lin_tok * sl, l_attn_sq * sl * sl,
                                             (bx, e_thr), (sx, lin_thr), (sx, attn_thr))
        # the encoder sees all images of the microbatch at once: its effective batch size is their sum
        e_pred = 1e3 * e_flop_img * b.sum() / B.mllm_interp(bx, e_thr, [b.sum()])[0] if b.sum() else 0.0
        l_item = 1e3 * l_dur.sum()
        _, l_attn_only = B.mllm_item_durations(b, sl, 0 * b, 0 * sl, l_attn_sq * sl * sl, (bx, e_thr), (sx, lin_thr), (sx, attn_thr))
        l_packed = 1e3 * (l_lin_tok * sl.sum() / B.mllm_interp(sx, lin_thr, [sl.sum()])[0] + l_attn_only.sum())
        e_meas = enc.time(wl.batch) if wl.batch.img.total_tokens else 0.0
        l_meas = llm.time(W.Batch(None, wl.batch.seq, None, samples))
        if e_meas:
            err_e.append(abs(e_pred / e_meas - 1))
        err_item.append(abs(l_item / l_meas - 1))
        err_packed.append(abs(l_packed / l_meas - 1))
        print("| mix %s, seed %d | %d | %d | %.1f | %.1f | %.1f | %.1f | %.1f |" % (
            mix, seed, budget, len(samples), e_meas, e_pred, l_meas, l_item, l_packed), flush=True)
    print("\nrelative error of the prediction, mean / max: encoder %.1f %% / %.1f %%; LLM per-item rule %.1f %% / %.1f %%; "
          "LLM packed-length rule %.1f %% / %.1f %%" % (
              100 * np.mean(err_e), 100 * np.max(err_e), 100 * np.mean(err_item), 100 * np.max(err_item),
              100 * np.mean(err_packed), 100 * np.max(err_packed)))
    enc.close()
    llm.close()

    # memory tables and Algorithm 1
    mem_b = [1.0, 8.0, 64.0, 256.0]
    mem_s = [1024.0, 8192.0, 32768.0, 65536.0]
    e_ms_tab, e_act = MP.memory_tables(lambda n: [W.vit_l_layer() for _ in range(n)],
                                       lambda x: W.batch_from_samples([(int(x), 1)]), mem_b)
    l_ms_tab, l_act = MP.memory_tables(lambda n: [W.dec8b_layer() for _ in range(n)],
                                       lambda x: W.equal_partition_batch(int(x), 8), mem_s)
    rng = np.random.default_rng(7)
    items = draw_items(rng, 4096)                                          # the Data Profiler's sample
    ib = np.array([k for k, _ in items], dtype=np.float64)
    isl = np.array([W.IMG_TOKENS * k + t for k, t in items], dtype=np.float64)
    layer_scale_e, layer_scale_l = 1.0, 32.0 / 8.0                           # profiled 8 LLM layers, the model has 32

    def regrid(x, y, grid):          # one input grid per module: read the throughput curve on the memory grid too
        g = np.unique(np.concatenate([x, grid]))
        return g, B.mllm_interp(x, y, g)

    eg, e_thr_g = regrid(bx, e_thr, mem_b)
    lg, l_thr_all = regrid(sx, (l_lin_tok * sx + l_attn_sq * sx * sx) / (l_lin_tok * sx / lin_thr + l_attn_sq * sx * sx / attn_thr), mem_s)
    enc_prof = dict(tp=[1], x=eg, thr=[e_thr_g], layers_lo=2, layers_hi=4,
                    model_state=[e_ms_tab],
                    act_state=[[B.mllm_interp(mem_b, e_act[0], eg, True), B.mllm_interp(mem_b, e_act[1], eg, True)]],
                    n_layers=24, flop_per_item=float(np.mean(e_flop_img * ib)) * layer_scale_e)
    llm_prof = dict(tp=[1], x=lg, thr=[l_thr_all], layers_lo=2, layers_hi=4,
                    model_state=[l_ms_tab],
                    act_state=[[B.mllm_interp(mem_s, l_act[0], lg, True), B.mllm_interp(mem_s, l_act[1], lg, True)]],
                    n_layers=32, flop_per_item=float(np.mean(l_lin_tok * isl + l_attn_sq * isl * isl)) * layer_scale_l)
    print("\n## Algorithm 1 on the measured tables (TP = 1 only, 288 GB per GPU)\n")
    print("data profile: %.2f images and %.0f LLM tokens per item on average (4096 sampled items)\n" % (ib.mean(), isl.mean()))
    print("| GPUs | global batch | E_tp E_pp E_dp | L_tp L_pp L_dp | N_mb | estimated makespan s | encoder GB | LLM GB | search ms |")
    print("|---|---|---|---|---|---|---|---|---|")
    for n_gpus, gbs in ((8, 64), (8, 256), (64, 256), (64, 2048), (512, 2048), (1024, 2048)):
        t0 = time.perf_counter()
        theta, t = B.mllm_optimize_parallelism(enc_prof, llm_prof, n_gpus, 1, 288e9, gbs, float(ib.mean()), float(isl.mean()))
        dt = time.perf_counter() - t0
        if theta is None:
            print("| %d | %d | nothing fits | | | | | | %.1f |" % (n_gpus, gbs, dt * 1e3))
            continue
        _, em, lm, _ = B.mllm_evaluate_parallelism(enc_prof, llm_prof, theta, 288e9, gbs, float(ib.mean()), float(isl.mean()))
        print("| %d | %d | %d %d %d | %d %d %d | %d | %.3f | %.1f | %.1f | %.1f |" % (
            (n_gpus, gbs) + theta + (t, em / 1e9, lm / 1e9, dt * 1e3)))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="full_stage_32k")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--sweep", action="store_true", help="print stage time versus microbatch shape instead")
    ap.add_argument("--schedule", action="store_true", help="run the microbatch-scheduling experiment instead")
    ap.add_argument("--plan", action="store_true", help="run the model profiler, its held-out check and Algorithm 1 instead")
    ap.add_argument("--gemm", type=int, nargs=6, metavar=("M", "N", "K", "A_LAYOUT", "B_LAYOUT", "OUT_FP32"),
                    help="time one GEMM of the library on its own instead")
    ap.add_argument("--sched-items", type=int, default=64)
    ap.add_argument("--sched-buckets", type=int, default=8)
    ap.add_argument("--sched-nodes", type=int, default=2_000_000)
    args = ap.parse_args()
    if args.gpus != 1:
        raise SystemExit("bench.py: this build measures one GPU's stage; run with --gpus 1 "
                         "(no collectives or sharding are part of it)")
    if args.gemm:
        return gemm_microbench(args)
    if args.sweep:
        return sweep(args)
    if args.schedule:
        return schedule_experiment(args)
    if args.plan:
        return plan_experiment(args)
    wl, desc = build_workload(args.workload)
    lin_f, attn_f = stage_fwd_flops(wl.layers, wl.batch)
    step_flops = 3.0 * (lin_f + attn_f)
    tokens = wl.batch.seq.total_tokens if wl.batch.seq is not None else wl.batch.img.total_tokens
    r = run_gpu(args, wl)
    ms_per_step = r["gpu_ms"] / args.steps
    tok_s = tokens / (ms_per_step * 1e-3)
    prof = r["prof"]
    # dominant kernel = the 256x256-tile GEMM instantiation with the largest share of time
    gemm_cls = max(("gemm_fwd", "gemm_dx", "gemm_dw"), key=lambda c: prof[c][1])
    n, ms, work = prof[gemm_cls]
    achieved = work / (ms * 1e-3) if ms > 0 else 0.0
    gemm_all = ("gemm_fwd", "gemm_dx", "gemm_dw", "gemm_small", "gemm_rows192")
    all_gemm_ms = sum(prof[c][1] for c in gemm_all)
    all_gemm_work = sum(prof[c][2] for c in gemm_all)
    kernel_names = {"gemm_fwd": "gemm4_kernel<4, false, true, false> and gemm4_swiglu_kernel (Y = X.W, 256x256x64 tiles)",
                    "gemm_dx": "gemm4_kernel<4, false, false, false> and gemm4_swiglu_bwd_kernel (dX = dY.W^T, 256x256x64 tiles)",
                    "gemm_dw": "gemm4_kernel<4, true, true, true> (dW = X^T.dY, fp32, 256x256x64 tiles)"}
    # weight gradients contract over the tokens: a token count that is no multiple of 64 takes the ragged-K form
    ragged = any(pk is not None and pk.total_tokens % 64 for pk in (wl.batch.img, wl.batch.seq))
    if ragged:
        kernel_names["gemm_dw"] = "gemm4_ragged_k_kernel<true> (dW = X^T.dY, fp32, 256x256x64 tiles, token count no multiple of 64)"
    traffic, traffic_note = recorded_traffic(gemm_cls, args.workload)
    # the large-tile kernels stream, per XCD, the 8 A panels and 4 B panels of an 8 x 4 block of 256 x 256 tiles
    # through L2 once: 2 M N K (1 / 2048 + 1 / 1024) bytes fetched per launch (bf16 operands)
    traffic_model = (work / n) * (1.0 / 2048 + 1.0 / 1024) if n else None
    out = {
        "metric": "packed tokens/s per stage fwd+bwd (bf16) + % of MFMA bf16 peak",
        "value": tok_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": args.workload, "description": desc, "packed_tokens": int(tokens),
                   "image_tokens": int(wl.batch.img.total_tokens) if wl.batch.img is not None else 0,
                   "n_samples": int(wl.batch.seq.n_segments) if wl.batch.seq is not None else 0,
                   "longest_sample": int(wl.batch.seq.max_seqlen) if wl.batch.seq is not None else 0},
        "model_tflop_per_step": step_flops / 1e12,
        "model_tflops": step_flops / (ms_per_step * 1e-3) / 1e12,
        "mfma_peak_frac": step_flops / (ms_per_step * 1e-3) / MFMA_BF16_PEAK,
        # the same against the peak scaled to the shader clock measured under this load (2.4 GHz nominal)
        "mfma_peak_frac_at_measured_clock": (step_flops / (ms_per_step * 1e-3) / (MFMA_BF16_PEAK * r["clocks"]["sclk_mhz_under_load"] / 2400.0)
                                             if r["clocks"].get("sclk_mhz_under_load") else None),
        "attention_flop_share": attn_f / (lin_f + attn_f),
        "fwd_ms": r["fwd_ms"], "bwd_over_fwd": (ms_per_step - r["fwd_ms"]) / r["fwd_ms"],
        "host_wall_ms_per_step": r["wall_ms"] / args.steps,
        "roofline": {"bound": "mfma", "kernel": kernel_names[gemm_cls], "achieved": achieved / 1e12,
                     "peak": MFMA_BF16_PEAK / 1e12, "unit": "TFLOP/s", "frac": achieved / MFMA_BF16_PEAK,
                     "traffic": traffic, "traffic_unit": "bytes per launch (L2 <-> fabric), FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0 KiB from rocprofv3 --pmc",
                     "traffic_source": traffic_note, "traffic_model_fetch_bytes": traffic_model, "launches": n, "avg_launch_ms": ms / n if n else None,
                     "all_gemm_tflops": all_gemm_work / (all_gemm_ms * 1e-3) / 1e12 if all_gemm_ms else None},
        "breakdown_ms_per_step": {c: prof[c][1] / args.steps for c in prof},
        "breakdown_rate": {
            **{c: {"TFLOP/s": prof[c][2] / (prof[c][1] * 1e-3) / 1e12} for c in prof
               if c != "elementwise" and prof[c][1] > 0},
            **({"elementwise": {"GB/s": prof["elementwise"][2] / (prof["elementwise"][1] * 1e-3) / 1e9,
                                "hbm_frac": prof["elementwise"][2] / (prof["elementwise"][1] * 1e-3) / HBM_PEAK}}
               if prof["elementwise"][1] > 0 else {})},
        "profile_records_dropped": r["dropped"], "outputs_finite": r["finite"],
        "saved_GiB": r["saved_gib"], "workspace_GiB": r["workspace_gib"],
        "device": r["device"], "compute_units": r["cus"], "clock_mhz": r["clock_mhz"], "clocks": r["clocks"],
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline()
        out["cpu_baseline"]["gpu_over_cpu"] = tok_s / out["cpu_baseline"]["value"]
    print(json.dumps(out))


if __name__ == "__main__":
    main()
