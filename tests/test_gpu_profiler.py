"""Throughput profiling on the GPU (Model Profiler, "Throughput Profiling"): the encoder measured over
its effective batch size, the LLM over the sequence length with attention and the linear operations
separately, read off between grid points by linear interpolation, then checked on microbatches that
were not on the grid.

Small stages keep this short: 2 ViT-L layers + connector, and 1 8B-GQA decoder layer.  Stated
bounds: the curves saturate (throughput at the largest grid point at least twice that at the
smallest, no grid point more than 15 % below its predecessor); stage times of held-out microbatches
are predicted within 25 % for the encoder and 12 % for the LLM (the full table of the benchmark
stages, with its finer grid, stays within 10.2 % and 3.7 %).
"""
import numpy as np
import pytest

import workloads as W

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2603_25120_amd import binding
    binding.lib()
    return binding


def _saturating(thr):
    assert thr[-1] >= 2.0 * thr[0], thr
    assert all(b >= 0.85 * a for a, b in zip(thr, thr[1:])), thr


def test_encoder_throughput_curve_and_held_out_batches(B):
    from paper_2603_25120_amd import profiler as MP
    layers = [W.vit_l_layer(), W.vit_l_layer(), W.projector_layer(1024, 4096)]
    enc = MP.StageRunner(layers)
    make = lambda b: W.batch_from_samples([(b, 1)])
    try:
        bx, thr, ms = MP.profile_encoder(enc, [1, 2, 4, 8, 16, 32], make)
        _saturating(thr)
        assert np.all(np.diff(ms) > 0)                       # more images take longer
        errs = []
        for samples in ([(3, 5), (2, 40), (1, 7)], [(12, 100)], [(5, 1)] * 5):    # 6, 12 and 25 images
            batch = W.batch_from_samples(samples)
            b = float(sum(k for k, _ in samples))
            lin, attn = MP.stage_fwd_flops(layers, batch)
            pred = 1e3 * 3.0 * (lin + attn) / B.mllm_interp(bx, thr, [b])[0]
            errs.append(abs(pred / enc.time(batch) - 1.0))
    finally:
        enc.close()
    print("E_thr TFLOP/s %s; held-out errors %s" % (np.round(thr / 1e12, 1), np.round(errs, 3)), flush=True)
    assert max(errs) <= 0.25, errs


def test_llm_throughput_curves_and_held_out_microbatches(B):
    from paper_2603_25120_amd import profiler as MP
    layers = [W.dec8b_layer()]
    llm = MP.StageRunner(layers)
    try:
        sx, lin_thr, attn_thr, ms, ms_attn, _ = MP.profile_llm(llm, [256, 1024, 4096, 16384], W.equal_partition_batch,
                                                              packed_tokens=16384)
        _saturating(lin_thr)
        _saturating(attn_thr)
        assert np.all(ms_attn < ms) and np.all(ms_attn > 0)   # attention is a part of the step, measured on its own
        tok = W.equal_partition_batch(1, 1)
        lin_tok, attn_sq = (3.0 * v for v in MP.stage_fwd_flops(layers, tok))
        errs = []
        for seed, budget in ((301, 8192), (302, 16384), (201, 8192)):
            samples = (W.draw_samples_mix7b if seed < 300 else W.draw_samples_mix8b)(seed, budget)
            batch = W.batch_from_samples(samples, with_images=False)
            sl = np.array([W.IMG_TOKENS * k + t for k, t in samples], dtype=np.float64)
            zero = np.zeros_like(sl)
            _, attn_dur = B.mllm_item_durations(zero, sl, zero, zero, attn_sq * sl * sl, (sx, lin_thr), (sx, lin_thr),
                                                (sx, attn_thr))
            pred = 1e3 * (lin_tok * sl.sum() / B.mllm_interp(sx, lin_thr, [sl.sum()])[0] + attn_dur.sum())
            errs.append(abs(pred / llm.time(batch) - 1.0))
    finally:
        llm.close()
    print("L_lin_thr %s, L_attn_thr %s TFLOP/s; held-out errors %s"
          % (np.round(lin_thr / 1e12, 1), np.round(attn_thr / 1e12, 1), np.round(errs, 3)), flush=True)
    assert max(errs) <= 0.12, errs
