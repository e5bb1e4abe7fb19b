"""Whole-stage parity: mllm_stage_fwd / mllm_stage_bwd through the C ABI against the fp64 oracle on
the same seeded inputs.  Tolerances are the stated ones: normalised max error <= 2e-2 on outputs and
<= 3e-2 on every gradient; packed-sequence indexing is exact (packed == per-sample bit for bit on
the GPU, causality and segment isolation bit for bit)."""
import numpy as np
import pytest

import workloads as W
from oracle import stage_oracle as O

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from tests.gpu_util import (GpuStage, TOL_GRAD, TOL_OUT, compare, dev_bf16, empty_bf16, host_f64, nmax_err,  # noqa: E402
                            oracle_run, scratch)



@pytest.fixture(scope="module")
def B():
    from paper_2603_25120_amd import binding
    binding.lib()
    return binding


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_tiny_stage_matches_oracle(B, seed):
    wl = W.workload_tiny(seed)
    st = GpuStage(B, wl.layers)
    try:
        compare(st, wl, st.run(wl), oracle_run(wl))
    finally:
        st.close()


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_tiny_variant_stage_matches_oracle(B, seed):
    """tanh-GELU encoder, two-layer MLP connector, grouped-query decoder with a QKV bias."""
    wl = W.workload_tiny_variant(seed)
    st = GpuStage(B, wl.layers)
    try:
        compare(st, wl, st.run(wl), oracle_run(wl))
    finally:
        st.close()


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_tiny_pooled_stage_matches_oracle(B, seed):
    """Connector that averages 3 consecutive encoder tokens (ragged last window) before its map."""
    wl = W.workload_tiny_pooled(seed)
    st = GpuStage(B, wl.layers)
    try:
        compare(st, wl, st.run(wl), oracle_run(wl))
    finally:
        st.close()


@pytest.mark.parametrize("seed", [0, 1])
def test_tiny_merged_stage_matches_oracle(B, seed):
    """MLP connector over rows that concatenate 4 consecutive encoder tokens."""
    wl = W.workload_tiny_merged(seed)
    st = GpuStage(B, wl.layers)
    try:
        compare(st, wl, st.run(wl), oracle_run(wl))
    finally:
        st.close()


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_tiny_qknorm_stage_matches_oracle(B, seed):
    """RMS-normalised q and k rows in the encoder layer and in a grouped-query decoder layer."""
    wl = W.workload_tiny_qknorm(seed)
    st = GpuStage(B, wl.layers)
    try:
        compare(st, wl, st.run(wl), oracle_run(wl))
    finally:
        st.close()


@pytest.mark.parametrize("case", ["vit_wide", "dec_gqa_hd128", "dec_bias_two_layers"])
def test_qk_norm_layer_shapes(B, case):
    """QK normalisation at widths that take each form of the norm kernels (rows of 128 to 2048
    values inside a wider QKV matrix), ragged segments with an empty and a one-token one."""
    if case == "vit_wide":
        layers = [W.vit_layer(1280, 20, 64, 512, qk_norm=1)]
        batch = W.Batch(W.make_pack([130, 0, 1, 77], W.MASK_BIDIR), None, None, [])
    elif case == "dec_gqa_hd128":
        layers = [W.decoder_layer(2048, 16, 2, 128, 512, 500000.0, qk_norm=1)]
        batch = W.Batch(None, W.make_pack([150, 1, 0, 93], W.MASK_CAUSAL), None, [])
    else:
        first = W.decoder_layer(512, 8, 1, 64, 256, 10000.0, qkv_bias=1, qk_norm=1)
        layers = [first, W.decoder_layer(512, 8, 8, 64, 320, 10000.0, qk_norm=1)]
        batch = W.Batch(None, W.make_pack([260, 3], W.MASK_CAUSAL), None, [])
    _layer_case(B, layers, batch, 41)


def test_qk_norm_gradients_accumulate(B):
    wl = W.workload_tiny_qknorm(3)
    st = GpuStage(B, wl.layers)
    try:
        a = st.run(wl)
        acc = [torch.zeros_like(g) for g in a[3]]
        st.run(wl, accumulate=1, dparams=acc)
        st.run(wl, accumulate=1, dparams=acc)
        for g2, g1 in zip(acc, a[3]):
            assert nmax_err(host_f64(g2), 2 * host_f64(g1)) < 1e-5
    finally:
        st.close()


def test_pooled_mlp_connector_ragged_segments(B):
    """Pooling by 4 over encoder segments of 1, 4, 9 and 130 tokens, MLP connector, image-only and
    text-only samples."""
    layers = [W.vit_layer(128, 2, 64, 256), W.projector_layer(128, 192, d_hidden=128, pool=4),
              W.decoder_layer(192, 3, 1, 64, 320, 10000.0, qkv_bias=1)]
    img_lens = [1, 4, 9, 130]
    con = [-(-n // 4) for n in img_lens]                      # connector rows per encoder segment
    seq_lens = [con[0] + 5, 40, con[1] + con[2], con[3] + 3]  # sample 1 is text only, sample 2 image only
    seq = W.make_pack(seq_lens, W.MASK_CAUSAL)
    cu = seq.cu_seqlens
    rows = np.concatenate([np.arange(cu[0], cu[0] + con[0]), np.arange(cu[2], cu[2] + con[1] + con[2]),
                           np.arange(cu[3], cu[3] + con[3])]).astype(np.int32)
    batch = W.Batch(W.make_pack(img_lens, W.MASK_BIDIR), seq, rows, [])
    _layer_case(B, layers, batch, 31)


def test_tiny_stage_deterministic_and_accumulates(B):
    wl = W.workload_tiny(4)
    st = GpuStage(B, wl.layers)
    try:
        a = st.run(wl)
        b = st.run(wl)
        assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1]) and torch.equal(a[2], b[2])
        for ga, gb in zip(a[3], b[3]):
            assert torch.equal(ga, gb)
        # accumulate: two passes into the same fp32 buffers give twice the gradient
        acc = [torch.zeros_like(g) for g in a[3]]
        st.run(wl, accumulate=1, dparams=acc)
        st.run(wl, accumulate=1, dparams=acc)
        for g2, g1 in zip(acc, a[3]):
            assert nmax_err(host_f64(g2), 2 * host_f64(g1)) < 1e-5
    finally:
        st.close()


def test_packed_equals_per_sample_on_gpu(B):
    """Rows of a sample do not depend on what else is packed with it: bitwise on the GPU."""
    wl = W.workload_tiny(5)
    st = GpuStage(B, wl.layers)
    try:
        y, dx_img, dx_seq, _ = st.run(wl)
        cu = wl.batch.seq.cu_seqlens
        for s, (k, t) in enumerate(wl.batch.samples):
            one = W.Workload("one", wl.layers, W.batch_from_samples([(k, t)], img_tokens=64), wl.params,
                             wl.x_img[64 * s:64 * (s + 1)], wl.x_seq[cu[s]:cu[s + 1]], wl.dy[cu[s]:cu[s + 1]])
            y1, dxi1, dxs1, _ = st.run(one)
            assert torch.equal(y1, y[cu[s]:cu[s + 1]])
            assert torch.equal(dxi1, dx_img[64 * s:64 * (s + 1)])
            assert torch.equal(dxs1, dx_seq[cu[s]:cu[s + 1]])
    finally:
        st.close()


def test_causality_and_isolation_on_gpu(B):
    wl = W.workload_tiny(6)
    st = GpuStage(B, wl.layers)
    try:
        y, _, _, _ = st.run(wl)
        cu = wl.batch.seq.cu_seqlens
        t = int(cu[1]) - 1
        xs = wl.x_seq.copy()
        xs[t] = W.bf16_round(xs[t] + np.linspace(-1, 1, xs.shape[1], dtype=np.float32))
        wl2 = W.Workload("p", wl.layers, wl.batch, wl.params, wl.x_img, xs, wl.dy)
        y2, _, _, _ = st.run(wl2)
        assert torch.equal(y2[:t], y[:t]) and torch.equal(y2[cu[1]:], y[cu[1]:])
        assert not torch.equal(y2[t], y[t])
    finally:
        st.close()


def _layer_case(B, layers, batch, seed):
    wl = W.make_workload("case", layers, batch, seed)
    st = GpuStage(B, layers)
    try:
        return compare(st, wl, st.run(wl), oracle_run(wl))
    finally:
        st.close()


def test_vit_layer_ragged_images(B):
    # ViT-L-shaped layer at reduced token count: 576-token images plus odd-sized segments
    batch = W.Batch(W.make_pack([576, 576, 100, 1, 0, 333], W.MASK_BIDIR), None, None, [])
    _layer_case(B, [W.vit_l_layer()], batch, 20)


def test_decoder_layer_gqa_long_tail(B):
    # 8B-GQA head geometry (4 query heads per kv head, head_dim 128) at reduced widths
    layer = W.decoder_layer(1024, 8, 2, 128, 1792, 500000.0)
    batch = W.Batch(None, W.make_pack([1200, 1, 77, 0, 640, 129], W.MASK_CAUSAL), None, [])
    _layer_case(B, [layer], batch, 21)


def test_decoder_layer_mha(B):
    layer = W.decoder_layer(512, 4, 4, 128, 1408, 10000.0)
    batch = W.batch_from_samples(W.draw_samples_mix7b(22, budget=1500), with_images=False)
    _layer_case(B, [layer], batch, 22)


def test_multi_layer_stage(B):
    # 2 ViT layers + projector + 2 decoder layers at small widths, mixed samples incl. a text-only one
    layers = [W.vit_layer(256, 4, 64, 512), W.vit_layer(256, 4, 64, 512), W.projector_layer(256, 384),
              W.decoder_layer(384, 6, 2, 64, 640, 500000.0), W.decoder_layer(384, 6, 2, 64, 640, 500000.0)]
    batch = W.batch_from_samples([(2, 37), (0, 150), (1, 1)], img_tokens=96)
    _layer_case(B, layers, batch, 23)


def test_deep_narrow_stage(B):
    """Error growth with depth: 12 encoder layers + connector + 8 decoder layers at small widths,
    every output and every gradient still within the stated tolerances."""
    layers = ([W.vit_layer(256, 4, 64, 512) for _ in range(12)] + [W.projector_layer(256, 384)]
              + [W.decoder_layer(384, 6, 2, 64, 640, 500000.0) for _ in range(8)])
    batch = W.batch_from_samples([(2, 61), (0, 200), (1, 7), (3, 130)], img_tokens=80)
    _layer_case(B, layers, batch, 29)


def test_stage_without_dx_and_vit_only(B):
    wl = W.make_workload("v", [W.vit_layer(192, 3, 64, 768)], W.Batch(W.make_pack([64, 30], 0), None, None, []), 24)
    st = GpuStage(B, wl.layers)
    try:
        got = st.run(wl, want_dx=False)
        ref = oracle_run(wl)
        assert nmax_err(host_f64(got[0]), ref[0]) <= TOL_OUT
        for g, r in zip(got[3], ref[3]):
            assert nmax_err(host_f64(g), r) <= TOL_GRAD
    finally:
        st.close()


def test_error_statuses_touch_nothing(B):
    wl = W.workload_tiny(7)
    st = GpuStage(B, wl.layers)
    try:
        sb, wb = B.mllm_stage_sizes(st.h, wl.batch)
        params = [dev_bf16(p) for p in wl.params]
        y = torch.full(wl.dy.shape, 7.0, dtype=torch.bfloat16, device="cuda")
        with pytest.raises(B.MllmError) as e:
            B.mllm_stage_fwd(st.h, wl.batch, params, dev_bf16(wl.x_img), dev_bf16(wl.x_seq), y, scratch(sb), scratch(wb // 2))
        assert e.value.status == 7
        torch.cuda.synchronize()
        assert float((y.float() - 7.0).abs().max()) == 0.0
    finally:
        st.close()


def test_empty_microbatch(B):
    """No tokens at all: every call succeeds, launches nothing that reads data, and an overwrite
    backward leaves zero parameter gradients."""
    layers = [W.vit_layer(192, 3, 64, 768), W.projector_layer(192, 256), W.decoder_layer(256, 4, 4, 64, 1024, 10000.0)]
    batch = W.Batch(W.make_pack([], W.MASK_BIDIR), W.make_pack([0, 0], W.MASK_CAUSAL), np.zeros(0, np.int32), [])
    h = B.mllm_stage_create(layers)
    try:
        infos = [B.mllm_stage_param_info(h, i) for i in range(B.mllm_stage_param_count(h))]
        params = [dev_bf16(p) for p in W.draw_params(layers, 3)]
        dparams = [torch.full((r, c), 5.0, dtype=torch.float32, device="cuda") for _, _, r, c in infos]
        sb, wb = B.mllm_stage_sizes(h, batch)
        saved, ws = scratch(sb), scratch(wb)
        one = empty_bf16(1, 256)
        B.mllm_stage_fwd(h, batch, params, one, one, one, saved, ws)
        B.mllm_stage_bwd(h, batch, params, one, saved, one, one, dparams, 0, ws)
        torch.cuda.synchronize()
        for g in dparams:
            assert float(g.abs().max()) == 0.0
    finally:
        B.mllm_stage_destroy(h)


def test_decoder_layer_rerun_is_bitwise_identical(B):
    layer = W.decoder_layer(1024, 8, 2, 128, 1792, 500000.0)
    batch = W.batch_from_samples(W.draw_samples_mix8b(31, budget=3000), with_images=False)
    wl = W.make_workload("det", [layer], batch, 31)
    st = GpuStage(B, [layer])
    try:
        a, b = st.run(wl), st.run(wl)
        assert torch.equal(a[0], b[0]) and torch.equal(a[2], b[2])
        for ga, gb in zip(a[3], b[3]):
            assert torch.equal(ga, gb)
    finally:
        st.close()
