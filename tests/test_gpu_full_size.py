"""Parity at the full benchmark sizes, in the launch configuration bench.py times.

* ViT-L layer and 7B decoder layer: the whole layer, forward and backward, every output and every
  gradient against the fp64 oracle (the oracle finishes these in seconds on the host cores).
* 8B-GQA decoder layer at 32768 packed tokens: the whole layer too, every output and every gradient.
* A 7-layer full-width stack on the benchmark's 32768-token microbatch: the oracle runs one sample
  ALONE through all layers.  Rows of a sample do not depend on what it is packed with (per-instance
  attention, row-wise linear maps: Model Profiler, "Throughput Profiling").  The benchmark's own
  33-layer stack is covered layer by layer in test_gpu_stack_in_situ.py.
* The kernels at the full shapes on sampled outputs: GEMM entries (all three layouts of the 8B
  layer, including the weight-gradient contraction over 32768 tokens) against fp64 dot products,
  attention rows of sampled (segment, head) pairs against the oracle run on that pair only.

Tolerances as everywhere: normalised max error 2e-2 on outputs, 3e-2 on gradients; fp32 GEMM
outputs 2e-3.
"""
import numpy as np
import pytest

import workloads as W
from oracle import stage_oracle as O

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from tests.gpu_util import GpuStage, compare, dev_bf16, host_f64, nmax_err, oracle_run, scratch  # noqa: E402


@pytest.fixture(scope="module")
def B():
    from paper_2603_25120_amd import binding
    binding.lib()
    return binding


def test_vit_l_layer_full(B):
    wl = W.workload_vit_l(100)                       # 16 samples x 1..4 images of 576 tokens
    st = GpuStage(B, wl.layers)
    try:
        compare(st, wl, st.run(wl), oracle_run(wl))
    finally:
        st.close()


def test_weight_gradient_split_with_empty_last_parts(B):
    """Weight gradient of a 1280 -> 1280 connector over 6720 image tokens (105 k-tiles of 64): the
    1280 x 1280 product is cut along the tokens into 13 parts of 9 k-tiles, so the last part starts
    past the end of the contraction and must contribute zeros."""
    layers = [W.projector_layer(1280, 1280)]
    batch = W.batch_from_samples([(1, 3)] * 12, img_tokens=560)
    assert batch.img.total_tokens == 105 * 64
    wl = W.make_workload("split_tail", layers, batch, 907)
    st = GpuStage(B, layers)
    try:
        compare(st, wl, st.run(wl), oracle_run(wl))
    finally:
        st.close()


def test_weight_gradient_split_over_ragged_token_count(B):
    """ViT-L layer on 7 images of 577 tokens: 4039 tokens are 63 k-tiles of 64 and one of 7 rows, and
    the layer's weight gradients are cut along the tokens into parts, the last of which holds the
    partial k-tile."""
    layers = [W.vit_l_layer()]
    batch = W.Batch(W.make_pack([577] * 7, W.MASK_BIDIR), None, None, [])
    wl = W.make_workload("vit_ragged_tokens", layers, batch, 911)
    st = GpuStage(B, layers)
    try:
        compare(st, wl, st.run(wl), oracle_run(wl))
    finally:
        st.close()


def test_decoder_layer_with_only_the_gradient_epilogue_fused(B):
    """SwiGLU width 3264 = 51 x 64 on 4096 tokens: the up-projection cannot take the fused forward
    form (f is no multiple of 128) and runs GEMM + activation kernel, the down-projection's input
    gradient has 208 tiles and takes the fused form, with a last tile column of 192 valid columns."""
    layers = [W.decoder_layer(512, 8, 2, 64, 3264, 10000.0)]
    batch = W.Batch(None, W.make_pack([1500, 700, 1, 1895], W.MASK_CAUSAL), None, [])
    wl = W.make_workload("dec_f3264", layers, batch, 913)
    st = GpuStage(B, layers)
    try:
        compare(st, wl, st.run(wl), oracle_run(wl))
    finally:
        st.close()


def test_decoder_layer_rotary_epilogue_heads_of_64_with_qkv_bias(B):
    """A narrow decoder layer (d = 512, 8 / 2 heads of 64, QKV bias) on 17200 tokens: its QKV projection has
    204 tiles of 256 x 256 and takes the form with the rotary positions in the epilogue (two heads per
    wavefront, bias added before the rotation); every output and gradient."""
    layers = [W.decoder_layer(512, 8, 2, 64, 1024, 10000.0, qkv_bias=1)]
    batch = W.Batch(None, W.make_pack([3000, 5000, 1, 9199], W.MASK_CAUSAL), None, [])
    assert batch.seq.total_tokens == 17200
    wl = W.make_workload("dec_rope64", layers, batch, 917)
    st = GpuStage(B, layers)
    try:
        compare(st, wl, st.run(wl), oracle_run(wl))
    finally:
        st.close()


def test_dec7b_layer_full(B):
    wl = W.workload_dec7b(200)                       # 8192 packed tokens, d = 4096, MHA, SwiGLU 11008
    st = GpuStage(B, wl.layers)
    try:
        compare(st, wl, st.run(wl), oracle_run(wl))
    finally:
        st.close()


def test_variant_stage_full_width(B):
    """tanh-GELU ViT-L layer + MLP connector 1024 -> 3584 -> 3584 + QKV-bias decoder layer of the 7B
    shape (d = 3584, 28/4 heads, SwiGLU 18944) on a 2048-token microbatch: every output and gradient."""
    wl = W.workload_variant_stage(500, budget=2048)
    st = GpuStage(B, wl.layers)
    try:
        compare(st, wl, st.run(wl), oracle_run(wl))
    finally:
        st.close()


def test_internvit_6b_layer_full_width(B):
    """QK-normalised encoder layer at the large InternViT width (d = 3200, 25 heads of 128, MLP
    12800) on one whole tile of 1025 tokens and a ragged one of 300: every output and gradient."""
    layers = [W.internvit_6b_layer()]
    batch = W.Batch(W.make_pack([W.INTERNVIT_TILE_TOKENS, 300], W.MASK_BIDIR), None, None, [])
    wl = W.make_workload("internvit_6b", layers, batch, 701)
    st = GpuStage(B, layers)
    try:
        compare(st, wl, st.run(wl), oracle_run(wl))
    finally:
        st.close()


def test_dec8b_layer_full(B):
    """The 8B-GQA decoder layer on its whole 32768-token microbatch (seed 300, 32 / 8 heads, SwiGLU
    14336): y, dx and EVERY parameter gradient (each a contraction over all 32768 tokens) against the
    fp64 oracle run on the same microbatch (about a minute on 16 host cores)."""
    wl = W.workload_dec8b(300)
    st = GpuStage(B, wl.layers)
    try:
        got = st.run(wl)
    finally:
        st.close()
    errs = compare(st, wl, got, oracle_run(wl))
    print("8B-GQA layer, 32768 tokens: %s" % ", ".join("%s %.2e" % kv for kv in errs.items()), flush=True)


@pytest.mark.parametrize("n_vit,n_dec", [(4, 2)])
def test_full_width_stack_32k_one_sample_through_all_layers(B, n_vit, n_dec):
    """The benchmark's microbatch (seed 414, 32768 packed tokens, 39 images) through 4 ViT-L layers +
    connector + 2 8B-GQA layers at full width.  The GPU runs the whole microbatch; the oracle runs the
    shortest image-bearing sample alone through every layer.  Its rows of y, dx_seq and dx_img must
    match at the stated tolerances: a sample's rows do not depend on what it is packed with (Model
    Profiler, "Throughput Profiling")."""
    wl = W.workload_full_stage(414, 32768, "8b", n_vit=n_vit, n_dec=n_dec)
    scale = 1.0
    assert len(wl.layers) <= 8
    st = GpuStage(B, wl.layers)
    try:
        y, dx_img, dx_seq, _ = st.run(wl)
        y, dx_img, dx_seq = host_f64(y), host_f64(dx_img), host_f64(dx_seq)
    finally:
        st.close()
    samples = wl.batch.samples
    _, i = min((W.IMG_TOKENS * k + t, i) for i, (k, t) in enumerate(samples) if k >= 1)
    k, t = samples[i]
    cu = wl.batch.seq.cu_seqlens
    a, b = int(cu[i]), int(cu[i + 1])
    i0 = W.IMG_TOKENS * sum(kk for kk, _ in samples[:i])
    i1 = i0 + W.IMG_TOKENS * k
    one = W.batch_from_samples([(k, t)])
    y_ref, caches = O.stage_fwd(wl.layers, wl.params, one, wl.x_img[i0:i1], wl.x_seq[a:b])
    dxi_ref, dxs_ref, _ = O.stage_bwd(wl.layers, wl.params, one, caches, wl.dy[a:b].astype(np.float64))
    errs = dict(y=nmax_err(y[a:b], y_ref), dx_seq=nmax_err(dx_seq[a:b], dxs_ref), dx_img=nmax_err(dx_img[i0:i1], dxi_ref))
    print("layers %d, tolerance scale %.2f, errors %s" % (len(wl.layers), scale, errs), flush=True)
    assert errs["y"] <= 2e-2 * scale, errs
    assert errs["dx_seq"] <= 3e-2 * scale and errs["dx_img"] <= 3e-2 * scale, errs
    assert np.all(dx_seq[a:a + W.IMG_TOKENS * k] == 0.0)      # rows the connector overwrote


@pytest.mark.parametrize("what", ["fwd_up", "dx_down", "dw_up", "dw_qkv", "dw_ragged_tokens"])
def test_gemm_full_shapes_sampled(B, what):
    T, d, f, nq = 32768, 4096, 14336, 6144
    rng = np.random.default_rng(7)
    if what == "dw_ragged_tokens":   # the InternViT-shaped MLP weight gradient over 23575 tokens (368 k-tiles + 23 rows)
        m, n, k, al, bl, f32 = 3200, 12800, 23575, 1, 0, 1
    elif what == "fwd_up":     # [T,d] . [d,2f]
        m, n, k, al, bl, f32 = T, 2 * f, d, 0, 0, 0
    elif what == "dx_down":    # dY[T,d] . W_d[f,d]^T
        m, n, k, al, bl, f32 = T, f, d, 0, 1, 0
    elif what == "dw_up":      # X[T,d]^T . dY[T,2f], fp32
        m, n, k, al, bl, f32 = d, 2 * f, T, 1, 0, 1
    else:                      # X[T,d]^T . dY[T,nq], fp32
        m, n, k, al, bl, f32 = d, nq, T, 1, 0, 1
    a = W.draw_tensor(71, *( (k, m) if al else (m, k) ))
    b = W.draw_tensor(72, *( (n, k) if bl else (k, n) ))
    c = torch.empty(m, n, dtype=torch.float32 if f32 else torch.bfloat16, device="cuda")
    B.mllm_op_gemm(dev_bf16(a), dev_bf16(b), c, m, n, k, al, bl, f32)
    rows = np.unique(np.concatenate([rng.integers(0, m, 24), [0, m - 1, 255, 256]]))
    cols = np.unique(np.concatenate([rng.integers(0, n, 48), [0, n - 1, 255, 256]]))
    got = host_f64(c[torch.as_tensor(rows, device="cuda")][:, torch.as_tensor(cols, device="cuda")])
    A = (a[:, rows].T if al else a[rows]).astype(np.float64)          # [rows, k]
    Bm = (b[cols].T if bl else b[:, cols]).astype(np.float64)         # [k, cols]
    ref = A @ Bm
    assert nmax_err(got, ref) < (2e-3 if f32 else 1e-2)


def test_attention_full_shape_sampled(B):
    """The 8B-GQA attention at 32768 packed tokens; oracle on sampled (segment, head) pairs."""
    hq, hkv, hd = 32, 8, 128
    pack = W.workload_dec8b(300, with_data=False).batch.seq
    T = pack.total_tokens
    nq = (hq + 2 * hkv) * hd
    qkv = W.draw_tensor(81, T, nq)
    do = W.draw_tensor(82, T, hq * hd)
    dq_ = dev_bf16(qkv)
    o = torch.zeros(T, hq * hd, dtype=torch.bfloat16, device="cuda")
    lse = torch.zeros(hq, T, dtype=torch.float32, device="cuda")
    delta = torch.zeros(hq, T, dtype=torch.float32, device="cuda")
    dqkv = torch.zeros(T, nq, dtype=torch.bfloat16, device="cuda")
    ws = scratch(B.mllm_op_attn_workspace_bytes(pack.n_segments, T, hq))
    qp = dq_.data_ptr()
    kp, vp = qp + hq * hd * 2, qp + (hq + hkv) * hd * 2
    gp = dqkv.data_ptr()
    B.mllm_op_attn_fwd(qp, kp, vp, o, lse, pack, hq, hkv, hd, nq, nq, hq * hd, ws)
    B.mllm_op_attn_bwd(qp, kp, vp, o, lse, dev_bf16(do), gp, gp + hq * hd * 2, gp + (hq + hkv) * hd * 2, delta,
                       pack, hq, hkv, hd, nq, nq, hq * hd, ws)
    o_h, g_h, lse_h = host_f64(o), host_f64(dqkv), host_f64(lse)
    cu = pack.cu_seqlens
    lens = np.diff(cu)
    order = np.argsort(lens)
    for s, g in ((int(order[-1]), 3), (int(order[len(order) // 2]), 0), (int(order[0]), 7)):
        a, b = int(cu[s]), int(cu[s + 1])
        heads = list(range(4 * g, 4 * g + 4))       # the whole GQA group, so that dk / dv can be checked
        q = qkv[a:b, :hq * hd].reshape(b - a, hq, hd)[:, heads].astype(np.float64)
        k = qkv[a:b, hq * hd:(hq + hkv) * hd].reshape(b - a, hkv, hd)[:, g:g + 1].astype(np.float64)
        v = qkv[a:b, (hq + hkv) * hd:].reshape(b - a, hkv, hd)[:, g:g + 1].astype(np.float64)
        d_o = do[a:b].reshape(b - a, hq, hd)[:, heads].astype(np.float64)
        one = W.make_pack([b - a], W.MASK_CAUSAL)
        o_ref, lse_ref = O.attention_fwd(q, k, v, one.cu_seqlens, one.mask_kind, return_lse=True)
        dq_ref, dk_ref, dv_ref = O.attention_bwd(d_o, q, k, v, one.cu_seqlens, one.mask_kind)
        got_o = o_h[a:b].reshape(b - a, hq, hd)[:, heads]
        assert nmax_err(got_o, o_ref) < 2e-2, (s, g)
        assert np.max(np.abs(lse_h[heads, a:b] - lse_ref)) < 2e-2
        got_dq = g_h[a:b, :hq * hd].reshape(b - a, hq, hd)[:, heads]
        got_dk = g_h[a:b, hq * hd:(hq + hkv) * hd].reshape(b - a, hkv, hd)[:, g:g + 1]
        got_dv = g_h[a:b, (hq + hkv) * hd:].reshape(b - a, hkv, hd)[:, g:g + 1]
        assert nmax_err(got_dq, dq_ref) < 3e-2, (s, g)
        assert nmax_err(got_dk, dk_ref) < 3e-2, (s, g)
        assert nmax_err(got_dv, dv_ref) < 3e-2, (s, g)


def test_gemm_operand_above_two_gib(B):
    """A weight-gradient product whose [tokens, width] operand is 2.3 GB (offsets beyond 2^31)."""
    T, m, n = 40000, 64, 28672
    x = W.draw_tensor(95, T, m)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(5)
    dy = torch.randn(T, n, generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    dw = torch.empty(m, n, dtype=torch.float32, device="cuda")
    B.mllm_op_gemm(dev_bf16(x), dy, dw, m, n, T, a_layout=1, b_layout=0, out_fp32=1)
    cols = torch.tensor([0, 1, 255, 256, 14335, 14336, 20000, n - 1], device="cuda")
    ref = x.astype(np.float64).T @ host_f64(dy[:, cols])
    assert nmax_err(host_f64(dw[:, cols]), ref) < 2e-3
