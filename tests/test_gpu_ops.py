"""Per-kernel parity: each HIP operation, called through the C ABI, against the fp64 oracle on the
same seeded bf16-grid inputs.  Sizes span several tiles and a ragged tail.

Tolerances (normalised max error, max|gpu - oracle| / max|oracle|):
  * a single operation whose output is bf16 carries one rounding of the result (2^-9 relative)
    plus fp32 accumulation error: 1e-2 is used (outputs far below the row maximum dominate);
  * fp32 outputs of bf16 products accumulated in fp32: 2e-3;
  * attention: bf16 probabilities inside the kernel, so the stage tolerances apply: 2e-2 on
    outputs, 3e-2 on gradients.
"""
import math

import numpy as np
import pytest

import workloads as W
from oracle import stage_oracle as O

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from tests.gpu_util import dev_bf16, empty_bf16, host_f64, nmax_err, scratch  # noqa: E402


@pytest.fixture(scope="module")
def B():
    from paper_2603_25120_amd import binding
    binding.lib()
    return binding


@pytest.mark.parametrize("m,n,k", [(263, 576, 192), (128, 128, 64), (300, 256, 1024), (1, 64, 64), (517, 192, 263 * 8)])
@pytest.mark.parametrize("a_layout,b_layout", [(0, 0), (0, 1), (1, 0), (1, 1)])
def test_gemm_layouts(B, m, n, k, a_layout, b_layout):
    a = W.draw_tensor(1, m, k)
    b = W.draw_tensor(2, k, n) * np.float32(0.125)
    a_st = np.ascontiguousarray(a.T) if a_layout else a
    b_st = np.ascontiguousarray(b.T) if b_layout else b
    if (a_layout and m % 8) or (b_layout and k % 8) or (not a_layout and k % 8):
        # an operand whose contiguous dimension is no multiple of 8 is outside the API: refused, nothing written
        c = torch.full((m, n), 3.0, dtype=torch.bfloat16, device="cuda")
        with pytest.raises(B.MllmError) as e:
            B.mllm_op_gemm(dev_bf16(a_st), dev_bf16(b_st), c, m, n, k, a_layout, b_layout)
        assert e.value.status == 3 and "multiples of 8" in str(e.value)
        torch.cuda.synchronize()
        assert bool((c == 3.0).all())
        return
    ref = a.astype(np.float64) @ b.astype(np.float64)
    c = empty_bf16(m, n)
    B.mllm_op_gemm(dev_bf16(a_st), dev_bf16(b_st), c, m, n, k, a_layout, b_layout)
    assert nmax_err(host_f64(c), ref) < 1e-2
    c32 = torch.empty(m, n, dtype=torch.float32, device="cuda")
    B.mllm_op_gemm(dev_bf16(a_st), dev_bf16(b_st), c32, m, n, k, a_layout, b_layout, out_fp32=1)
    assert nmax_err(host_f64(c32), ref) < 2e-3


@pytest.mark.parametrize("a_layout,b_layout,f32", [(0, 0, 0), (0, 1, 0), (1, 0, 1), (1, 1, 0), (0, 0, 1)])
def test_gemm_large_ragged(B, a_layout, b_layout, f32):
    """Enough 256x256 tiles to take the large-tile kernel, with ragged M, N and K edges."""
    m, n, k = 3512, 4104, 264
    a = W.draw_tensor(61, m, k)
    b = W.bf16_round(W.draw_tensor(62, k, n) * np.float32(0.125))
    a_st = np.ascontiguousarray(a.T) if a_layout else a
    b_st = np.ascontiguousarray(b.T) if b_layout else b
    ref = a.astype(np.float64) @ b.astype(np.float64)
    bias = W.draw_tensor(63, 1, n)
    c = torch.zeros(m, n, dtype=torch.float32 if f32 else torch.bfloat16, device="cuda")
    B.mllm_op_gemm(dev_bf16(a_st), dev_bf16(b_st), c, m, n, k, a_layout, b_layout, out_fp32=f32, bias=dev_bf16(bias))
    assert nmax_err(host_f64(c), ref + bias) < (2e-3 if f32 else 1e-2)
    # second call with a different K so that stale LDS contents would show
    k2 = 72
    ref2 = a[:, :k2].astype(np.float64) @ b[:k2].astype(np.float64)
    a2 = np.ascontiguousarray(a[:, :k2].T) if a_layout else np.ascontiguousarray(a[:, :k2])
    b2 = np.ascontiguousarray(b[:k2].T) if b_layout else np.ascontiguousarray(b[:k2])
    B.mllm_op_gemm(dev_bf16(a2), dev_bf16(b2), c, m, n, k2, a_layout, b_layout, out_fp32=f32)
    assert nmax_err(host_f64(c), ref2) < (2e-3 if f32 else 1e-2)


@pytest.mark.parametrize("k", [64, 128, 192, 320, 1024])
@pytest.mark.parametrize("a_layout,b_layout,f32", [(0, 0, 0), (0, 1, 0), (1, 0, 0), (1, 1, 0),
                                                   (0, 0, 1), (0, 1, 1), (1, 0, 1), (1, 1, 1)])
def test_gemm_large_tiles_k_multiple_of_64(B, k, a_layout, b_layout, f32):
    """The four-wavefront 256x256 kernel (enough tiles, K a multiple of 64): one, two, an odd and
    an even number of k-tiles, ragged M and N, every layout, with the fused epilogue terms."""
    m, n = 3512, 4104
    a = W.draw_tensor(71, m, k)
    b = W.bf16_round(W.draw_tensor(72, k, n) * np.float32(0.125))
    a_st = np.ascontiguousarray(a.T) if a_layout else a
    b_st = np.ascontiguousarray(b.T) if b_layout else b
    ref = a.astype(np.float64) @ b.astype(np.float64)
    bias = W.draw_tensor(73, 1, n)
    if f32:
        init = np.random.default_rng(74).standard_normal((m, n)).astype(np.float32)
        c = torch.from_numpy(init.copy()).cuda()
        B.mllm_op_gemm(dev_bf16(a_st), dev_bf16(b_st), c, m, n, k, a_layout, b_layout, out_fp32=1, accumulate=1,
                       bias=dev_bf16(bias))
        assert nmax_err(host_f64(c), ref + bias + init) < 2e-3
    else:
        res = W.draw_tensor(75, m, n)
        c = empty_bf16(m, n)
        B.mllm_op_gemm(dev_bf16(a_st), dev_bf16(b_st), c, m, n, k, a_layout, b_layout, bias=dev_bf16(bias),
                       residual=dev_bf16(res))
        assert nmax_err(host_f64(c), ref + bias + res) < 1e-2


@pytest.mark.parametrize("k", [65, 127, 129, 200, 1000, 2350])
@pytest.mark.parametrize("f32", [1, 0])
def test_gemm_large_tiles_weight_gradient_ragged_k(B, k, f32):
    """The weight-gradient layout (both operands stored [K, .]) keeps the four-wavefront kernel when
    K is no multiple of 64: the rows of the last k-tile past K must read as zeros.  The operands are
    the leading K rows of longer buffers whose later rows hold large values, so a row read past K
    would show."""
    m, n = 3512, 4104
    a = W.draw_tensor(171, k + 64, m)
    b = W.bf16_round(W.draw_tensor(172, k + 64, n) * np.float32(0.125))
    a[k:] = 1000.0
    b[k:] = 1000.0
    ref = a[:k].T.astype(np.float64) @ b[:k].astype(np.float64)
    a_dev, b_dev = dev_bf16(a), dev_bf16(b)
    if f32:
        init = np.random.default_rng(174).standard_normal((m, n)).astype(np.float32)
        c = torch.from_numpy(init.copy()).cuda()
        B.mllm_op_gemm(a_dev, b_dev, c, m, n, k, 1, 0, out_fp32=1, accumulate=1)
        assert nmax_err(host_f64(c), ref + init) < 2e-3
    else:
        c = empty_bf16(m, n)
        B.mllm_op_gemm(a_dev, b_dev, c, m, n, k, 1, 0)
        assert nmax_err(host_f64(c), ref) < 1e-2


@pytest.mark.parametrize("m,f,k", [(4200, 1536, 320), (4352, 1664, 64), (6401, 1024, 192)])
def test_gemm_swiglu_fused(B, m, f, k):
    """Up-projection with the activation in the same pass: [gate | up] = x.W and silu(gate) * up,
    ragged rows, one to five k-tiles; the unfused pair of operations must agree with it too."""
    x = W.draw_tensor(181, m, k)
    w = W.bf16_round(W.draw_tensor(182, k, 2 * f) * np.float32(0.125))
    pre_ref = x.astype(np.float64) @ w.astype(np.float64)
    g, u = pre_ref[:, :f], pre_ref[:, f:]
    act_ref = g / (1.0 + np.exp(-g)) * u
    pre = torch.full((m, 2 * f), float("nan"), dtype=torch.bfloat16, device="cuda")
    act = torch.full((m, f), float("nan"), dtype=torch.bfloat16, device="cuda")
    xd, wd = dev_bf16(x), dev_bf16(w)
    B.mllm_op_gemm_swiglu(xd, wd, pre, act, m, f, k)
    assert nmax_err(host_f64(pre), pre_ref) < 1e-2
    assert nmax_err(host_f64(act), act_ref) < 2e-2
    pre2, act2 = empty_bf16(m, 2 * f), empty_bf16(m, f)
    B.mllm_op_gemm(xd, wd, pre2, m, 2 * f, k)
    B.mllm_op_act_fwd(W.ACT_SWIGLU, pre2, act2, m, f)
    assert torch.equal(pre, pre2)                       # the same accumulators, the same rounding
    assert nmax_err(host_f64(act), host_f64(act2)) < 2e-2


@pytest.mark.parametrize("m,f,k", [(4200, 3080, 320), (4352, 3328, 64), (6401, 2048, 192)])
def test_gemm_swiglu_gradient_fused(B, m, f, k):
    """Down-projection's input gradient with SwiGLU's gradient in the same pass: dA = dy.W_d^T is
    never stored, [d gate | d up] is; ragged rows and (first case) a ragged last tile column."""
    dy = W.draw_tensor(191, m, k)
    w = W.bf16_round(W.draw_tensor(192, f, k) * np.float32(0.125))
    pre = W.draw_tensor(193, m, 2 * f)
    da = dy.astype(np.float64) @ w.astype(np.float64).T
    g, u = pre[:, :f].astype(np.float64), pre[:, f:].astype(np.float64)
    s = 1.0 / (1.0 + np.exp(-g))
    ref = np.concatenate([da * u * s * (1.0 + g * (1.0 - s)), da * g * s], axis=1)
    dpre = torch.full((m, 2 * f), float("nan"), dtype=torch.bfloat16, device="cuda")
    dyd, wd, pred = dev_bf16(dy), dev_bf16(w), dev_bf16(pre)
    B.mllm_op_gemm_swiglu_bwd(dyd, wd, pred, dpre, m, f, k)
    assert nmax_err(host_f64(dpre), ref) < 2e-2
    da2, dpre2 = empty_bf16(m, f), empty_bf16(m, 2 * f)
    B.mllm_op_gemm(dyd, wd, da2, m, f, k, 0, 1)
    B.mllm_op_act_bwd(W.ACT_SWIGLU, da2, pred, dpre2, m, f)
    assert nmax_err(host_f64(dpre), host_f64(dpre2)) < 2e-2


@pytest.mark.parametrize("seed", range(8))
def test_gemm_large_tiles_random_shapes(B, seed):
    """Seeded random problems that take the four-wavefront kernel: ragged M and N in every
    residue class of the 256-wide tiles, 1 to 12 k-tiles, random layouts and output types."""
    rng = np.random.default_rng(9000 + seed)
    m, n = 8 * int(rng.integers(365, 520)), 8 * int(rng.integers(375, 540))
    k = 64 * int(rng.integers(1, 13))
    a_layout, b_layout, f32 = (int(v) for v in rng.integers(0, 2, 3))
    a = W.draw_tensor(81 + seed, m, k)
    b = W.bf16_round(W.draw_tensor(91 + seed, k, n) * np.float32(0.125))
    a_st = np.ascontiguousarray(a.T) if a_layout else a
    b_st = np.ascontiguousarray(b.T) if b_layout else b
    ref = a.astype(np.float64) @ b.astype(np.float64)
    c = torch.empty(m, n, dtype=torch.float32 if f32 else torch.bfloat16, device="cuda")
    B.mllm_op_gemm(dev_bf16(a_st), dev_bf16(b_st), c, m, n, k, a_layout, b_layout, out_fp32=f32)
    assert nmax_err(host_f64(c), ref) < (2e-3 if f32 else 1e-2)


@pytest.mark.parametrize("k", [64, 192, 1024])
@pytest.mark.parametrize("b_layout,f32", [(0, 0), (1, 0), (0, 1), (1, 1)])
def test_gemm_192_row_tiles(B, k, b_layout, f32):
    """5640 x 4096 outputs are 368 tiles of 256x256 (two rounds of 256 workgroups, the second
    mostly empty) and 480 tiles of 192x256: the kernel's 192-row form takes these.  Ragged last
    row tile, both B layouts, both output types, fused epilogue terms."""
    m, n = 5640, 4096
    a = W.draw_tensor(101, m, k)
    b = W.bf16_round(W.draw_tensor(102, k, n) * np.float32(0.125))
    b_st = np.ascontiguousarray(b.T) if b_layout else b
    ref = a.astype(np.float64) @ b.astype(np.float64)
    bias = W.draw_tensor(103, 1, n)
    if f32:
        c = torch.zeros(m, n, dtype=torch.float32, device="cuda")
        B.mllm_op_gemm(dev_bf16(a), dev_bf16(b_st), c, m, n, k, 0, b_layout, out_fp32=1, bias=dev_bf16(bias))
        assert nmax_err(host_f64(c), ref + bias) < 2e-3
    else:
        res = W.draw_tensor(104, m, n)
        c = empty_bf16(m, n)
        B.mllm_op_gemm(dev_bf16(a), dev_bf16(b_st), c, m, n, k, 0, b_layout, bias=dev_bf16(bias), residual=dev_bf16(res))
        assert nmax_err(host_f64(c), ref + bias + res) < 1e-2


def test_gemm_epilogues(B):
    m, n, k = 333, 192, 256
    a, b = W.draw_tensor(3, m, k), W.bf16_round(W.draw_tensor(4, k, n) * np.float32(0.1))
    bias, res = W.draw_tensor(5, 1, n), W.draw_tensor(6, m, n)
    ref = a.astype(np.float64) @ b + bias + res
    c = empty_bf16(m, n)
    B.mllm_op_gemm(dev_bf16(a), dev_bf16(b), c, m, n, k, bias=dev_bf16(bias), residual=dev_bf16(res))
    assert nmax_err(host_f64(c), ref) < 1e-2
    # fp32 accumulate: C += A.B twice on top of an initial value
    init = np.random.default_rng(7).standard_normal((m, n)).astype(np.float32)
    c32 = torch.from_numpy(init.copy()).cuda()
    for _ in range(2):
        B.mllm_op_gemm(dev_bf16(a), dev_bf16(b), c32, m, n, k, out_fp32=1, accumulate=1)
    assert nmax_err(host_f64(c32), init + 2 * (a.astype(np.float64) @ b)) < 2e-3


def test_gemm_weight_gradient_shape(B):
    # dW[k, n] = X[T, k]^T . dY[T, n], contraction over a ragged token count
    T, k, n = 263, 192, 576
    x, dy = W.draw_tensor(8, T, k), W.draw_tensor(9, T, n)
    dw = torch.empty(k, n, dtype=torch.float32, device="cuda")
    B.mllm_op_gemm(dev_bf16(x), dev_bf16(dy), dw, k, n, T, a_layout=1, b_layout=0, out_fp32=1)
    assert nmax_err(host_f64(dw), x.astype(np.float64).T @ dy) < 2e-3


def test_gemm_zero_contraction(B):
    c32 = torch.full((64, 64), 3.0, dtype=torch.float32, device="cuda")
    dummy = empty_bf16(64, 8)
    B.mllm_op_gemm(dummy, dummy, c32, 64, 64, 0, a_layout=1, b_layout=0, out_fp32=1)
    assert float(c32.abs().max()) == 0.0


ATTN_CASES = [
    # (head_dim, n_q, n_kv, lengths, kinds)
    (64, 3, 3, [64, 64], [0, 0]),
    (64, 4, 4, [96, 0, 1, 130, 257], [1, 1, 1, 1, 1]),
    (128, 4, 2, [300, 5, 127, 128, 129], [1, 0, 1, 0, 1]),
    (128, 8, 2, [700], [1]),
    (64, 2, 2, [576, 576], [0, 0]),
    (128, 2, 1, [0, 1, 64, 65, 191, 260], [1, 0, 1, 0, 1, 1]),   # empty, one-row and just-over-a-tile samples, one kv head
]


@pytest.mark.parametrize("hd,hq,hkv,lengths,kinds", ATTN_CASES)
def test_attention_fwd_bwd(B, hd, hq, hkv, lengths, kinds):
    pack = W.make_pack(lengths, 0)
    pack.mask_kind[:] = np.asarray(kinds, dtype=np.uint8)
    T = pack.total_tokens
    nq = (hq + 2 * hkv) * hd
    qkv = W.draw_tensor(11, T, nq)
    do = W.draw_tensor(12, T, hq * hd)
    q = qkv[:, :hq * hd].reshape(T, hq, hd).astype(np.float64)
    k = qkv[:, hq * hd:(hq + hkv) * hd].reshape(T, hkv, hd).astype(np.float64)
    v = qkv[:, (hq + hkv) * hd:].reshape(T, hkv, hd).astype(np.float64)
    o_ref, lse_ref = O.attention_fwd(q, k, v, pack.cu_seqlens, pack.mask_kind, return_lse=True)
    dq_ref, dk_ref, dv_ref = O.attention_bwd(do.reshape(T, hq, hd).astype(np.float64), q, k, v,
                                             pack.cu_seqlens, pack.mask_kind)
    d_qkv = dev_bf16(qkv)
    o = torch.zeros(T, hq * hd, dtype=torch.bfloat16, device="cuda")
    lse = torch.zeros(hq, T, dtype=torch.float32, device="cuda")
    ws = scratch(B.mllm_op_attn_workspace_bytes(pack.n_segments, T, hq))
    esz = 2
    qp, kp, vp = d_qkv.data_ptr(), d_qkv.data_ptr() + hq * hd * esz, d_qkv.data_ptr() + (hq + hkv) * hd * esz
    B.mllm_op_attn_fwd(qp, kp, vp, o, lse, pack, hq, hkv, hd, nq, nq, hq * hd, ws)
    assert nmax_err(host_f64(o), o_ref.reshape(T, -1)) < 2e-2
    assert np.max(np.abs(host_f64(lse) - lse_ref)) < 2e-2
    dqkv = torch.zeros(T, nq, dtype=torch.bfloat16, device="cuda")
    delta = torch.zeros(hq, T, dtype=torch.float32, device="cuda")
    gp = dqkv.data_ptr()
    B.mllm_op_attn_bwd(qp, kp, vp, o, lse, dev_bf16(do), gp, gp + hq * hd * esz, gp + (hq + hkv) * hd * esz,
                       delta, pack, hq, hkv, hd, nq, nq, hq * hd, ws)
    g = host_f64(dqkv)
    assert nmax_err(g[:, :hq * hd], dq_ref.reshape(T, -1)) < 3e-2
    assert nmax_err(g[:, hq * hd:(hq + hkv) * hd], dk_ref.reshape(T, -1)) < 3e-2
    assert nmax_err(g[:, (hq + hkv) * hd:], dv_ref.reshape(T, -1)) < 3e-2


def test_attention_exact_cases(B):
    """Length-1 segments and the first token of a causal segment return v bit for bit."""
    hd, hq = 64, 2
    pack = W.make_pack([1, 40, 1], 1)
    T = pack.total_tokens
    qkv = W.draw_tensor(13, T, 3 * hq * hd)
    d = dev_bf16(qkv)
    o = empty_bf16(T, hq * hd)
    lse = torch.zeros(hq, T, dtype=torch.float32, device="cuda")
    ws = scratch(B.mllm_op_attn_workspace_bytes(3, T, hq))
    B.mllm_op_attn_fwd(d.data_ptr(), d.data_ptr() + hq * hd * 2, d.data_ptr() + 2 * hq * hd * 2, o, lse, pack,
                       hq, hq, hd, 3 * hq * hd, 3 * hq * hd, hq * hd, ws)
    got = host_f64(o)
    v = qkv[:, 2 * hq * hd:].astype(np.float64)
    for t in (0, 1, T - 1):
        assert np.array_equal(got[t], v[t])


@pytest.mark.parametrize("kind", [0, 1])
@pytest.mark.parametrize("t,d", [(263, 192), (130, 1024), (37, 4096), (5, 256)])
def test_norm_fwd_bwd(B, kind, t, d):
    x = W.bf16_round(W.draw_tensor(21, t, d) * np.float32(1.5) + np.float32(0.25))
    g = W.bf16_round(1 + 0.02 * np.random.default_rng(22).standard_normal((1, d)).astype(np.float32))
    b = W.bf16_round(0.02 * np.random.default_rng(23).standard_normal((1, d)).astype(np.float32))
    dy, dres = W.draw_tensor(24, t, d), W.draw_tensor(25, t, d)
    eps = 1e-5
    if kind == 0:
        y_ref, cache = O.layernorm_fwd(x.astype(np.float64), g.astype(np.float64), b.astype(np.float64), eps)
        dx_ref, dg_ref, db_ref = O.layernorm_bwd(dy.astype(np.float64), cache, g.astype(np.float64))
    else:
        y_ref, cache = O.rmsnorm_fwd(x.astype(np.float64), g.astype(np.float64), eps)
        dx_ref, dg_ref = O.rmsnorm_bwd(dy.astype(np.float64), cache, g.astype(np.float64))
    dx_ref = dx_ref + dres
    dx_, dg_, db_ = dev_bf16(x), dev_bf16(g), dev_bf16(b)
    y = empty_bf16(t, d)
    stats = torch.zeros(2, t, dtype=torch.float32, device="cuda")
    B.mllm_op_norm_fwd(kind, dx_, dg_, db_, y, stats, t, d, eps)
    assert nmax_err(host_f64(y), y_ref) < 1e-2
    dx = empty_bf16(t, d)
    dgam = torch.full((d,), 1.0, dtype=torch.float32, device="cuda")
    dbet = torch.full((d,), 1.0, dtype=torch.float32, device="cuda")
    part = scratch(B.mllm_op_norm_bwd_partial_bytes(t, d))
    B.mllm_op_norm_bwd(kind, dev_bf16(dy), dx_, dg_, stats, dev_bf16(dres), dx, dgam, dbet, 1, part, t, d)
    assert nmax_err(host_f64(dx), dx_ref) < 1e-2
    assert nmax_err(host_f64(dgam), dg_ref[0] + 1.0) < 2e-3
    if kind == 0:
        assert nmax_err(host_f64(dbet), db_ref[0] + 1.0) < 2e-3
    if d > 1024:
        with pytest.raises(B.MllmError):
            B.mllm_op_norm_bwd_colsum(kind, dev_bf16(dy), dx_, dg_, stats, dev_bf16(dres), dx, dgam, dbet, dgam, 0, part, t, d)
        return
    # the same pass also sums the columns of dx (before rounding): dx itself and the other sums must not change
    dx2 = empty_bf16(t, d)
    dgam2 = torch.full((d,), 1.0, dtype=torch.float32, device="cuda")
    dbet2 = torch.full((d,), 1.0, dtype=torch.float32, device="cuda")
    dcol = torch.full((d,), -2.0, dtype=torch.float32, device="cuda")
    B.mllm_op_norm_bwd_colsum(kind, dev_bf16(dy), dx_, dg_, stats, dev_bf16(dres), dx2, dgam2, dbet2, dcol, 1, part, t, d)
    assert torch.equal(dx2, dx)
    assert nmax_err(host_f64(dgam2), dg_ref[0] + 1.0) < 2e-3
    if kind == 0:
        assert nmax_err(host_f64(dbet2), db_ref[0] + 1.0) < 2e-3
    assert nmax_err(host_f64(dcol), dx_ref.sum(axis=0) - 2.0) < 2e-3


@pytest.mark.parametrize("hd,base", [(64, 10000.0), (128, 500000.0)])
def test_rope(B, hd, base):
    lengths = [70, 1, 129]
    T, heads = sum(lengths), 5
    stride = heads * hd + 64
    z = W.draw_tensor(31, T, stride)
    pos = O.segment_positions(W.make_pack(lengths, 1).cu_seqlens) + 13000   # large angles too
    cos, sin = O.rope_tables(pos, hd, base)
    ref = O.rope_apply(z[:, :heads * hd].reshape(T, heads, hd).astype(np.float64), cos, sin).reshape(T, -1)
    dz = dev_bf16(z)
    dpos = torch.from_numpy(pos.astype(np.int32)).cuda()
    B.mllm_op_rope(dz, dpos, T, stride, 0, heads, hd, base, 0)
    got = host_f64(dz)
    assert nmax_err(got[:, :heads * hd], ref) < 1e-2
    assert np.array_equal(got[:, heads * hd:], z[:, heads * hd:].astype(np.float64))   # untouched columns
    B.mllm_op_rope(dz, dpos, T, stride, 0, heads, hd, base, 1)                          # inverse brings it back
    assert nmax_err(host_f64(dz)[:, :heads * hd], z[:, :heads * hd].astype(np.float64)) < 2e-2


@pytest.mark.parametrize("hd,base,bias", [(128, 500000.0, False), (64, 10000.0, True), (128, 10000.0, True)])
def test_gemm_with_rotary_epilogue(B, hd, base, bias):
    """The QKV projection with the rotary positions in its epilogue: 7 q/k heads + value columns, ragged last
    row tile, positions up to 13000 + 2300, against the fp64 product rotated by the oracle."""
    lengths = [2300, 1, 700, 1095 + 37]
    m, k = sum(lengths), 320
    n_rot = 7 * 128 if hd == 128 else 14 * 64              # rotated heads: a multiple of 128 columns
    n = n_rot + 256 + 3584                                  # plus value columns: 18 column tiles x 17 row tiles >= 200
    x = W.draw_tensor(51, m, k)
    w = W.bf16_round(W.draw_tensor(52, k, n) * np.float32(0.06))
    b = W.bf16_round(W.draw_tensor(53, 1, n) * np.float32(0.5)) if bias else None
    pos = (O.segment_positions(W.make_pack(lengths, 1).cu_seqlens) + 13000).astype(np.int32)
    n_pos = int(pos.max()) + 1
    table = torch.empty(n_pos, hd, dtype=torch.float32, device="cuda")
    B.mllm_op_rope_table(table, n_pos, hd, base)
    cos, sin = O.rope_tables(pos, hd, base)
    tab = host_f64(table)[pos]
    assert np.max(np.abs(tab[:, :hd // 2] - cos)) < 1e-6 and np.max(np.abs(tab[:, hd // 2:] - sin)) < 1e-6
    y64 = x.astype(np.float64) @ w.astype(np.float64) + (b.astype(np.float64) if bias else 0.0)
    ref = y64.copy()
    ref[:, :n_rot] = O.rope_apply(y64[:, :n_rot].reshape(m, n_rot // hd, hd), cos, sin).reshape(m, n_rot)
    y = torch.zeros(m, n, dtype=torch.bfloat16, device="cuda")
    B.mllm_op_gemm_rope(dev_bf16(x), dev_bf16(w), dev_bf16(b) if bias else None, y, m, n, k,
                        torch.from_numpy(pos).cuda(), table, n_rot, hd)
    got = host_f64(y)
    assert nmax_err(got[:, :n_rot], ref[:, :n_rot]) < 1e-2
    assert nmax_err(got[:, n_rot:], ref[:, n_rot:]) < 1e-2
    with pytest.raises(B.MllmError):                         # too few tiles for the large-tile kernel
        B.mllm_op_gemm_rope(dev_bf16(x), dev_bf16(w), None, y, 256, n, k, torch.from_numpy(pos).cuda(), table, n_rot, hd)


@pytest.mark.parametrize("hd,hq,hkv,lengths,kinds", [(128, 4, 1, [300, 1, 77], [1, 1, 1]), (64, 4, 2, [130, 64, 5], [1, 0, 1])])
def test_attention_bwd_with_rotary_gradient(B, hd, hq, hkv, lengths, kinds):
    """dq and dk leave the backward kernels rotated back: equal to the oracle's attention gradient followed
    by the oracle's inverse rotation; dv is untouched."""
    pack = W.make_pack(lengths, 0)
    pack.mask_kind[:] = np.asarray(kinds, dtype=np.uint8)
    T = pack.total_tokens
    nq = (hq + 2 * hkv) * hd
    qkv = W.draw_tensor(14, T, nq)
    do = W.draw_tensor(15, T, hq * hd)
    q = qkv[:, :hq * hd].reshape(T, hq, hd).astype(np.float64)
    k = qkv[:, hq * hd:(hq + hkv) * hd].reshape(T, hkv, hd).astype(np.float64)
    v = qkv[:, (hq + hkv) * hd:].reshape(T, hkv, hd).astype(np.float64)
    dq_ref, dk_ref, dv_ref = O.attention_bwd(do.reshape(T, hq, hd).astype(np.float64), q, k, v, pack.cu_seqlens, pack.mask_kind)
    cos, sin = O.rope_tables(O.segment_positions(pack.cu_seqlens), hd, 10000.0)
    dq_ref, dk_ref = O.rope_apply_inverse(dq_ref, cos, sin), O.rope_apply_inverse(dk_ref, cos, sin)
    table = torch.empty(max(lengths), hd, dtype=torch.float32, device="cuda")
    B.mllm_op_rope_table(table, max(lengths), hd, 10000.0)
    d_qkv = dev_bf16(qkv)
    o = torch.zeros(T, hq * hd, dtype=torch.bfloat16, device="cuda")
    lse = torch.zeros(hq, T, dtype=torch.float32, device="cuda")
    ws = scratch(B.mllm_op_attn_workspace_bytes(pack.n_segments, T, hq))
    qp, kp, vp = d_qkv.data_ptr(), d_qkv.data_ptr() + hq * hd * 2, d_qkv.data_ptr() + (hq + hkv) * hd * 2
    B.mllm_op_attn_fwd(qp, kp, vp, o, lse, pack, hq, hkv, hd, nq, nq, hq * hd, ws)
    dqkv = torch.zeros(T, nq, dtype=torch.bfloat16, device="cuda")
    delta = torch.zeros(hq, T, dtype=torch.float32, device="cuda")
    gp = dqkv.data_ptr()
    B.mllm_op_attn_bwd_rope(qp, kp, vp, o, lse, dev_bf16(do), gp, gp + hq * hd * 2, gp + (hq + hkv) * hd * 2, delta,
                            pack, hq, hkv, hd, nq, nq, hq * hd, table, ws)
    g = host_f64(dqkv)
    assert nmax_err(g[:, :hq * hd], dq_ref.reshape(T, -1)) < 3e-2
    assert nmax_err(g[:, hq * hd:(hq + hkv) * hd], dk_ref.reshape(T, -1)) < 3e-2
    assert nmax_err(g[:, (hq + hkv) * hd:], dv_ref.reshape(T, -1)) < 3e-2


@pytest.mark.parametrize("act", [0, 1, 2])
def test_activations(B, act):
    t, f = 77, 768
    width = 2 * f if act == 2 else f
    pre = W.draw_tensor(41, t, width) * np.float32(2.0)
    da = W.draw_tensor(42, t, f)
    p64 = pre.astype(np.float64)
    if act == 2:
        a_ref = O.swiglu_fwd(p64[:, :f], p64[:, f:])
        dgate, dup = O.swiglu_bwd(da.astype(np.float64), p64[:, :f], p64[:, f:])
        d_ref = np.concatenate([dgate, dup], axis=1)
    elif act == 1:
        a_ref, d_ref = O.gelu_tanh(p64), da * O.gelu_tanh_grad(p64)
    else:
        a_ref, d_ref = O.gelu_erf(p64), da * O.gelu_erf_grad(p64)
    a, dpre = empty_bf16(t, f), empty_bf16(t, width)
    B.mllm_op_act_fwd(act, dev_bf16(pre), a, t, f)
    B.mllm_op_act_bwd(act, dev_bf16(da), dev_bf16(pre), dpre, t, f)
    assert nmax_err(host_f64(a), a_ref) < 1e-2
    assert nmax_err(host_f64(dpre), d_ref) < 1e-2


@pytest.mark.parametrize("t,n", [(263, 576), (1, 64), (2000, 192), (0, 64)])
def test_colsum(B, t, n):
    x = W.draw_tensor(51, max(t, 1), n)[:t]
    out = torch.full((n,), 2.0, dtype=torch.float32, device="cuda")
    part = scratch(B.mllm_op_colsum_partial_bytes(t, n))
    xd = dev_bf16(x) if t else empty_bf16(1, n)
    B.mllm_op_colsum(xd, out, 1, part, t, n)
    ref = x.astype(np.float64).sum(axis=0) + 2.0
    assert np.max(np.abs(host_f64(out) - ref)) < 1e-3 * max(1.0, math.sqrt(t))


def test_attention_longest_possible_sample(B):
    """One causal sample of 13312 tokens (16 images + 4096 text tokens, the cap of the long-tailed
    mix), one GQA group: many key tiles per query tile, ragged last tile (13312 = 104 * 128)."""
    hd, hq, hkv, L = 128, 4, 1, 13312 - 57
    pack = W.make_pack([L], 1)
    nq = (hq + 2 * hkv) * hd
    qkv = W.draw_tensor(91, L, nq)
    do = W.draw_tensor(92, L, hq * hd)
    q = qkv[:, :hq * hd].reshape(L, hq, hd).astype(np.float64)
    k = qkv[:, hq * hd:(hq + hkv) * hd].reshape(L, hkv, hd).astype(np.float64)
    v = qkv[:, (hq + hkv) * hd:].reshape(L, hkv, hd).astype(np.float64)
    o_ref = O.attention_fwd(q, k, v, pack.cu_seqlens, pack.mask_kind)
    dq_ref, dk_ref, dv_ref = O.attention_bwd(do.reshape(L, hq, hd).astype(np.float64), q, k, v,
                                             pack.cu_seqlens, pack.mask_kind)
    d = dev_bf16(qkv)
    o = torch.zeros(L, hq * hd, dtype=torch.bfloat16, device="cuda")
    lse = torch.zeros(hq, L, dtype=torch.float32, device="cuda")
    delta = torch.zeros(hq, L, dtype=torch.float32, device="cuda")
    g = torch.zeros(L, nq, dtype=torch.bfloat16, device="cuda")
    ws = scratch(B.mllm_op_attn_workspace_bytes(1, L, hq))
    qp = d.data_ptr()
    B.mllm_op_attn_fwd(qp, qp + hq * hd * 2, qp + (hq + hkv) * hd * 2, o, lse, pack, hq, hkv, hd, nq, nq, hq * hd, ws)
    gp = g.data_ptr()
    B.mllm_op_attn_bwd(qp, qp + hq * hd * 2, qp + (hq + hkv) * hd * 2, o, lse, dev_bf16(do), gp, gp + hq * hd * 2,
                       gp + (hq + hkv) * hd * 2, delta, pack, hq, hkv, hd, nq, nq, hq * hd, ws)
    gh = host_f64(g)
    assert nmax_err(host_f64(o), o_ref.reshape(L, -1)) < 2e-2
    assert nmax_err(gh[:, :hq * hd], dq_ref.reshape(L, -1)) < 3e-2
    assert nmax_err(gh[:, hq * hd:(hq + hkv) * hd], dk_ref.reshape(L, -1)) < 3e-2
    assert nmax_err(gh[:, (hq + hkv) * hd:], dv_ref.reshape(L, -1)) < 3e-2
