"""Pins for the fp64 oracle: each test fixes the oracle against something that is not
the oracle itself -- brute force in scalar Python, closed forms, invariants, finite
differences, and (as a second opinion) PyTorch CPU fp64 autograd on a per-sample module.

The paper prints no worked numeric example for the stage computation, so the properties
below are the ones its text fixes: per-instance attention with causal integrity and
row-wise linear maps over the packed sequence (Model Profiler, "Throughput Profiling"),
packing along the sequence dimension ("Memory Profiling"), encoder on visual tokens and
LLM on visual + text tokens (Fig. 1 caption).
"""
import math

import numpy as np
import pytest

import workloads as W
from oracle import stage_oracle as O

RNG = np.random.default_rng(12345)


def _rand(*shape):
    return RNG.standard_normal(shape)


# ---------------------------------------------------------------------------
# attention: brute force, closed forms, invariants
# ---------------------------------------------------------------------------
def _attention_scalar(q, k, v, cu, kinds):
    """Scalar-loop definition: softmax over the visible keys of the token's own segment."""
    T, Hq, hd = q.shape
    grp = Hq // k.shape[1]
    o = np.zeros_like(q)
    for s in range(len(cu) - 1):
        for t in range(cu[s], cu[s + 1]):
            last = t if kinds[s] == W.MASK_CAUSAL else cu[s + 1] - 1
            for h in range(Hq):
                g = h // grp
                sc = [sum(q[t, h, c] * k[u, g, c] for c in range(hd)) / math.sqrt(hd)
                      for u in range(cu[s], last + 1)]
                m = max(sc)
                e = [math.exp(x - m) for x in sc]
                z = sum(e)
                for c in range(hd):
                    o[t, h, c] = sum(e[i] / z * v[cu[s] + i, g, c] for i in range(len(e)))
    return o


def test_attention_matches_scalar_brute_force():
    cu = np.array([0, 5, 5, 12, 13], dtype=np.int32)     # includes an empty and a length-1 segment
    kinds = np.array([1, 1, 0, 1], dtype=np.uint8)
    q, k, v = _rand(13, 4, 8), _rand(13, 2, 8), _rand(13, 2, 8)
    got = O.attention_fwd(q, k, v, cu, kinds)
    ref = _attention_scalar(q, k, v, cu, kinds)
    assert np.max(np.abs(got - ref)) < 1e-13


def test_attention_lse_is_log_sum_exp():
    cu = np.array([0, 7, 16], dtype=np.int32)
    kinds = np.array([1, 0], dtype=np.uint8)
    q, k, v = _rand(16, 2, 8), _rand(16, 2, 8), _rand(16, 2, 8)
    _, lse = O.attention_fwd(q, k, v, cu, kinds, return_lse=True)
    # token 9 (bidirectional segment 7..15), head 1
    sc = (k[7:16, 1] @ q[9, 1]) / math.sqrt(8)
    assert abs(lse[1, 9] - math.log(np.exp(sc).sum())) < 1e-13
    # token 3 of the causal segment sees keys 0..3
    sc = (k[0:4, 0] @ q[3, 0]) / math.sqrt(8)
    assert abs(lse[0, 3] - math.log(np.exp(sc).sum())) < 1e-13


def test_attention_query_blocking_changes_nothing(monkeypatch):
    cu = np.array([0, 37, 50], dtype=np.int32)
    kinds = np.array([1, 0], dtype=np.uint8)
    q, k, v, do = _rand(50, 2, 8), _rand(50, 1, 8), _rand(50, 1, 8), _rand(50, 2, 8)
    o1 = O.attention_fwd(q, k, v, cu, kinds)
    g1 = O.attention_bwd(do, q, k, v, cu, kinds)
    monkeypatch.setattr(O, "_Q_BLOCK", 7)
    o2 = O.attention_fwd(q, k, v, cu, kinds)
    g2 = O.attention_bwd(do, q, k, v, cu, kinds)
    assert np.max(np.abs(o1 - o2)) < 1e-13
    for a, b in zip(g1, g2):
        assert np.max(np.abs(a - b)) < 1e-12


def test_softmax_rows_sum_to_one_and_ds_rows_sum_to_zero():
    cu = np.array([0, 9, 20], dtype=np.int32)
    kinds = np.array([1, 0], dtype=np.uint8)
    q, k = _rand(20, 2, 8), _rand(20, 2, 8)
    ones = np.ones((20, 2, 8))
    # v == 1  =>  o = sum of the probabilities of the row
    assert np.max(np.abs(O.attention_fwd(q, k, ones, cu, kinds) - 1.0)) < 1e-14
    # all keys of a head equal  =>  dq = (sum_u dS_tu) k = 0
    kconst = np.broadcast_to(_rand(1, 2, 8), (20, 2, 8)).copy()
    dq, _, _ = O.attention_bwd(_rand(20, 2, 8), q, kconst, _rand(20, 2, 8), cu, kinds)
    assert np.max(np.abs(dq)) < 1e-13


def test_attention_closed_forms():
    cu = np.array([0, 6, 7, 15], dtype=np.int32)
    kinds = np.array([1, 1, 0], dtype=np.uint8)
    k, v = _rand(15, 2, 4), _rand(15, 2, 4)
    o = O.attention_fwd(np.zeros((15, 2, 4)), k, v, cu, kinds)
    for t in range(6):                       # q == 0, causal: prefix mean of v
        assert np.max(np.abs(o[t] - v[0:t + 1].mean(axis=0))) < 1e-14
    assert np.max(np.abs(o[6] - v[6])) < 1e-15          # a length-1 segment returns v
    for t in range(7, 15):                   # q == 0, bidirectional: mean over the image
        assert np.max(np.abs(o[t] - v[7:15].mean(axis=0))) < 1e-14
    q = _rand(15, 2, 4)
    o = O.attention_fwd(q, k, v, cu, kinds)
    assert np.max(np.abs(o[0] - v[0])) < 1e-15          # first token of a causal segment


def test_gqa_equals_mha_with_repeated_kv_heads():
    cu = np.array([0, 11, 19], dtype=np.int32)
    kinds = np.array([1, 1], dtype=np.uint8)
    q, k, v, do = _rand(19, 8, 4), _rand(19, 2, 4), _rand(19, 2, 4), _rand(19, 8, 4)
    kr, vr = np.repeat(k, 4, axis=1), np.repeat(v, 4, axis=1)   # blocked head map h -> h // 4
    assert np.max(np.abs(O.attention_fwd(q, k, v, cu, kinds) - O.attention_fwd(q, kr, vr, cu, kinds))) < 1e-14
    dq, dk, dv = O.attention_bwd(do, q, k, v, cu, kinds)
    dq2, dk2, dv2 = O.attention_bwd(do, q, kr, vr, cu, kinds)
    assert np.max(np.abs(dq - dq2)) < 1e-13
    assert np.max(np.abs(dk - dk2.reshape(19, 2, 4, 4).sum(axis=2))) < 1e-13
    assert np.max(np.abs(dv - dv2.reshape(19, 2, 4, 4).sum(axis=2))) < 1e-13


def test_attention_backward_finite_differences():
    cu = np.array([0, 6, 14], dtype=np.int32)
    kinds = np.array([1, 0], dtype=np.uint8)
    q, k, v, do = _rand(14, 4, 8), _rand(14, 2, 8), _rand(14, 2, 8), _rand(14, 4, 8)
    dq, dk, dv = O.attention_bwd(do, q, k, v, cu, kinds)
    h = 1e-6
    for name, arr, grad in (("q", q, dq), ("k", k, dk), ("v", v, dv)):
        dirn = _rand(*arr.shape)
        args = dict(q=q, k=k, v=v)
        args[name] = arr + h * dirn
        fp = O.attention_fwd(args["q"], args["k"], args["v"], cu, kinds)
        args[name] = arr - h * dirn
        fm = O.attention_fwd(args["q"], args["k"], args["v"], cu, kinds)
        num = np.sum(do * (fp - fm)) / (2 * h)
        ana = np.sum(grad * dirn)
        assert abs(num - ana) <= 1e-7 * max(1.0, abs(ana)), name


# ---------------------------------------------------------------------------
# rotary positions
# ---------------------------------------------------------------------------
def test_rope_properties():
    hd = 16
    pos = np.array([0, 1, 5, 300, 13311])
    cos, sin = O.rope_tables(pos, hd, 10000.0)
    z = _rand(5, 3, hd)
    r = O.rope_apply(z, cos, sin)
    assert np.max(np.abs(np.linalg.norm(r, axis=2) - np.linalg.norm(z, axis=2))) < 1e-12
    assert np.max(np.abs(r[0] - z[0])) == 0.0                               # position 0 is identity
    assert np.max(np.abs(O.rope_apply_inverse(r, cos, sin) - z)) < 1e-12    # inverse = transpose
    # explicit pair rotation for one element: pairs are (i, i + hd/2), theta_i = base^(-2i/hd)
    i, t = 3, 2
    th = pos[t] * 10000.0 ** (-2.0 * i / hd)
    a, b = z[t, 1, i], z[t, 1, i + hd // 2]
    assert abs(r[t, 1, i] - (a * math.cos(th) - b * math.sin(th))) < 1e-12
    assert abs(r[t, 1, i + hd // 2] - (b * math.cos(th) + a * math.sin(th))) < 1e-12


def test_rope_inner_product_depends_on_offset_only():
    hd = 8
    qv, kv = _rand(1, 1, hd), _rand(1, 1, hd)

    def dot(m, n):
        cm, sm = O.rope_tables(np.array([m]), hd, 500000.0)
        cn, sn = O.rope_tables(np.array([n]), hd, 500000.0)
        return float(np.sum(O.rope_apply(qv, cm, sm) * O.rope_apply(kv, cn, sn)))

    assert abs(dot(17, 5) - dot(112, 100)) < 1e-12
    assert abs(dot(17, 5) - dot(12, 0)) < 1e-12
    assert abs(dot(17, 5) - dot(5, 17)) > 1e-6


def test_positions_restart_at_every_segment():
    cu = np.array([0, 3, 3, 7], dtype=np.int32)
    assert O.segment_positions(cu).tolist() == [0, 1, 2, 0, 1, 2, 3]


# ---------------------------------------------------------------------------
# norms and activations
# ---------------------------------------------------------------------------
def test_layernorm_closed_forms():
    x = _rand(6, 32) * 3 + 1.5
    eps = 1e-5
    y, _ = O.layernorm_fwd(x, np.ones((1, 32)), np.zeros((1, 32)), eps)
    var = x.var(axis=1)
    assert np.max(np.abs(y.mean(axis=1))) < 1e-14
    assert np.max(np.abs(y.var(axis=1) - var / (var + eps))) < 1e-13
    g, b = _rand(1, 32), _rand(1, 32)
    y2, cache = O.layernorm_fwd(x, g, b, eps)
    assert np.max(np.abs(y2 - (y * g + b))) < 1e-13
    dyv = _rand(6, 32)
    dx, dg, db = O.layernorm_bwd(dyv, cache, g)
    assert np.max(np.abs(dx.sum(axis=1))) < 1e-12              # orthogonal to the constant vector
    # ... and to the normalised row up to the eps term: sum(dx * xhat) = rstd * sum(dy*g*xhat) * eps/(var+eps)
    expect = (dyv * g * cache[0]).sum(axis=1) / np.sqrt(var + eps) * eps / (var + eps)
    assert np.max(np.abs((dx * cache[0]).sum(axis=1) - expect)) < 1e-12


def test_rmsnorm_closed_forms():
    eps = 1e-5
    g = _rand(1, 16)
    for c in (2.0, -0.5):
        y, _ = O.rmsnorm_fwd(np.full((1, 16), c), g, eps)
        assert np.max(np.abs(y - np.sign(c) * g / math.sqrt(1 + eps / c ** 2))) < 1e-14
    x = _rand(5, 16)
    y, cache = O.rmsnorm_fwd(x, g, eps)
    assert np.max(np.abs(y - x / np.sqrt((x ** 2).mean(axis=1, keepdims=True) + eps) * g)) < 1e-14


@pytest.mark.parametrize("which", ["ln", "rms"])
def test_norm_backward_finite_differences(which):
    x, dy, g, b = _rand(4, 24), _rand(4, 24), _rand(1, 24), _rand(1, 24)
    eps, h = 1e-5, 1e-6
    if which == "ln":
        f = lambda x_, g_, b_: O.layernorm_fwd(x_, g_, b_, eps)[0]
        dx, dg, db = O.layernorm_bwd(dy, O.layernorm_fwd(x, g, b, eps)[1], g)
    else:
        f = lambda x_, g_, b_: O.rmsnorm_fwd(x_, g_, eps)[0]
        dx, dg = O.rmsnorm_bwd(dy, O.rmsnorm_fwd(x, g, eps)[1], g)
        db = None
    vx, vg, vb = _rand(4, 24), _rand(1, 24), _rand(1, 24)
    num = np.sum(dy * (f(x + h * vx, g, b) - f(x - h * vx, g, b))) / (2 * h)
    assert abs(num - np.sum(dx * vx)) < 1e-7 * max(1, abs(num))
    num = np.sum(dy * (f(x, g + h * vg, b) - f(x, g - h * vg, b))) / (2 * h)
    assert abs(num - np.sum(dg * vg)) < 1e-7 * max(1, abs(num))
    if db is not None:
        num = np.sum(dy * (f(x, g, b + h * vb) - f(x, g, b - h * vb))) / (2 * h)
        assert abs(num - np.sum(db * vb)) < 1e-7 * max(1, abs(num))


def test_activation_values():
    assert O.gelu_erf(np.array([0.0]))[0] == 0.0
    assert abs(O.gelu_erf_grad(np.array([0.0]))[0] - 0.5) < 1e-15
    # GELU(z) = z * Phi(z): compare with the scalar error function of the C library
    for z in (-3.0, -0.7, 0.3, 1.0, 2.5):
        assert abs(O.gelu_erf(np.array([z]))[0] - z * 0.5 * (1 + math.erf(z / math.sqrt(2)))) < 1e-15
    assert abs(O.gelu_erf(np.array([1.0]))[0] - 0.8413447460685429) < 1e-15   # Phi(1)
    assert O.swiglu_fwd(np.array([0.0]), np.array([3.0]))[0] == 0.0
    assert abs(O.swiglu_fwd(np.array([1.0]), np.array([2.0]))[0] - 2.0 / (1 + math.exp(-1.0))) < 1e-15
    dg, du = O.swiglu_bwd(np.array([1.0]), np.array([0.7]), np.array([0.0]))
    assert dg[0] == 0.0 and abs(du[0] - 0.7 / (1 + math.exp(-0.7))) < 1e-15
    # tanh flavour stays within its known distance of the exact one
    z = np.linspace(-4, 4, 101)
    assert np.max(np.abs(O.gelu_tanh(z) - O.gelu_erf(z))) < 1e-3
    h = 1e-6
    for fn, gr in ((O.gelu_erf, O.gelu_erf_grad), (O.gelu_tanh, O.gelu_tanh_grad)):
        assert np.max(np.abs((fn(z + h) - fn(z - h)) / (2 * h) - gr(z))) < 1e-8


# ---------------------------------------------------------------------------
# whole stage at the tiny configuration
# ---------------------------------------------------------------------------
def _tiny(seed=0):
    wl = W.workload_tiny(seed)
    return wl


def _fwd(wl, params=None, x_img=None, x_seq=None):
    return O.stage_fwd(wl.layers, wl.params if params is None else params, wl.batch,
                       wl.x_img if x_img is None else x_img,
                       wl.x_seq if x_seq is None else x_seq)


@pytest.mark.parametrize("seed,variant", [(0, 0), (3, 0), (1, 1), (2, 2), (4, 3), (5, 4)])
def test_stage_gradients_by_central_differences(seed, variant):
    wl = (_tiny, W.workload_tiny_variant, W.workload_tiny_pooled, W.workload_tiny_merged,
          W.workload_tiny_qknorm)[variant](seed)
    y, caches = _fwd(wl)
    dy = wl.dy.astype(np.float64)
    dx_img, dx_seq, dparams = O.stage_bwd(wl.layers, wl.params, wl.batch, caches, dy)
    rng = np.random.default_rng(seed + 77)
    text_rows = np.setdiff1d(np.arange(wl.batch.seq.total_tokens), wl.batch.img_to_seq_row)

    def check(num, ana, what):
        assert abs(num - ana) <= 2e-6 * max(abs(ana), 1e-3), (what, num, ana)

    # the normalised q and k rows are small before the norm, so the same step is a larger relative
    # perturbation there: a smaller step keeps the truncation error under the bound
    h = 2e-6 if variant == 4 else 1e-5
    v = rng.standard_normal(wl.x_img.shape)
    num = np.sum(dy * (_fwd(wl, x_img=wl.x_img + h * v)[0] - _fwd(wl, x_img=wl.x_img - h * v)[0])) / (2 * h)
    check(num, np.sum(dx_img * v), "x_img")
    v = rng.standard_normal(wl.x_seq.shape)
    num = np.sum(dy * (_fwd(wl, x_seq=wl.x_seq + h * v)[0] - _fwd(wl, x_seq=wl.x_seq - h * v)[0])) / (2 * h)
    check(num, np.sum(dx_seq * v), "x_seq")
    # image rows of x_seq are overwritten by the projector output: zero gradient there
    assert np.all(dx_seq[wl.batch.img_to_seq_row] == 0.0)
    assert np.any(dx_seq[text_rows] != 0.0)
    names = [n for L in wl.layers for n, _, _ in W.param_specs(L)]
    for i, p in enumerate(wl.params):
        v = rng.standard_normal(p.shape)
        pp = [q.astype(np.float64) for q in wl.params]
        pm = [q.astype(np.float64) for q in wl.params]
        pp[i] = pp[i] + h * v
        pm[i] = pm[i] - h * v
        num = np.sum(dy * (_fwd(wl, params=pp)[0] - _fwd(wl, params=pm)[0])) / (2 * h)
        check(num, np.sum(dparams[i] * v), names[i])
    # a few single coordinates
    for i in (2, 4, 8, 10, 13, 15, 17, 19):
        p = wl.params[i].astype(np.float64)
        r, c = rng.integers(0, p.shape[0]), rng.integers(0, p.shape[1])
        pp = [q.astype(np.float64) for q in wl.params]
        pm = [q.astype(np.float64) for q in wl.params]
        pp[i][r, c] += h
        pm[i][r, c] -= h
        num = np.sum(dy * (_fwd(wl, params=pp)[0] - _fwd(wl, params=pm)[0])) / (2 * h)
        check(num, dparams[i][r, c], (names[i], r, c))


def test_packed_equals_each_sample_alone():
    wl = _tiny(1)
    y, caches = _fwd(wl)
    dy = wl.dy.astype(np.float64)
    dx_img, dx_seq, dparams = O.stage_bwd(wl.layers, wl.params, wl.batch, caches, dy)
    acc = [np.zeros_like(g) for g in dparams]
    cu = wl.batch.seq.cu_seqlens
    for s, (k, t) in enumerate(wl.batch.samples):
        b1 = W.batch_from_samples([(k, t)], img_tokens=64)
        xi = wl.x_img[64 * s:64 * (s + 1)]
        xs = wl.x_seq[cu[s]:cu[s + 1]]
        y1, c1 = O.stage_fwd(wl.layers, wl.params, b1, xi, xs)
        assert np.max(np.abs(y1 - y[cu[s]:cu[s + 1]])) < 1e-12
        gi, gs, gp = O.stage_bwd(wl.layers, wl.params, b1, c1, dy[cu[s]:cu[s + 1]])
        assert np.max(np.abs(gi - dx_img[64 * s:64 * (s + 1)])) < 1e-12
        assert np.max(np.abs(gs - dx_seq[cu[s]:cu[s + 1]])) < 1e-12
        for a, g in zip(acc, gp):
            a += g
    for a, g in zip(acc, dparams):
        assert np.max(np.abs(a - g)) < 1e-10 * max(1.0, np.max(np.abs(g)))


def test_causality_and_segment_isolation():
    wl = _tiny(2)
    y, caches = _fwd(wl)
    cu = wl.batch.seq.cu_seqlens
    # perturb the last text token of sample 0: earlier rows of sample 0 and all of sample 1 unchanged
    xs = wl.x_seq.astype(np.float64).copy()
    t = int(cu[1]) - 1
    xs[t] += _rand(256)
    y2, _ = _fwd(wl, x_seq=xs)
    assert np.array_equal(y2[:t], y[:t]) and np.array_equal(y2[cu[1]:], y[cu[1]:])
    assert np.any(y2[t] != y[t])
    # perturb one patch of image 1: every row of sample 1 may change (image rows come first and the
    # image is bidirectional), sample 0 must not
    xi = wl.x_img.astype(np.float64).copy()
    xi[64 + 40] += _rand(192)          # not a constant shift: LayerNorm removes those
    y3, _ = _fwd(wl, x_img=xi)
    assert np.array_equal(y3[:cu[1]], y[:cu[1]])
    assert np.all(np.any(y3[cu[1]:cu[1] + 64] != y[cu[1]:cu[1] + 64], axis=1))
    # backward mirror: dy confined to sample 1 gives zero input gradient on sample 0; under the causal
    # mask dy at one row gives zero dx_seq at later rows of that sample
    dy = np.zeros_like(y)
    r = int(cu[1]) + 64 + 5
    dy[r] = 1.0
    dx_img, dx_seq, _ = O.stage_bwd(wl.layers, wl.params, wl.batch, caches, dy)
    assert np.all(dx_seq[:cu[1]] == 0) and np.all(dx_img[:64] == 0)
    assert np.all(dx_seq[r + 1:] == 0) and np.any(dx_seq[r] != 0)
    assert np.all(np.any(dx_img[64:] != 0, axis=1))


def test_vit_image_isolation_bidirectional():
    L = W.vit_layer(64, 2, 32, 128)
    params = W.draw_params([L], 5)
    batch = W.Batch(W.make_pack([6, 9], W.MASK_BIDIR), None, None, [])
    x = _rand(15, 64)
    y, _ = O.stage_fwd([L], params, batch, x_img=x)
    x2 = x.copy()
    x2[8] += _rand(64)
    y2, _ = O.stage_fwd([L], params, batch, x_img=x2)
    assert np.array_equal(y2[:6], y[:6])
    assert np.all(np.any(y2[6:] != y[6:], axis=1))


def test_linear_in_upstream_gradient():
    wl = _tiny(4)
    _, caches = _fwd(wl)
    dy = wl.dy.astype(np.float64)
    g1 = O.stage_bwd(wl.layers, wl.params, wl.batch, caches, dy)
    g2 = O.stage_bwd(wl.layers, wl.params, wl.batch, caches, -2.5 * dy)
    assert np.max(np.abs(g2[0] + 2.5 * g1[0])) < 1e-10
    assert np.max(np.abs(g2[2][2] + 2.5 * g1[2][2])) < 1e-10


# ---------------------------------------------------------------------------
# second opinion: PyTorch CPU fp64 autograd on a straightforward per-sample module
# ---------------------------------------------------------------------------
def test_stage_against_torch_cpu_autograd():
    torch = pytest.importorskip("torch")
    F = torch.nn.functional
    wl = _tiny(5)
    t64 = lambda a: torch.tensor(np.asarray(a, dtype=np.float64), requires_grad=True)
    P = [t64(p) for p in wl.params]
    x_img, x_seq = t64(wl.x_img), t64(wl.x_seq)
    vit, proj, dec = wl.layers
    outs = []
    cu = wl.batch.seq.cu_seqlens
    for s, (k, t) in enumerate(wl.batch.samples):
        xi = x_img[64 * s:64 * (s + 1)]
        g1, b1, wqkv, bqkv, wo, bo, g2, b2, w1, bb1, w2, bb2 = P[:12]
        n = F.layer_norm(xi, (192,), g1[0], b1[0], vit.norm_eps)
        qkv = (n @ wqkv + bqkv).reshape(64, 3, 3, 64).permute(1, 2, 0, 3)   # [which, head, tok, hd]
        o = F.scaled_dot_product_attention(qkv[0], qkv[1], qkv[2])          # bidirectional
        x1 = xi + o.permute(1, 0, 2).reshape(64, 192) @ wo + bo
        n2 = F.layer_norm(x1, (192,), g2[0], b2[0], vit.norm_eps)
        yv = x1 + F.gelu(n2 @ w1 + bb1) @ w2 + bb2
        pr = yv @ P[12] + P[13]
        xs = torch.cat([pr, x_seq[cu[s] + 64:cu[s + 1]]], dim=0)
        Ls = xs.shape[0]
        r1, wqkv, wo, r2, wgu, wd = P[14:]
        rms = lambda z, g: z * torch.rsqrt((z * z).mean(dim=1, keepdim=True) + dec.norm_eps) * g
        n = rms(xs, r1)
        qkv = (n @ wqkv).reshape(Ls, 3, 4, 64).permute(1, 2, 0, 3)
        inv = 10000.0 ** (-torch.arange(0, 32, dtype=torch.float64) * 2 / 64)
        ang = torch.arange(Ls, dtype=torch.float64)[:, None] * inv[None, :]
        cos, sin = torch.cos(ang), torch.sin(ang)
        rot = lambda z: torch.cat([z[..., :32] * cos - z[..., 32:] * sin,
                                   z[..., 32:] * cos + z[..., :32] * sin], dim=-1)
        o = F.scaled_dot_product_attention(rot(qkv[0]), rot(qkv[1]), qkv[2], is_causal=True)
        x1 = xs + o.permute(1, 0, 2).reshape(Ls, 256) @ wo
        n2 = rms(x1, r2)
        gu = n2 @ wgu
        outs.append(x1 + (F.silu(gu[:, :1024]) * gu[:, 1024:]) @ wd)
    y_t = torch.cat(outs, dim=0)
    y_t.backward(torch.tensor(wl.dy.astype(np.float64)))
    y, caches = _fwd(wl)
    dx_img, dx_seq, dparams = O.stage_bwd(wl.layers, wl.params, wl.batch, caches, wl.dy.astype(np.float64))
    rel = lambda a, b: np.max(np.abs(a - b)) / max(np.max(np.abs(b)), 1e-30)
    assert rel(y, y_t.detach().numpy()) < 1e-11
    assert rel(dx_img, x_img.grad.numpy()) < 1e-10
    assert rel(dx_seq, x_seq.grad.numpy()) < 1e-10
    for g, p in zip(dparams, P):
        assert rel(g, p.grad.numpy()) < 1e-10


def test_variant_stage_against_torch_cpu_autograd():
    """The variants (tanh-GELU encoder, two-layer MLP connector, grouped-query decoder with a QKV
    bias) against PyTorch CPU fp64 autograd, sample by sample."""
    torch = pytest.importorskip("torch")
    F = torch.nn.functional
    wl = W.workload_tiny_variant(6)
    t64 = lambda a: torch.tensor(np.asarray(a, dtype=np.float64), requires_grad=True)
    P = [t64(p) for p in wl.params]
    assert len(P) == 12 + 4 + 7
    x_img, x_seq = t64(wl.x_img), t64(wl.x_seq)
    vit, proj, dec = wl.layers
    outs = []
    cu = wl.batch.seq.cu_seqlens
    for s, (k, t) in enumerate(wl.batch.samples):
        xi = x_img[64 * s:64 * (s + 1)]
        g1, b1, wqkv, bqkv, wo, bo, g2, b2, w1, bb1, w2, bb2 = P[:12]
        n = F.layer_norm(xi, (192,), g1[0], b1[0], vit.norm_eps)
        qkv = (n @ wqkv + bqkv).reshape(64, 3, 3, 64).permute(1, 2, 0, 3)
        o = F.scaled_dot_product_attention(qkv[0], qkv[1], qkv[2])
        x1 = xi + o.permute(1, 0, 2).reshape(64, 192) @ wo + bo
        n2 = F.layer_norm(x1, (192,), g2[0], b2[0], vit.norm_eps)
        yv = x1 + F.gelu(n2 @ w1 + bb1, approximate="tanh") @ w2 + bb2
        wp1, bp1, wp2, bp2 = P[12:16]
        pr = F.gelu(yv @ wp1 + bp1) @ wp2 + bp2
        xs = torch.cat([pr, x_seq[cu[s] + 64:cu[s + 1]]], dim=0)
        Ls = xs.shape[0]
        r1, wqkv, bqkv, wo, r2, wgu, wd = P[16:]
        rms = lambda z, g: z * torch.rsqrt((z * z).mean(dim=1, keepdim=True) + dec.norm_eps) * g
        n = rms(xs, r1)
        qkv = n @ wqkv + bqkv
        q = qkv[:, :256].reshape(Ls, 4, 64).permute(1, 0, 2)
        kk = qkv[:, 256:384].reshape(Ls, 2, 64).permute(1, 0, 2)
        v = qkv[:, 384:].reshape(Ls, 2, 64).permute(1, 0, 2)
        inv = 10000.0 ** (-torch.arange(0, 32, dtype=torch.float64) * 2 / 64)
        ang = torch.arange(Ls, dtype=torch.float64)[:, None] * inv[None, :]
        cos, sin = torch.cos(ang), torch.sin(ang)
        rot = lambda z: torch.cat([z[..., :32] * cos - z[..., 32:] * sin,
                                   z[..., 32:] * cos + z[..., :32] * sin], dim=-1)
        o = F.scaled_dot_product_attention(rot(q), rot(kk).repeat_interleave(2, dim=0),
                                           v.repeat_interleave(2, dim=0), is_causal=True)
        x1 = xs + o.permute(1, 0, 2).reshape(Ls, 256) @ wo
        n2 = rms(x1, r2)
        gu = n2 @ wgu
        outs.append(x1 + (F.silu(gu[:, :1024]) * gu[:, 1024:]) @ wd)
    y_t = torch.cat(outs, dim=0)
    y_t.backward(torch.tensor(wl.dy.astype(np.float64)))
    y, caches = _fwd(wl)
    dx_img, dx_seq, dparams = O.stage_bwd(wl.layers, wl.params, wl.batch, caches, wl.dy.astype(np.float64))
    rel = lambda a, b: np.max(np.abs(a - b)) / max(np.max(np.abs(b)), 1e-30)
    assert rel(y, y_t.detach().numpy()) < 1e-11
    assert rel(dx_img, x_img.grad.numpy()) < 1e-10
    assert rel(dx_seq, x_seq.grad.numpy()) < 1e-10
    for g, p in zip(dparams, P):
        assert rel(g, p.grad.numpy()) < 1e-10


def test_qk_norm_stage_against_torch_cpu_autograd():
    """QK normalisation in the encoder layer and in a grouped-query decoder layer (before the rotary
    embedding) against PyTorch CPU fp64 autograd with the library's own rms_norm, sample by sample."""
    torch = pytest.importorskip("torch")
    F = torch.nn.functional
    wl = W.workload_tiny_qknorm(7)
    t64 = lambda a: torch.tensor(np.asarray(a, dtype=np.float64), requires_grad=True)
    P = [t64(p) for p in wl.params]
    assert len(P) == 14 + 2 + 8
    x_img, x_seq = t64(wl.x_img), t64(wl.x_seq)
    vit, proj, dec = wl.layers
    outs = []
    cu = wl.batch.seq.cu_seqlens
    for s, (k, t) in enumerate(wl.batch.samples):
        xi = x_img[64 * s:64 * (s + 1)]
        g1, b1, wqkv, bqkv, wo, bo, g2, b2, w1, bb1, w2, bb2, gq, gk = P[:14]
        n = F.layer_norm(xi, (192,), g1[0], b1[0], vit.norm_eps)
        qkv = n @ wqkv + bqkv
        heads = lambda z, h: z.reshape(z.shape[0], h, 64).permute(1, 0, 2)
        q = heads(F.rms_norm(qkv[:, :192], (192,), gq[0], vit.norm_eps), 3)
        kk = heads(F.rms_norm(qkv[:, 192:384], (192,), gk[0], vit.norm_eps), 3)
        o = F.scaled_dot_product_attention(q, kk, heads(qkv[:, 384:], 3))
        x1 = xi + o.permute(1, 0, 2).reshape(64, 192) @ wo + bo
        n2 = F.layer_norm(x1, (192,), g2[0], b2[0], vit.norm_eps)
        yv = x1 + F.gelu(n2 @ w1 + bb1) @ w2 + bb2
        pr = yv @ P[14] + P[15]
        xs = torch.cat([pr, x_seq[cu[s] + 64:cu[s + 1]]], dim=0)
        Ls = xs.shape[0]
        r1, wqkv, wo, r2, wgu, wd, gq, gk = P[16:]
        n = F.rms_norm(xs, (256,), r1[0], dec.norm_eps)
        qkv = n @ wqkv
        q = heads(F.rms_norm(qkv[:, :256], (256,), gq[0], dec.norm_eps), 4)
        kk = heads(F.rms_norm(qkv[:, 256:384], (128,), gk[0], dec.norm_eps), 2)
        v = heads(qkv[:, 384:], 2)
        inv = 10000.0 ** (-torch.arange(0, 32, dtype=torch.float64) * 2 / 64)
        ang = torch.arange(Ls, dtype=torch.float64)[:, None] * inv[None, :]
        cos, sin = torch.cos(ang), torch.sin(ang)
        rot = lambda z: torch.cat([z[..., :32] * cos - z[..., 32:] * sin,
                                   z[..., 32:] * cos + z[..., :32] * sin], dim=-1)
        o = F.scaled_dot_product_attention(rot(q), rot(kk).repeat_interleave(2, dim=0),
                                           v.repeat_interleave(2, dim=0), is_causal=True)
        x1 = xs + o.permute(1, 0, 2).reshape(Ls, 256) @ wo
        n2 = F.rms_norm(x1, (256,), r2[0], dec.norm_eps)
        gu = n2 @ wgu
        outs.append(x1 + (F.silu(gu[:, :1024]) * gu[:, 1024:]) @ wd)
    y_t = torch.cat(outs, dim=0)
    y_t.backward(torch.tensor(wl.dy.astype(np.float64)))
    y, caches = _fwd(wl)
    dx_img, dx_seq, dparams = O.stage_bwd(wl.layers, wl.params, wl.batch, caches, wl.dy.astype(np.float64))
    rel = lambda a, b: np.max(np.abs(a - b)) / max(np.max(np.abs(b)), 1e-30)
    assert rel(y, y_t.detach().numpy()) < 1e-11
    assert rel(dx_img, x_img.grad.numpy()) < 1e-10
    assert rel(dx_seq, x_seq.grad.numpy()) < 1e-10
    for g, p in zip(dparams, P):
        assert rel(g, p.grad.numpy()) < 1e-10


def test_qk_norm_with_unit_gains_makes_rows_unit_rms_and_scale_free():
    """With gains of one every normalised q and k row has mean square 1 (up to eps), and scaling the
    columns of W_qkv that produce q and k by any positive factor leaves the stage output unchanged."""
    wl = W.workload_tiny_qknorm(8)
    names = [n for L in wl.layers for n, _, _ in W.param_specs(L)]
    params = [p.astype(np.float64) for p in wl.params]
    for i, n in enumerate(names):
        if n.startswith("qkn_"):
            params[i] = np.ones_like(params[i])
    y, caches = _fwd(wl, params=params)
    for c in (caches[0], caches[2]):
        for z in (c["q"], c["k"]):
            if "cos" in c:
                continue                     # rotated afterwards: norm preserved, checked below
            ms = (z.reshape(z.shape[0], -1) ** 2).mean(axis=1)
            assert np.max(np.abs(ms - 1.0)) < 1e-3
    c = caches[2]
    for z in (c["q"], c["k"]):               # rotation keeps each row's norm
        ms = (z.reshape(z.shape[0], -1) ** 2).mean(axis=1)
        assert np.max(np.abs(ms - 1.0)) < 1e-3
    scaled = [p.copy() for p in params]
    eps_free = [p.copy() for p in params]
    iw = names.index("w_qkv")
    ib = names.index("b_qkv")
    for P in (scaled,):
        P[iw][:, :384] *= 64.0
        P[ib][:, :384] *= 64.0
    eps_free[iw][:, :384] *= 8.0
    eps_free[ib][:, :384] *= 8.0
    y64 = _fwd(wl, params=scaled)[0]
    y8 = _fwd(wl, params=eps_free)[0]
    assert np.max(np.abs(y64 - y8)) < 1e-4 * np.max(np.abs(y8))   # equal but for eps under the root


def test_variant_reductions():
    """A zero QKV bias gives the bias-free decoder layer; the MLP connector with an identity-like
    second map reduces to its first map followed by the activation."""
    wl = W.workload_tiny_variant(2)
    vit, proj, dec = wl.layers
    x = wl.x_seq.astype(np.float64)
    cu, kinds = wl.batch.seq.cu_seqlens, wl.batch.seq.mask_kind
    Pd = [p.astype(np.float64) for p in wl.params[16:]]
    Pd[2] = np.zeros_like(Pd[2])
    y_bias0, _ = O.decoder_layer_fwd(dec, Pd, x, cu, kinds)
    plain = W.decoder_layer(256, 4, 2, 64, 1024, 10000.0)
    y_plain, _ = O.decoder_layer_fwd(plain, Pd[:2] + Pd[3:], x, cu, kinds)
    assert np.array_equal(y_bias0, y_plain)
    xi = wl.x_img.astype(np.float64)
    w1, b1 = wl.params[12].astype(np.float64), wl.params[13].astype(np.float64)
    eye = np.eye(320, 256)
    p, _ = O.projector_fwd(proj, [w1, b1, eye, np.zeros((1, 256))], xi)
    assert np.allclose(p, O.gelu_erf(xi @ w1 + b1)[:, :256], rtol=0, atol=1e-15)


def test_pooling_is_the_averaging_matrix():
    """Average pooling against an explicit [windows x rows] averaging matrix built here; backward is
    its transpose; pool = 1 is the identity; a ragged last window averages what it has."""
    cu = np.array([0, 7, 7, 12, 13])
    x = _rand(13, 5)
    A = np.zeros((0, 13))
    for s in range(4):
        a, b = cu[s], cu[s + 1]
        for r in range(a, b, 3):
            row = np.zeros(13)
            row[r:min(r + 3, b)] = 1.0 / (min(r + 3, b) - r)
            A = np.vstack([A, row])
    assert A.shape[0] == 3 + 0 + 2 + 1
    assert np.allclose(O.pool_fwd(x, cu, 3), A @ x, rtol=0, atol=1e-15)
    dp = _rand(A.shape[0], 5)
    assert np.allclose(O.pool_bwd(dp, cu, 3, 13), A.T @ dp, rtol=0, atol=1e-15)
    assert np.array_equal(O.pool_fwd(x, cu, 1), x)
    assert np.allclose(O.pool_fwd(x, cu, 3)[2], (x[6] + 0) / 1)            # rows 6..6: the 7-row segment's tail


def test_pooled_connector_equals_connector_on_pooled_rows():
    wl = W.workload_tiny_pooled(3)
    proj = wl.layers[1]
    P = [p.astype(np.float64) for p in wl.params[12:14]]
    x = wl.x_img.astype(np.float64)
    y, _ = O.projector_fwd(proj, P, x, wl.batch.img.cu_seqlens)
    assert y.shape[0] == 2 * 17 == len(wl.batch.img_to_seq_row)
    ref = np.stack([x[50 * c + 3 * j:min(50 * c + 3 * j + 3, 50 * (c + 1))].mean(axis=0) for c in range(2) for j in range(17)])
    assert np.allclose(y, ref @ P[0] + P[1], rtol=0, atol=1e-13)


def test_token_merging_is_a_reshape():
    """Concatenating r consecutive rows is the row-major reshape [T, d] -> [T / r, r d] when every
    segment is a multiple of r; the backward is the inverse reshape."""
    cu = np.array([0, 8, 8, 20])
    x = _rand(20, 6)
    m = O.merge_fwd(x, cu, 4)
    assert np.array_equal(m, x.reshape(5, 24))
    dm = _rand(5, 24)
    assert np.array_equal(O.merge_bwd(dm, 4), dm.reshape(20, 6))
    with pytest.raises(AssertionError):
        O.merge_fwd(x, np.array([0, 7, 20]), 4)
