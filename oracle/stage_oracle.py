"""fp64 CPU oracle for the pipeline-stage forward and backward pass.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the HIP
path is checked against.  Only tests, the smoke check and the benchmark's
cpu_baseline leg may import it; the product never does, and it shares no code
with the product.

What it computes (row-vector convention, Y = X.W with W stored [in, out]):

* The work of one pipeline stage on one microbatch (Background and Motivation,
  Fig. 1 caption: the modality encoder sees only visual tokens, the LLM sees
  visual and text tokens; backward follows forward).
* Items are packed along the sequence dimension with batch size 1 (Model
  Profiler, "Memory Profiling").  Attention treats each original instance on
  its own and keeps causal integrity, while linear operations act on the whole
  concatenated sequence (Model Profiler, "Throughput Profiling").
* Encoder -> connector -> LLM order (MLLM Architecture, Section 2.1).

The paper names its layers only by model family, so the layer arithmetic is the
textbook pre-norm transformer: LayerNorm / GELU / biased linear maps for the
ViT encoder layer, RMSNorm / rotary positions (half-split pairing, positions
restart at every sample) / grouped-query attention / SwiGLU for the decoder
layer, a biased linear connector whose rows are scattered into the packed LLM
sequence.  Backward is the hand-derived reverse mode of exactly these formulas.
Variants of the evaluated model families (Evaluation, Table 4) are flags of a
layer: tanh-GELU, a QKV bias in the decoder, a two-layer MLP connector, average
pooling or token merging in front of the connector, RMS normalisation of the
q and k rows.  Every function is pinned in tests/test_oracle_pins.py.

Everything is float64 NumPy.  A BLAS matmul is used as a step for the dense
contractions; attention materialises the score matrix per (segment, head,
block of query rows) -- rows of a softmax are independent, so blocking the
query rows changes no arithmetic.
"""
from __future__ import annotations

import math
from typing import List, Optional, Sequence

import numpy as np
from scipy.special import erf as _erf

LAYER_VIT, LAYER_DECODER, LAYER_PROJECTOR = 0, 1, 2
ACT_GELU_ERF, ACT_GELU_TANH, ACT_SWIGLU = 0, 1, 2
MASK_BIDIR, MASK_CAUSAL = 0, 1

_Q_BLOCK = 1024  # query rows whose scores are held at once


# ---------------------------------------------------------------------------
# normalisation
# ---------------------------------------------------------------------------
def layernorm_fwd(x, gamma, beta, eps):
    """y = (x - mean) / sqrt(var + eps) * gamma + beta, biased variance, per row."""
    mu = x.mean(axis=1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (x - mu) * rstd
    return xhat * gamma + beta, (xhat, rstd)


def layernorm_bwd(dy, cache, gamma):
    xhat, rstd = cache
    dxhat = dy * gamma
    m1 = dxhat.mean(axis=1, keepdims=True)
    m2 = (dxhat * xhat).mean(axis=1, keepdims=True)
    dx = (dxhat - m1 - xhat * m2) * rstd
    dgamma = (dy * xhat).sum(axis=0, keepdims=True)
    dbeta = dy.sum(axis=0, keepdims=True)
    return dx, dgamma, dbeta


def rmsnorm_fwd(x, gamma, eps):
    """y = x / sqrt(mean(x^2) + eps) * gamma, per row."""
    rstd = 1.0 / np.sqrt((x * x).mean(axis=1, keepdims=True) + eps)
    return x * rstd * gamma, (x, rstd)


def rmsnorm_bwd(dy, cache, gamma):
    x, rstd = cache
    xhat = x * rstd
    dxhat = dy * gamma
    m2 = (dxhat * xhat).mean(axis=1, keepdims=True)
    dx = (dxhat - xhat * m2) * rstd
    dgamma = (dy * xhat).sum(axis=0, keepdims=True)
    return dx, dgamma


# ---------------------------------------------------------------------------
# activations
# ---------------------------------------------------------------------------
def gelu_erf(z):
    return 0.5 * z * (1.0 + _erf(z / math.sqrt(2.0)))


def gelu_erf_grad(z):
    return 0.5 * (1.0 + _erf(z / math.sqrt(2.0))) + z * np.exp(-0.5 * z * z) / math.sqrt(2.0 * math.pi)


_TANH_C = math.sqrt(2.0 / math.pi)


def gelu_tanh(z):
    return 0.5 * z * (1.0 + np.tanh(_TANH_C * (z + 0.044715 * z ** 3)))


def gelu_tanh_grad(z):
    u = _TANH_C * (z + 0.044715 * z ** 3)
    t = np.tanh(u)
    return 0.5 * (1.0 + t) + 0.5 * z * (1.0 - t * t) * _TANH_C * (1.0 + 3 * 0.044715 * z * z)


def sigmoid(z):
    return 1.0 / (1.0 + np.exp(-z))


def swiglu_fwd(g, u):
    """SiLU(g) * u with SiLU(z) = z / (1 + exp(-z))."""
    return g * sigmoid(g) * u


def swiglu_bwd(da, g, u):
    s = sigmoid(g)
    dg = da * u * (s + g * s * (1.0 - s))
    du = da * g * s
    return dg, du


# ---------------------------------------------------------------------------
# packed-sequence helpers and rotary positions
# ---------------------------------------------------------------------------
def segment_positions(cu):
    """Position of every packed token inside its own segment (restarts at 0)."""
    cu = np.asarray(cu, dtype=np.int64)
    pos = np.zeros(int(cu[-1]), dtype=np.int64)
    for s in range(len(cu) - 1):
        pos[cu[s]:cu[s + 1]] = np.arange(cu[s + 1] - cu[s])
    return pos


def rope_tables(pos, head_dim, base):
    """cos/sin of pos * base^(-2i/head_dim), i in [0, head_dim/2)."""
    half = head_dim // 2
    inv = base ** (-2.0 * np.arange(half, dtype=np.float64) / head_dim)
    ang = pos.astype(np.float64)[:, None] * inv[None, :]
    return np.cos(ang), np.sin(ang)


def rope_apply(z, cos, sin):
    """Rotate pairs (i, i + head_dim/2) of z [T, H, head_dim] by the row's angle."""
    half = z.shape[2] // 2
    z1, z2 = z[:, :, :half], z[:, :, half:]
    c, s = cos[:, None, :], sin[:, None, :]
    return np.concatenate([z1 * c - z2 * s, z2 * c + z1 * s], axis=2)


def rope_apply_inverse(dz, cos, sin):
    """Transpose (= inverse) of the rotation: rotate by the negative angle."""
    return rope_apply(dz, cos, -sin)


# ---------------------------------------------------------------------------
# per-instance attention over a packed sequence
# ---------------------------------------------------------------------------
def _visible(mask_kind, q0, q1, L):
    """Boolean [q1-q0, L]: may query row (q0+i) of a segment see key j?"""
    if mask_kind == MASK_CAUSAL:
        return np.arange(L)[None, :] <= np.arange(q0, q1)[:, None]
    return np.ones((q1 - q0, L), dtype=bool)


def _softmax_rows(scores, vis):
    """Softmax over the visible keys of each row; hidden keys get probability 0."""
    s = np.where(vis, scores, -np.inf)
    s = s - s.max(axis=1, keepdims=True)
    e = np.where(vis, np.exp(s), 0.0)
    return e / e.sum(axis=1, keepdims=True)


def attention_fwd(q, k, v, cu, mask_kind, return_lse=False):
    """o[t,h] = sum_u softmax_u(q[t,h].k[u,g]/sqrt(hd)) v[u,g] over the keys u of t's own
    segment (all of them, or those at or before t under the causal kind), g = h // (Hq/Hkv)."""
    T, Hq, hd = q.shape
    Hkv = k.shape[1]
    grp = Hq // Hkv
    scale = 1.0 / math.sqrt(hd)
    o = np.zeros_like(q)
    lse = np.zeros((Hq, T))
    for s in range(len(cu) - 1):
        a, b = int(cu[s]), int(cu[s + 1])
        L = b - a
        if L == 0:
            continue
        for h in range(Hq):
            g = h // grp
            ks, vs = k[a:b, g, :], v[a:b, g, :]
            for q0 in range(0, L, _Q_BLOCK):
                q1 = min(L, q0 + _Q_BLOCK)
                sc = (q[a + q0:a + q1, h, :] @ ks.T) * scale
                vis = _visible(int(mask_kind[s]), q0, q1, L)
                p = _softmax_rows(sc, vis)
                o[a + q0:a + q1, h, :] = p @ vs
                if return_lse:
                    sm = np.where(vis, sc, -np.inf)
                    mx = sm.max(axis=1)
                    lse[h, a + q0:a + q1] = mx + np.log(np.exp(sm - mx[:, None]).sum(axis=1))
    if return_lse:
        return o, lse
    return o


def attention_bwd(do, q, k, v, cu, mask_kind):
    """Reverse mode of attention_fwd: dS = P * (dP - rowsum(dP * P)), dP = dO.V^T."""
    T, Hq, hd = q.shape
    Hkv = k.shape[1]
    grp = Hq // Hkv
    scale = 1.0 / math.sqrt(hd)
    dq = np.zeros_like(q)
    dk = np.zeros_like(k)
    dv = np.zeros_like(v)
    for s in range(len(cu) - 1):
        a, b = int(cu[s]), int(cu[s + 1])
        L = b - a
        if L == 0:
            continue
        for h in range(Hq):
            g = h // grp
            ks, vs = k[a:b, g, :], v[a:b, g, :]
            for q0 in range(0, L, _Q_BLOCK):
                q1 = min(L, q0 + _Q_BLOCK)
                qs = q[a + q0:a + q1, h, :]
                dos = do[a + q0:a + q1, h, :]
                vis = _visible(int(mask_kind[s]), q0, q1, L)
                p = _softmax_rows((qs @ ks.T) * scale, vis)
                dp = dos @ vs.T
                ds = p * (dp - (dp * p).sum(axis=1, keepdims=True))
                dq[a + q0:a + q1, h, :] = (ds @ ks) * scale
                dk[a:b, g, :] += (ds.T @ qs) * scale
                dv[a:b, g, :] += p.T @ dos
    return dq, dk, dv


# ---------------------------------------------------------------------------
# QK normalisation (layer variant of the evaluated encoders, Evaluation, Table 4: InternViT).  The
# query row of a token (all its heads side by side) and its key row each pass through an RMSNorm
# with a gain vector of their own; in a decoder layer this comes before the rotary embedding.
# ---------------------------------------------------------------------------
def qk_norm_fwd(q, k, gq, gk, eps):
    T = q.shape[0]
    qn, cq = rmsnorm_fwd(q.reshape(T, -1), gq, eps)
    kn, ck = rmsnorm_fwd(k.reshape(T, -1), gk, eps)
    return qn.reshape(q.shape), kn.reshape(k.shape), cq, ck


def qk_norm_bwd(dq, dk, cq, ck, gq, gk):
    T = dq.shape[0]
    dqp, d_gq = rmsnorm_bwd(dq.reshape(T, -1), cq, gq)
    dkp, d_gk = rmsnorm_bwd(dk.reshape(T, -1), ck, gk)
    return dqp.reshape(dq.shape), dkp.reshape(dk.shape), d_gq, d_gk


# ---------------------------------------------------------------------------
# layers
# ---------------------------------------------------------------------------
def _f64(a):
    return np.asarray(a, dtype=np.float64)


def _act_fwd(act, h):
    return gelu_tanh(h) if act == ACT_GELU_TANH else gelu_erf(h)


def _act_grad(act, h):
    return gelu_tanh_grad(h) if act == ACT_GELU_TANH else gelu_erf_grad(h)


def vit_layer_fwd(L, P, x, cu, mask_kind):
    """n = LN1(x); qkv = n.Wqkv + b; o = Attn(q,k,v); x1 = x + o.Wo + bo;
    n2 = LN2(x1); y = x1 + GELU(n2.W1 + b1).W2 + b2."""
    g1, b1n, wqkv, bqkv, wo, bo, g2, b2n, w1, bb1, w2, bb2 = P[:12]
    H, hd = L.n_q_heads, L.head_dim
    T = x.shape[0]
    n1, c1 = layernorm_fwd(x, g1, b1n, L.norm_eps)
    qkv = n1 @ wqkv + bqkv
    q = qkv[:, :H * hd].reshape(T, H, hd)
    k = qkv[:, H * hd:2 * H * hd].reshape(T, H, hd)
    v = qkv[:, 2 * H * hd:].reshape(T, H, hd)
    cq = ck = None
    if L.qk_norm:
        q, k, cq, ck = qk_norm_fwd(q, k, P[12], P[13], L.norm_eps)
    o = attention_fwd(q, k, v, cu, mask_kind).reshape(T, H * hd)
    x1 = x + o @ wo + bo
    n2, c2 = layernorm_fwd(x1, g2, b2n, L.norm_eps)
    h = n2 @ w1 + bb1
    a = _act_fwd(L.act, h)
    y = x1 + a @ w2 + bb2
    return y, dict(c1=c1, n1=n1, q=q, k=k, v=v, o=o, c2=c2, n2=n2, h=h, a=a, cq=cq, ck=ck)


def vit_layer_bwd(L, P, C, dy, cu, mask_kind):
    g1, b1n, wqkv, bqkv, wo, bo, g2, b2n, w1, bb1, w2, bb2 = P[:12]
    T = dy.shape[0]
    H, hd = L.n_q_heads, L.head_dim
    d_b2 = dy.sum(axis=0, keepdims=True)
    d_w2 = C["a"].T @ dy
    da = dy @ w2.T
    dh = da * _act_grad(L.act, C["h"])
    d_b1 = dh.sum(axis=0, keepdims=True)
    d_w1 = C["n2"].T @ dh
    dn2 = dh @ w1.T
    dx1_n, d_g2, d_b2n = layernorm_bwd(dn2, C["c2"], g2)
    dx1 = dy + dx1_n
    d_bo = dx1.sum(axis=0, keepdims=True)
    d_wo = C["o"].T @ dx1
    do = (dx1 @ wo.T).reshape(T, H, hd)
    dq, dk, dv = attention_bwd(do, C["q"], C["k"], C["v"], cu, mask_kind)
    d_qkn = []
    if L.qk_norm:
        dq, dk, d_gq, d_gk = qk_norm_bwd(dq, dk, C["cq"], C["ck"], P[12], P[13])
        d_qkn = [d_gq, d_gk]
    dqkv = np.concatenate([dq.reshape(T, -1), dk.reshape(T, -1), dv.reshape(T, -1)], axis=1)
    d_bqkv = dqkv.sum(axis=0, keepdims=True)
    d_wqkv = C["n1"].T @ dqkv
    dn1 = dqkv @ wqkv.T
    dx_n, d_g1, d_b1n = layernorm_bwd(dn1, C["c1"], g1)
    dx = dx1 + dx_n
    return dx, [d_g1, d_b1n, d_wqkv, d_bqkv, d_wo, d_bo, d_g2, d_b2n, d_w1, d_b1, d_w2, d_b2] + d_qkn


def decoder_layer_fwd(L, P, x, cu, mask_kind):
    """n = RMS1(x); q,k,v = n.[Wq|Wk|Wv] (+ [bq|bk|bv] when the layer has a QKV bias);
    q,k <- RoPE; o = causal GQA attention; x1 = x + o.Wo; n2 = RMS2(x1);
    y = x1 + (SiLU(n2.Wg) * (n2.Wu)).Wd."""
    nb = 7 if L.has_bias else 6
    if L.has_bias:
        g1, wqkv, bqkv, wo, g2, wgu, wd = P[:nb]
    else:
        g1, wqkv, wo, g2, wgu, wd = P[:nb]
        bqkv = 0.0
    Hq, Hkv, hd, f = L.n_q_heads, L.n_kv_heads, L.head_dim, L.d_ff
    T = x.shape[0]
    n1, c1 = rmsnorm_fwd(x, g1, L.norm_eps)
    qkv = n1 @ wqkv + bqkv
    q = qkv[:, :Hq * hd].reshape(T, Hq, hd)
    k = qkv[:, Hq * hd:(Hq + Hkv) * hd].reshape(T, Hkv, hd)
    v = qkv[:, (Hq + Hkv) * hd:].reshape(T, Hkv, hd)
    cq = ck = None
    if L.qk_norm:
        q, k, cq, ck = qk_norm_fwd(q, k, P[nb], P[nb + 1], L.norm_eps)
    cos, sin = rope_tables(segment_positions(cu), hd, L.rope_base)
    q = rope_apply(q, cos, sin)
    k = rope_apply(k, cos, sin)
    o = attention_fwd(q, k, v, cu, mask_kind).reshape(T, Hq * hd)
    x1 = x + o @ wo
    n2, c2 = rmsnorm_fwd(x1, g2, L.norm_eps)
    gu = n2 @ wgu
    gate, up = gu[:, :f], gu[:, f:]
    a = swiglu_fwd(gate, up)
    y = x1 + a @ wd
    return y, dict(c1=c1, n1=n1, q=q, k=k, v=v, o=o, c2=c2, n2=n2, gate=gate, up=up, a=a,
                   cos=cos, sin=sin, cq=cq, ck=ck)


def decoder_layer_bwd(L, P, C, dy, cu, mask_kind):
    nb = 7 if L.has_bias else 6
    if L.has_bias:
        g1, wqkv, _bqkv, wo, g2, wgu, wd = P[:nb]
    else:
        g1, wqkv, wo, g2, wgu, wd = P[:nb]
    Hq, Hkv, hd, f = L.n_q_heads, L.n_kv_heads, L.head_dim, L.d_ff
    T = dy.shape[0]
    d_wd = C["a"].T @ dy
    da = dy @ wd.T
    dgate, dup = swiglu_bwd(da, C["gate"], C["up"])
    dgu = np.concatenate([dgate, dup], axis=1)
    d_wgu = C["n2"].T @ dgu
    dn2 = dgu @ wgu.T
    dx1_n, d_g2 = rmsnorm_bwd(dn2, C["c2"], g2)
    dx1 = dy + dx1_n
    d_wo = C["o"].T @ dx1
    do = (dx1 @ wo.T).reshape(T, Hq, hd)
    dq, dk, dv = attention_bwd(do, C["q"], C["k"], C["v"], cu, mask_kind)
    dq = rope_apply_inverse(dq, C["cos"], C["sin"])
    dk = rope_apply_inverse(dk, C["cos"], C["sin"])
    d_qkn = []
    if L.qk_norm:
        dq, dk, d_gq, d_gk = qk_norm_bwd(dq, dk, C["cq"], C["ck"], P[nb], P[nb + 1])
        d_qkn = [d_gq, d_gk]
    dqkv = np.concatenate([dq.reshape(T, -1), dk.reshape(T, -1), dv.reshape(T, -1)], axis=1)
    d_wqkv = C["n1"].T @ dqkv
    dn1 = dqkv @ wqkv.T
    dx_n, d_g1 = rmsnorm_bwd(dn1, C["c1"], g1)
    dx = dx1 + dx_n
    if L.has_bias:
        return dx, [d_g1, d_wqkv, dqkv.sum(axis=0, keepdims=True), d_wo, d_g2, d_wgu, d_wd] + d_qkn
    return dx, [d_g1, d_wqkv, d_wo, d_g2, d_wgu, d_wd] + d_qkn


def pool_windows(cu, pool):
    """(first row, row count) of every pooling window: consecutive windows of `pool` rows inside
    each segment, the last one of a segment shorter when the length is no multiple."""
    out = []
    for s in range(len(cu) - 1):
        a, b = int(cu[s]), int(cu[s + 1])
        for r in range(a, b, pool):
            out.append((r, min(pool, b - r)))
    return out


def pool_fwd(x, cu, pool):
    """Average pooling at the end of the encoder (Evaluation, audio modality): row j of the result
    is the mean of the encoder rows of window j."""
    return np.stack([x[r:r + n].sum(axis=0) / n for r, n in pool_windows(cu, pool)]) if len(cu) > 1 and cu[-1] > 0 \
        else np.zeros((0, x.shape[1]))


def pool_bwd(dp, cu, pool, rows):
    dx = np.zeros((rows, dp.shape[1]))
    for j, (r, n) in enumerate(pool_windows(cu, pool)):
        dx[r:r + n] = dp[j] / n
    return dx


def merge_fwd(x, cu, merge):
    """Token merging: row j of the result is the concatenation of the encoder rows of window j
    (consecutive windows of `merge` rows; every segment's length is a multiple of `merge`)."""
    out = []
    for r, n in pool_windows(cu, merge):
        assert n == merge, "segment length is no multiple of the merge width"
        out.append(np.concatenate([x[r + q] for q in range(merge)]))
    return np.stack(out) if out else np.zeros((0, x.shape[1] * merge))


def merge_bwd(dm, merge):
    d = dm.shape[1] // merge
    return np.stack([dm[j, q * d:(q + 1) * d] for j in range(dm.shape[0]) for q in range(merge)]) if dm.shape[0] \
        else np.zeros((0, d))


def projector_fwd(L, P, x, cu=None):
    """Connector (MLLM Architecture: a linear projector or a multi-layer perceptron):
    p = x.Wp + bp, or p = act(x.W1 + b1).W2 + b2 when the layer has a hidden width; with
    pool > 1 the encoder rows are average-pooled first."""
    if getattr(L, "merge", 0) > 1:
        merged = merge_fwd(x, cu, L.merge)
        plain = type(L)(**{**L.__dict__, "merge": 0, "d_model": L.d_model * L.merge})
        return projector_fwd(plain, P, merged)
    if getattr(L, "pool", 0) > 1:
        pooled = pool_fwd(x, cu, L.pool)
        plain = type(L)(**{**L.__dict__, "pool": 0})
        y, c = projector_fwd(plain, P, pooled)
        c["rows"] = x.shape[0]
        return y, c
    if L.d_ff:
        w1, b1, w2, b2 = P
        h = x @ w1 + b1
        a = _act_fwd(L.act, h)
        return a @ w2 + b2, dict(x=x, h=h, a=a)
    return x @ P[0] + P[1], dict(x=x)


def projector_bwd(L, P, C, dp, cu=None):
    if getattr(L, "merge", 0) > 1:
        plain = type(L)(**{**L.__dict__, "merge": 0, "d_model": L.d_model * L.merge})
        dmerged, g = projector_bwd(plain, P, C, dp)
        return merge_bwd(dmerged, L.merge), g
    if getattr(L, "pool", 0) > 1:
        plain = type(L)(**{**L.__dict__, "pool": 0})
        dpooled, g = projector_bwd(plain, P, C, dp)
        return pool_bwd(dpooled, cu, L.pool, C["rows"]), g
    if L.d_ff:
        w1, _b1, w2, _b2 = P
        da = dp @ w2.T
        dh = da * _act_grad(L.act, C["h"])
        g = [C["x"].T @ dh, dh.sum(axis=0, keepdims=True), C["a"].T @ dp, dp.sum(axis=0, keepdims=True)]
        return dh @ w1.T, g
    return dp @ P[0].T, [C["x"].T @ dp, dp.sum(axis=0, keepdims=True)]


# ---------------------------------------------------------------------------
# stage = ViT layers -> projector (+ scatter into the packed sequence) -> decoder layers
# ---------------------------------------------------------------------------
def n_params(layer) -> int:
    qkn = 2 if getattr(layer, "qk_norm", 0) else 0
    if layer.kind == LAYER_VIT:
        return 12 + qkn
    if layer.kind == LAYER_DECODER:
        return (7 if layer.has_bias else 6) + qkn
    return 4 if layer.d_ff else 2


def stage_fwd(layers, params, batch, x_img=None, x_seq=None):
    """Run every layer of the stage in order.  Returns (y, cache)."""
    caches = []
    cur_img = _f64(x_img) if x_img is not None else None
    cur_seq = _f64(x_seq).copy() if x_seq is not None else None
    in_seq_space = layers[0].kind == LAYER_DECODER
    pi = 0
    for L in layers:
        P = [_f64(p) for p in params[pi:pi + n_params(L)]]
        pi += n_params(L)
        if L.kind == LAYER_VIT:
            cur_img, c = vit_layer_fwd(L, P, cur_img, batch.img.cu_seqlens, batch.img.mask_kind)
        elif L.kind == LAYER_PROJECTOR:
            proj, c = projector_fwd(L, P, cur_img, batch.img.cu_seqlens)
            cur_seq[np.asarray(batch.img_to_seq_row, dtype=np.int64), :] = proj
            in_seq_space = True
        else:
            cur_seq, c = decoder_layer_fwd(L, P, cur_seq, batch.seq.cu_seqlens, batch.seq.mask_kind)
            in_seq_space = True
        caches.append(c)
    return (cur_seq if in_seq_space else cur_img), caches


def stage_bwd(layers, params, batch, caches, dy):
    """Reverse pass.  Returns (dx_img, dx_seq, dparams) with dparams in interface order;
    dx_seq is zero at rows that the projector overwrote."""
    d = _f64(dy)
    dparams: List[Optional[np.ndarray]] = [None] * len(params)
    offs = []
    pi = 0
    for L in layers:
        offs.append(pi)
        pi += n_params(L)
    dx_seq = None
    dx_img = None
    for li in range(len(layers) - 1, -1, -1):
        L = layers[li]
        P = [_f64(p) for p in params[offs[li]:offs[li] + n_params(L)]]
        C = caches[li]
        if L.kind == LAYER_DECODER:
            d, g = decoder_layer_bwd(L, P, C, d, batch.seq.cu_seqlens, batch.seq.mask_kind)
        elif L.kind == LAYER_PROJECTOR:
            rows = np.asarray(batch.img_to_seq_row, dtype=np.int64)
            dproj = d[rows, :]
            dx_seq = d.copy()
            dx_seq[rows, :] = 0.0
            d, g = projector_bwd(L, P, C, dproj, batch.img.cu_seqlens)
        else:
            d, g = vit_layer_bwd(L, P, C, d, batch.img.cu_seqlens, batch.img.mask_kind)
        for j, gj in enumerate(g):
            dparams[offs[li] + j] = gj
    if layers[0].kind == LAYER_DECODER:
        dx_seq = d
    else:
        dx_img = d
    return dx_img, dx_seq, dparams
