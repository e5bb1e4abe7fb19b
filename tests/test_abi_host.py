"""Host-only checks of the C ABI: the library loads, exports every entry point that the header
declares, and rejects bad arguments with the documented status before touching a GPU."""
import ctypes
import os
import re

import numpy as np
import pytest

import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    from paper_2603_25120_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2603_25120_amd import build
        build.build()
    binding.lib()
    return binding


def test_library_exports_every_declared_symbol(B):
    header = open(os.path.join(ROOT, "include", "mllm_stage.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(mllm_[a-z0-9_]+)\s*\(", header))
    assert declared, "no declarations found"
    lib = ctypes.CDLL(B.LIB_PATH)
    for name in sorted(declared):
        assert hasattr(lib, name), name
    assert declared == set(B.EXPORTS)


def test_param_table_matches_the_generator(B):
    for layers in (W.tiny_stage_layers(), W.full_stage_layers(2, 2), [W.dec7b_layer()], [W.vit_l_layer()],
                   W.tiny_variant_layers(), [W.dec_qkvbias_7b_layer()], W.tiny_pooled_layers(), W.tiny_merged_layers(),
                   W.tiny_qknorm_layers(), [W.decoder_layer(256, 4, 2, 64, 512, 1e4, qkv_bias=1, qk_norm=1)]):
        h = B.mllm_stage_create(layers)
        got = [B.mllm_stage_param_info(h, i) for i in range(B.mllm_stage_param_count(h))]
        want = [(n, li, r, c) for li, L in enumerate(layers) for n, r, c in W.param_specs(L)]
        assert got == want
        B.mllm_stage_destroy(h)


def _bad(layer, **kw):
    import copy
    l = copy.copy(layer)
    for k, v in kw.items():
        setattr(l, k, v)
    return l


def test_descriptor_validation(B):
    vit, proj, dec = W.tiny_stage_layers()
    cases = [
        [_bad(dec, head_dim=32, n_q_heads=8, n_kv_heads=8)],       # unsupported head_dim
        [_bad(dec, n_kv_heads=3)],                                 # heads not divisible
        [_bad(dec, d_model=320)],                                  # d_model != heads * head_dim
        [_bad(dec, d_ff=1000)],                                    # width not a multiple of 64
        [vit, dec],                                                # decoder after ViT without a connector
        [dec, vit],                                                # wrong order
        [vit, _bad(proj, d_model=256), dec],                       # widths do not chain
        [_bad(vit, act=W.ACT_SWIGLU)],
        [_bad(dec, has_bias=2)],                                   # decoder: 0, or 1 for a QKV bias
        [vit, _bad(proj, d_ff=100), dec],                          # connector hidden width not a multiple of 64
        [vit, _bad(proj, d_ff=128, act=W.ACT_SWIGLU), dec],        # MLP connector needs a GELU
        [vit, _bad(proj, pool=-1), dec],                           # pooling width out of range
        [vit, _bad(proj, pool=2, merge=2), dec],                   # a connector either pools or merges
        [_bad(dec, qk_norm=2)],                                    # QK normalisation is 0 or 1
        [vit, _bad(proj, qk_norm=1), dec],                         # a connector has none
        [],
    ]
    for layers in cases:
        with pytest.raises(B.MllmError) as e:
            B.mllm_stage_create(layers)
        assert e.value.status == 2, layers


class _P:
    def __init__(self, cu, mk, total=None, longest=None):
        self.cu_seqlens, self.mask_kind = np.asarray(cu, np.int32), np.asarray(mk, np.uint8)
        if total is not None:
            self.total_tokens_override = total
        if longest is not None:
            self.max_seqlen_override = longest


class _Bt:
    def __init__(self, img, seq, rows):
        self.img, self.seq, self.img_to_seq_row = img, seq, rows


def test_batch_validation_statuses(B):
    h = B.mllm_stage_create(W.tiny_stage_layers())
    img = _P([0, 64, 128], [0, 0])
    seq = _P([0, 100, 220], [1, 1])
    rows = np.concatenate([np.arange(0, 64), np.arange(100, 164)]).astype(np.int32)
    assert B.mllm_stage_sizes(h, _Bt(img, seq, rows))[0] > 0
    bad = [
        (_Bt(_P([1, 64, 128], [0, 0]), seq, rows), 4),                    # does not start at 0
        (_Bt(_P([0, 80, 64], [0, 0], total=64), seq, rows), 4),           # decreasing
        (_Bt(img, _P([0, 100, 220], [1, 1], total=221), rows), 4),        # wrong total
        (_Bt(img, _P([0, 100, 220], [1, 2]), rows), 5),                   # mask kind
        (_Bt(img, _P([0, 100, 220], [1, 1], longest=50), rows), 3),       # max_seqlen too small
        (_Bt(img, seq, np.where(rows == 163, 220, rows).astype(np.int32)), 6),   # out of range
        (_Bt(img, seq, rows[::-1].copy()), 6),                            # not increasing
    ]
    for batch, status in bad:
        with pytest.raises(B.MllmError) as e:
            B.mllm_stage_sizes(h, batch)
        assert e.value.status == status
    B.mllm_stage_destroy(h)


def test_fwd_rejects_bad_buffers_before_any_launch(B):
    """NULL / undersized / misaligned buffers are refused on the host (no GPU in this test)."""
    wl = W.workload_tiny(0)
    h = B.mllm_stage_create(wl.layers)
    sb, wb = B.mllm_stage_sizes(h, wl.batch)
    n = B.mllm_stage_param_count(h)
    fake = 0x10000          # never dereferenced: validation fails first
    with pytest.raises(B.MllmError) as e:
        B.mllm_stage_fwd(h, wl.batch, [fake] * (n - 1) + [None], fake, fake, fake, fake, fake, stream=1,
                         saved_bytes=sb, workspace_bytes=wb)
    assert e.value.status == 1
    with pytest.raises(B.MllmError) as e:
        B.mllm_stage_fwd(h, wl.batch, [fake] * n, fake, fake, fake, fake, fake, stream=1,
                         saved_bytes=sb - 1, workspace_bytes=wb)
    assert e.value.status == 7
    with pytest.raises(B.MllmError) as e:
        B.mllm_stage_fwd(h, wl.batch, [fake] * n, fake, fake, fake, fake + 8, fake, stream=1,
                         saved_bytes=sb, workspace_bytes=wb)
    assert e.value.status == 7
    with pytest.raises(B.MllmError) as e:
        B.mllm_stage_bwd(h, wl.batch, [fake] * n, None, fake, fake, fake, [fake] * n, 0, fake, stream=1,
                         saved_bytes=sb, workspace_bytes=wb)
    assert e.value.status == 1
    assert "dy" in B.mllm_last_error()
    B.mllm_stage_destroy(h)


def test_op_argument_checks(B):
    fake = 0x10000
    with pytest.raises(B.MllmError) as e:
        B.mllm_op_gemm(fake, fake, fake, 64, 60, 64, stream=1)
    assert e.value.status == 3
    with pytest.raises(B.MllmError) as e:
        B.mllm_op_gemm(fake, fake, fake, 64, 64, 64, out_fp32=0, accumulate=1, stream=1)
    assert e.value.status == 8
    with pytest.raises(B.MllmError) as e:
        B.mllm_op_norm_fwd(0, fake, fake, None, fake, fake, 4, 64, 1e-5, stream=1)
    assert e.value.status == 1
    for m, f, k in ((100000, 64, 64), (256, 128, 64), (100000, 128, 96)):   # f not a multiple of 128; too few tiles; ragged K
        with pytest.raises(B.MllmError) as e:
            B.mllm_op_gemm_swiglu(fake, fake, fake, fake, m, f, k, stream=1)
        assert e.value.status == 8
    with pytest.raises(B.MllmError) as e:
        B.mllm_op_gemm_swiglu(fake, fake, fake, None, 100000, 128, 64, stream=1)
    assert e.value.status == 1
    for m, f, k in ((256, 256, 64), (100000, 256, 96)):                     # too few tiles; ragged K
        with pytest.raises(B.MllmError) as e:
            B.mllm_op_gemm_swiglu_bwd(fake, fake, fake, fake, m, f, k, stream=1)
        assert e.value.status == 8
    with pytest.raises(B.MllmError) as e:
        B.mllm_op_rope(fake, fake, 4, 64, 0, 2, 64, 10000.0, stream=1)     # 2 heads of 64 do not fit a 64-wide row
    assert e.value.status == 3


def test_sizes_grow_with_tokens_and_are_aligned(B):
    h = B.mllm_stage_create([W.dec8b_layer()])
    prev = (0, 0)
    for budget in (1024, 4096, 16384):
        wl = W.workload_dec8b(300, budget, with_data=False)
        cur = B.mllm_stage_sizes(h, wl.batch)
        assert cur[0] > prev[0] and cur[1] > prev[1]
        assert cur[0] % 256 == 0 and cur[1] % 256 == 0
        prev = cur
    B.mllm_stage_destroy(h)


def test_qk_norm_adds_its_buffers_to_the_sizes(B):
    """QK normalisation keeps a second [T, nq] matrix and two statistics arrays per layer in `saved`
    and one more [T, nq] gradient matrix in the workspace (each rounded up to 256 bytes)."""
    import dataclasses
    base = W.decoder_layer(512, 8, 2, 64, 1024, 10000.0)
    batch = W.Batch(None, W.make_pack([300, 212], W.MASK_CAUSAL), None, [])
    T, nq = 512, (8 + 2 * 2) * 64
    sizes = []
    for layers in ([base, base], [dataclasses.replace(base, qk_norm=1)] * 2):
        h = B.mllm_stage_create(layers)
        sizes.append(B.mllm_stage_sizes(h, batch))
        B.mllm_stage_destroy(h)
    up = lambda v: (v + 255) // 256 * 256
    assert sizes[1][0] - sizes[0][0] == 2 * (up(T * nq * 2) + 2 * up(T * 2 * 4))
    assert sizes[1][1] - sizes[0][1] == up(T * nq * 2)


def test_workload_recipes():
    for seed in range(300, 304):
        s = W.draw_samples_mix8b(seed)
        assert sum(576 * k + t for k, t in s) == 32768
        assert all(0 <= k <= 16 and 0 <= t <= 4096 and 576 * k + t > 0 for k, t in s)
    for seed in range(200, 204):
        s = W.draw_samples_mix7b(seed)
        assert sum(576 * k + t for k, t in s) == 8192
        assert all(0 <= k <= 4 and t <= 2048 for k, t in s)
    wl = W.workload_full_stage(414, 32768, "8b", with_data=False)
    b = wl.batch
    assert b.seq.total_tokens == 32768 and b.img.total_tokens % 576 == 0
    assert np.all(np.diff(b.img_to_seq_row) > 0)
    x = np.array([1.0, 1.0078125, 1.00390625, 1.01171875, 3.14159, -2.71828e-3], dtype=np.float32)
    r = W.bf16_round(x)
    assert r[0] == 1.0 and r[1] == np.float32(1.0078125)       # representable values stay (ulp 2^-7)
    assert r[2] == 1.0 and r[3] == np.float32(1.015625)         # ties go to the even mantissa
    assert np.all(np.abs(r - x) <= np.abs(x) * 2.0 ** -8)
    assert len(W.full_stage_sweep()) == 16


def test_product_never_touches_the_oracle():
    """The oracle is test infrastructure: nothing in the package may import, read or run it."""
    pkg = os.path.join(ROOT, "paper_2603_25120_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f), errors="ignore").read()
                assert "oracle" not in text.lower(), os.path.join(dirpath, f)
    assert "oracle" not in open(os.path.join(ROOT, "workloads.py")).read().replace("oracle's tests", "")
    # and the oracle never imports the product
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith(".py"):
            assert "paper_2603_25120_amd" not in open(os.path.join(ROOT, "oracle", f)).read()


def test_microbatch_beyond_the_addressing_limit_is_refused(B):
    h = B.mllm_stage_create([W.dec8b_layer()])
    ok = W.Batch(None, W.make_pack([37000, 37000], W.MASK_CAUSAL), None, [])      # 74000 x 28672 x 2 B < 4 GiB
    assert B.mllm_stage_sizes(h, ok)[0] > 0
    too_big = W.Batch(None, W.make_pack([40000, 40000], W.MASK_CAUSAL), None, [])
    with pytest.raises(B.MllmError) as e:
        B.mllm_stage_sizes(h, too_big)
    assert e.value.status == 3 and "too large" in str(e.value)
    B.mllm_stage_destroy(h)


def test_pooling_connector_row_count(B):
    """With pool = 3 the connector has ceil(length / 3) rows per encoder segment, and that is how
    many entries img_to_seq_row must have (one more or one fewer entry in range is an error only
    when it breaks the ordering or the range; a NULL table is refused)."""
    wl = W.workload_tiny_pooled(0)
    h = B.mllm_stage_create(wl.layers)
    try:
        assert len(wl.batch.img_to_seq_row) == 2 * 17
        sb, wb = B.mllm_stage_sizes(h, wl.batch)
        plain = B.mllm_stage_create(W.tiny_stage_layers())
        assert sb > 0 and wb > 0
        B.mllm_stage_destroy(plain)
        bad = W.Batch(wl.batch.img, wl.batch.seq, None, wl.batch.samples)
        with pytest.raises(B.MllmError) as e:
            B.mllm_stage_sizes(h, bad)
        assert e.value.status == 1
    finally:
        B.mllm_stage_destroy(h)


def test_merging_connector_needs_segment_multiples(B):
    wl = W.workload_tiny_merged(0)
    h = B.mllm_stage_create(wl.layers)
    try:
        assert len(wl.batch.img_to_seq_row) == 2 * 16
        assert B.mllm_stage_sizes(h, wl.batch)[0] > 0
        odd = W.Batch(W.make_pack([64, 62, 2], W.MASK_BIDIR), wl.batch.seq, wl.batch.img_to_seq_row, [])
        with pytest.raises(B.MllmError) as e:
            B.mllm_stage_sizes(h, odd)
        assert e.value.status == 3
    finally:
        B.mllm_stage_destroy(h)
