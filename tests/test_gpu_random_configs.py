"""Seeded random stage configurations against the fp64 oracle: head geometry, widths, layer kinds,
connector kinds, QK normalisation and ragged segment mixes that the hand-picked cases do not reach (odd segment
lengths, empty segments, single-token samples, text-only and image-only samples, tile tails of
every size).  Every output and every gradient is held to the stated tolerances."""
import dataclasses

import numpy as np
import pytest

import workloads as W

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from tests.gpu_util import GpuStage, compare, oracle_run  # noqa: E402


@pytest.fixture(scope="module")
def B():
    from paper_2603_25120_amd import binding
    binding.lib()
    return binding


def random_case(seed):
    rng = np.random.default_rng(10_000 + seed)
    kind = ["vit", "dec", "stage"][seed % 3]
    hd = int(rng.choice([64, 128]))

    def vit():
        heads = int(rng.integers(1, 5))
        return W.vit_layer(heads * hd, heads, hd, 64 * int(rng.integers(1, 9)),
                           act=int(rng.choice([W.ACT_GELU_ERF, W.ACT_GELU_TANH])))

    def dec(d_in=None):
        hkv = int(rng.integers(1, 4))
        grp = int(rng.choice([1, 2, 4]))
        if d_in is not None:                      # width fixed by the connector: pick heads to match
            hq = d_in // hd
            hkv = int(rng.choice([h for h in range(1, hq + 1) if hq % h == 0]))
        else:
            hq = hkv * grp
        return W.decoder_layer(hq * hd, hq, hkv, hd, 64 * int(rng.integers(1, 12)),
                               float(rng.choice([10000.0, 500000.0])), qkv_bias=int(rng.integers(0, 2)))

    def lengths(n, lo, hi):
        out = [int(v) for v in rng.integers(lo, hi, n)]
        if n > 2 and rng.random() < 0.5:
            out[int(rng.integers(0, n))] = 0      # an empty segment
        if rng.random() < 0.5:
            out.append(1)                         # a single-token segment
        return out

    if kind == "vit":
        layers = [vit()]
        layers += [W.vit_layer(layers[0].d_model, layers[0].n_q_heads, hd, 64 * int(rng.integers(1, 6)))] * int(rng.integers(0, 2))
        batch = W.Batch(W.make_pack(lengths(int(rng.integers(1, 6)), 1, 300), W.MASK_BIDIR), None, None, [])
    elif kind == "dec":
        first = dec()
        layers = [first] + [first] * int(rng.integers(0, 2))
        batch = W.Batch(None, W.make_pack(lengths(int(rng.integers(1, 6)), 1, 400), W.MASK_CAUSAL), None, [])
    else:
        v = vit()
        d_llm = hd * int(rng.integers(1, 5))
        hidden = int(rng.choice([0, 64 * int(rng.integers(1, 6))]))
        reduce = [(0, 0), (2, 0), (3, 0), (0, 2)][(seed // 3) % 4]      # (pool, merge): none, average 2 / 3, concatenate 2
        layers = [v, W.projector_layer(v.d_model, d_llm, d_hidden=hidden, pool=reduce[0], merge=reduce[1]), dec(d_llm)]
        img_tokens = int(rng.choice([16, 40, 96, 130]))
        samples = [(int(rng.integers(0, 3)), int(rng.integers(0, 150))) for _ in range(int(rng.integers(1, 5)))]
        samples = [(k, t) for k, t in samples if k * img_tokens + t > 0] or [(1, 5)]
        if sum(k for k, _ in samples) == 0:
            samples.append((1, 0))                # an image-only sample
        batch = W.batch_from_samples(samples, img_tokens=img_tokens, pool=max(1, reduce[0], reduce[1]))
    if seed % 4 == 1:                             # QK normalisation in every transformer layer of the case
        layers = [l if l.kind == W.LAYER_PROJECTOR else dataclasses.replace(l, qk_norm=1) for l in layers]
    return layers, batch


@pytest.mark.parametrize("seed", range(24))
def test_random_configuration_matches_oracle(B, seed):
    layers, batch = random_case(seed)
    wl = W.make_workload("random", layers, batch, 700 + seed)
    st = GpuStage(B, layers)
    try:
        compare(st, wl, st.run(wl), oracle_run(wl))
    finally:
        st.close()
