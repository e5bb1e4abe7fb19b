"""The attention kernels' work lists (host logic, no GPU): every (segment, tile, head) exactly once, the
items that share rows together on one XCD, the XCDs evenly loaded."""
import numpy as np
import pytest

import workloads as W


@pytest.fixture(scope="module")
def B():
    from paper_2603_25120_amd import binding
    binding.lib()
    return binding


def expected_items(pack, heads, tile=128):
    out = set()
    for s in range(pack.n_segments):
        a, b = int(pack.cu_seqlens[s]), int(pack.cu_seqlens[s + 1])
        for t0 in range(0, b - a, tile):
            for h in range(heads):
                out.add((a, b - a, t0, int(pack.mask_kind[s]), h))
    return out


def item_work(it, kv_major, tile=128):
    _, length, t0, causal, _ = it
    if not causal:
        return length
    return length - t0 if kv_major else min(length, t0 + tile)


CASES = [("8b", W.workload_dec8b(300, with_data=False).batch.seq, 32, 8, 128),
         ("7b", W.workload_dec7b(200, with_data=False).batch.seq, 32, 32, 128),
         ("vit", W.workload_vit_l(100, with_data=False).batch.img, 16, 16, 64),
         ("one long sample", W.equal_partition_batch(32768, 1).seq, 32, 8, 128),
         ("tiny", W.make_pack([70, 1, 0, 129], W.MASK_CAUSAL), 4, 2, 64),
         ("empty", W.make_pack([], W.MASK_CAUSAL), 4, 4, 64)]


def sublists(entries):
    """Entry pid is item pid // 8 of XCD pid % 8: the eight XCDs' item sequences, padding dropped."""
    per = [entries[x::8] for x in range(8)]
    for sub in per:
        live = sub[:, 1] > 0
        assert not np.any(live[1:] & ~live[:-1])               # padding only at the end of a sub-list
    return [sub[sub[:, 1] > 0] for sub in per]


@pytest.mark.parametrize("name,pack,hq,hkv,hd", CASES, ids=[c[0] for c in CASES])
def test_query_list_covers_everything_once_and_balances(B, name, pack, hq, hkv, hd):
    entries = B.mllm_attn_work_list(pack, False, hq, hkv, hd)
    per = sublists(entries) if len(entries) else [np.zeros((0, 5), np.int32)] * 8
    got = [tuple(int(v) for v in row) for sub in per for row in sub]
    assert len(got) == len(set(got)) and set(got) == expected_items(pack, hq)
    assert len(entries) == 8 * max(len(sub) for sub in per)
    if not got:
        return
    # the XCDs carry about the same work: no XCD above the mean by more than the heaviest run of items
    per_xcd = [sum(item_work(tuple(r), False) for r in sub) for sub in per]
    heaviest_run = max(item_work(it, False) for it in got) * 64
    assert max(per_xcd) <= sum(per_xcd) / 8 + heaviest_run
    if len(got) >= 64:
        assert min(len(sub) for sub in per) > 0


@pytest.mark.parametrize("name,pack,hq,hkv,hd", CASES, ids=[c[0] for c in CASES])
def test_key_list_is_every_tile_once_heaviest_first(B, name, pack, hq, hkv, hd):
    entries = B.mllm_attn_work_list(pack, True, hq, hkv, hd)
    got = [tuple(int(v) for v in row) for row in entries]
    assert len(got) == len(set(got)) and set(got) == expected_items(pack, hkv)       # no padding entries
    work = [item_work(it, True) for it in got]
    assert all(a >= b for a, b in zip(work, work[1:]))
    if got:
        tiles = entries.reshape(-1, hkv, 5)
        assert np.all(tiles[:, :, :4] == tiles[:, :1, :4]) and np.all(tiles[:, :, 4] == np.arange(hkv))


def test_items_that_share_rows_sit_together(B):
    """8B-GQA mix: on every XCD the four query heads of a kv head follow one another on the same tile, and a
    (segment, kv head) occupies one contiguous stretch per run of 16 tiles, heaviest tile first."""
    pack = W.workload_dec8b(300, with_data=False).batch.seq
    for sub in sublists(B.mllm_attn_work_list(pack, False, 32, 8, 128)):
        assert len(sub) % 4 == 0
        quads = sub.reshape(-1, 4, 5)
        assert np.all(quads[:, :, :4] == quads[:, :1, :4])                 # same segment and tile
        assert np.all(quads[:, :, 4] == quads[:, :1, 4] // 4 * 4 + np.arange(4))   # heads 4g .. 4g + 3
        key = quads[:, 0, [0, 4]]                                          # (segment start, first head)
        same = ~np.any(key[1:] != key[:-1], axis=1)
        assert np.all(quads[1:, 0, 2][same] < quads[:-1, 0, 2][same])      # causal: later (heavier) tiles first
