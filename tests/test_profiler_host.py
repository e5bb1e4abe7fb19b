"""Model Profiler, host side (Profiling Engine, "Model Profiler"): the FLOP counts that turn measured
times into throughputs, and the memory tables, checked without a GPU.

Pins: the per-token linear totals of the three layer shapes worked out by hand from their widths
(25.17 M, 404.8 M and 436.2 M forward FLOPs per token); an independent count from the shapes the
library itself reports for its parameter matrices (a row-vector times an [in, out] matrix costs
2 in out FLOPs, so a token's linear FLOPs are twice the number of matrix entries of the stage);
hand-worked attention counts on small segments.
"""
import numpy as np
import pytest

import workloads as W
from paper_2603_25120_amd import profiler as MP


@pytest.fixture(scope="module")
def B():
    from paper_2603_25120_amd import binding
    binding.lib()
    return binding


def test_linear_flops_per_token_hand_totals():
    one = W.Batch(W.make_pack([1], W.MASK_BIDIR), W.make_pack([1], W.MASK_CAUSAL), np.zeros(1, np.int32), [])
    # ViT-L: 2 * 1024 * (3072 + 1024 + 4096) + 2 * 4096 * 1024
    assert MP.stage_fwd_flops([W.vit_l_layer()], one)[0] == 25_165_824
    # 7B: 2 * 4096 * (12288 + 4096 + 22016) + 2 * 11008 * 4096
    assert MP.stage_fwd_flops([W.dec7b_layer()], one)[0] == 404_750_336
    # 8B-GQA: 2 * 4096 * (6144 + 4096 + 28672) + 2 * 14336 * 4096
    assert MP.stage_fwd_flops([W.dec8b_layer()], one)[0] == 436_207_616
    # connector 1024 -> 4096: 2 * 1024 * 4096 per image token
    assert MP.stage_fwd_flops([W.projector_layer(1024, 4096)], one)[0] == 8_388_608


@pytest.mark.parametrize("layers", [[W.vit_l_layer()], [W.dec7b_layer()], [W.dec8b_layer()], W.full_stage_layers(3, 2),
                                    W.tiny_stage_layers(), [W.dec_qkvbias_7b_layer()]])
def test_linear_flops_equal_twice_the_matrix_entries_the_library_reports(B, layers):
    h = B.mllm_stage_create(layers)
    infos = [B.mllm_stage_param_info(h, i) for i in range(B.mllm_stage_param_count(h))]
    B.mllm_stage_destroy(h)
    t_img, t_seq = 7, 11
    batch = W.Batch(W.make_pack([t_img], W.MASK_BIDIR), W.make_pack([t_seq], W.MASK_CAUSAL),
                    np.arange(t_img, dtype=np.int32), [])
    expect = 0
    for name, layer, rows, cols in infos:
        if rows > 1:                                      # a matrix (vectors are biases and gains)
            kind = layers[layer].kind
            tokens = t_seq if kind == W.LAYER_DECODER else t_img
            expect += 2 * rows * cols * tokens
    assert MP.stage_fwd_flops(layers, batch)[0] == expect


def test_attention_flops_hand_worked():
    vit = W.vit_layer(128, 2, 64, 256)
    dec = W.decoder_layer(128, 2, 1, 64, 256, 10000.0)
    # one image of 10 tokens, bidirectional: 100 (query, key) pairs, 4 hd FLOPs per pair and head = 4 * 100 * 2 * 64
    img = W.Batch(W.make_pack([10], W.MASK_BIDIR), None, None, [])
    assert MP.stage_fwd_flops([vit], img)[1] == 51_200
    # causal samples of 10 and 4 tokens: half the squares, 50 + 8 pairs (the model-FLOP convention)
    seq = W.Batch(None, W.make_pack([10, 4], W.MASK_CAUSAL), None, [])
    assert MP.stage_fwd_flops([dec], seq)[1] == 4 * 58 * 2 * 64
    # two segments never see each other: twice one segment, not (2 L)^2
    two = W.Batch(W.make_pack([10, 10], W.MASK_BIDIR), None, None, [])
    assert MP.stage_fwd_flops([vit], two)[1] == 2 * 51_200


def test_memory_tables_from_the_size_queries(B):
    grid = [1.0, 4.0, 16.0]
    ms, act = MP.memory_tables(lambda n: [W.vit_l_layer() for _ in range(n)],
                               lambda x: W.batch_from_samples([(int(x), 1)]), grid)
    per_layer = sum(r * c for _, r, c in W.param_specs(W.vit_l_layer()))
    assert ms == [18.0 * 2 * per_layer, 18.0 * 4 * per_layer]
    # what forward keeps for backward grows with the layers and with the images, and is the number the size query gives
    assert all(act[1][j] > act[0][j] for j in range(3)) and act[0][0] < act[0][1] < act[0][2]
    h = B.mllm_stage_create([W.vit_l_layer()] * 2)
    assert act[0][1] == float(B.mllm_stage_sizes(h, W.batch_from_samples([(4, 1)]))[0])
    B.mllm_stage_destroy(h)
    # per layer of a ViT-L stage and image token: x, n1, qkv (3 d), o, x1, n2, pre (4 d), act (4 d) in bf16 = 32 KiB,
    # plus fp32 statistics and log-sum-exps: 2 * 8 + 16 * 4 bytes
    tokens = 16 * W.IMG_TOKENS
    assert act[1][2] - act[0][2] == pytest.approx(2 * tokens * (16 * 1024 * 2 + 16 + 64), rel=0.01)
