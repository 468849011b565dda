"""The FLOP count in the numerator of every TFLOP/s figure (MFU accounting: paper Section 4, MFU definition:
operations per precision over the peak of that precision) pinned to the count the paper prints for its 7B model
(Section 4, "Impact of FP8"), whose block config 3 reproduces: 28 blocks of QKV, attention-out, gate/up and down
projections at hidden size 3584."""
import os

from paper_2512_15306_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "fp8_ops_per_token.txt")
BLOCKS_7B = 28           # transformer blocks of the 7B model whose shapes config 3 carries (28 query heads of 128)


def _golden():
    out = {}
    for line in open(GOLDEN):
        if line.strip() and not line.startswith("#"):
            k, v = line.split()
            out[k] = float(v)
    return out


def test_linear_flops_is_three_gemms_per_linear():
    for cfg in synth.CONFIGS.values():
        by_hand = 0
        for lin in cfg.linears:
            by_hand += 2 * cfg.M * lin.N * lin.K         # forward  Y  = X W^T
            by_hand += 2 * cfg.M * lin.K * lin.N         # dgrad    dX = dY W
            by_hand += 2 * lin.N * lin.K * cfg.M         # wgrad    dW = dY^T X
        assert synth.linear_flops(cfg) == by_hand
        assert synth.quantize_elements(cfg) == sum(cfg.M * l.K + l.N * l.K + cfg.M * l.N for l in cfg.linears)


def test_config_3_reproduces_the_fp8_operations_per_token_of_the_7b_model():
    cfg = synth.CONFIGS[3]
    per_token_per_block = synth.linear_flops(cfg) / cfg.M
    assert per_token_per_block == 6 * (3584 * 4608 + 3584 * 3584 + 3584 * 37888 + 18944 * 3584)
    printed = _golden()["fp8_block_linears"]
    # the paper prints three digits: 39.2e9 means [39.15e9, 39.25e9)
    assert abs(per_token_per_block * BLOCKS_7B - printed) <= 0.05e9 + 1e6, per_token_per_block * BLOCKS_7B
    # a dropped GEMM (4 M K N), a missing linear or a wrong block count would be far outside
    assert abs(per_token_per_block * BLOCKS_7B * 4 / 6 - printed) > 10e9
    assert abs(per_token_per_block * (BLOCKS_7B - 1) - printed) > 1e9


def test_share_of_the_work_that_runs_in_fp8():
    """With the printed split, FP8 at twice the BF16 rate cannot make the whole model more than about 1.8-1.9 times
    faster: what the linears' speed-up can buy is bounded, which is why the benchmark reports the block linears
    on their own."""
    g = _golden()
    total = g["fp8_block_linears"] + g["bf16_lm_head"] + g["bf16_attention"]
    share = g["fp8_block_linears"] / total
    assert 0.90 < share < 0.92
    bound = total / (g["fp8_block_linears"] / 2 + g["bf16_lm_head"] + g["bf16_attention"])
    assert 1.8 < bound < 1.9
