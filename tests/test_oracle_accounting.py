"""Pins for the accounting formulas (App. E) against the paper's Table 7."""
import os

import numpy as np

from oracle import vitcop_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "table7_retention_ratios.txt")


def rows():
    out = []
    for line in open(GOLDEN):
        if line.strip() and not line.startswith("#"):
            f = line.split()
            out.append((float(f[0]), int(f[1]), tuple(float(x) for x in f[2:5])))
    return out


def test_table7_reproduces_named_token_counts_only_with_zero_indexed_layers():
    counts = O.stage_layer_counts(2, 22, 32, zero_indexed=True)
    assert counts == (2, 20, 10)
    printed = O.stage_layer_counts(2, 22, 32, zero_indexed=False)
    assert printed == (1, 20, 11)
    for rate, named, ratios in rows():
        mean = O.mean_retained_tokens(576, ratios, counts)
        assert abs(mean - named) < 0.06, (named, mean)
        assert abs(O.cr_int(576, ratios, counts) - rate / 100.0) < 6e-4
        off = O.mean_retained_tokens(576, ratios, printed)
        assert abs(off - named) > 4.0                     # Eq. 10 as printed misses by 4-8 tokens
        assert abs(ratios[2] - ratios[1] / 5.0) < 1e-4     # pi3 = pi2 / 5 in every column


def test_flops_model():
    assert O.flops_layer(10, 3) == 4 * 100 * 3 + 16 * 10 * 9
    # Eq. 9 collapses to n * FLOPs_layer when nothing is pruned
    full = O.schedule_flops(576, 64, 4096, (1.0, 1.0, 1.0), (2, 20, 10))
    assert np.isclose(full, 32 * O.flops_layer(640, 4096))
    # monotone in every ratio
    a = O.schedule_flops(576, 64, 4096, (0.5, 0.4394, 0.0879), (2, 20, 10))
    b = O.schedule_flops(576, 64, 4096, (0.3, 0.1343, 0.0269), (2, 20, 10))
    assert b < a < full
    assert O.causal_attention_flops(1, 128, 32, 128) == 4 * 128 * 32 * 128 * 129 / 2


def test_config2_schedule_compression():
    # budgets 576 -> 192 @2 -> 128 @8 -> 64 @16 over 32 layers
    lens = [576] * 2 + [192] * 6 + [128] * 8 + [64] * 16
    assert len(lens) == 32
    assert abs((1 - sum(lens) / (32 * 576)) - 0.764) < 5e-4
