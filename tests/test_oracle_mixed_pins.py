"""Pins for the mixed-precision layer schedule and the factor budget (Sec. 4.2, Table 3).

The bit labels and the #Float column come from the paper (tests/golden/table3_mixed_bits.txt); the
layer shapes of Llama3-8B come from Appendix A, Table 7 (tests/golden/table7_ranks.txt)."""
import os

import pytest

from oracle import lords_oracle as onp


def _table3(golden_dir):
    mix, flt = [], {}
    with open(os.path.join(golden_dir, "table3_mixed_bits.txt")) as f:
        for line in f:
            t = line.split()
            if not t or t[0].startswith("#"):
                continue
            if t[0] == "mix":
                mix.append((float(t[1]), float(t[2])))
            else:
                flt[t[1]] = int(t[2])
    return mix, flt


def _llama3_8b_block(golden_dir):
    """The seven linear layers of one block: Q, K, V, O, Up, Gate, Down (Table 7 lists Q/O, K/V, Up/Gate once)."""
    shapes = {}
    with open(os.path.join(golden_dir, "table7_ranks.txt")) as f:
        for line in f:
            t = line.split()
            if t and t[0] == "Llama3-8B":
                shapes[t[1]] = (int(t[2]), int(t[3]))
    return [shapes["Q/O"]] * 2 + [shapes["K/V"]] * 2 + [shapes["Up/Gate"]] * 2 + [shapes["Down"]]


def test_bit_labels_of_table3(golden_dir):
    mix, _ = _table3(golden_dir)
    assert len(mix) == 3
    for label, fraction in mix:
        bits = onp.mixed_schedule(32, fraction)
        assert onp.average_bits(bits) == label
        n4 = int(32 * fraction)
        assert bits == [4] * n4 + [2] * (32 - n4)


def test_schedule_shape_and_extremes():
    assert onp.mixed_schedule(32, 0.0) == [2] * 32
    assert onp.mixed_schedule(32, 1.0) == [4] * 32
    assert onp.mixed_schedule(5, 0.5) == [4, 4, 4, 2, 2]          # 2.5 layers: rounded half up
    assert onp.mixed_schedule(5, 0.3) == [4, 4, 2, 2, 2]          # 1.5 -> 2
    assert onp.mixed_schedule(5, 0.29) == [4, 2, 2, 2, 2]         # 1.45 -> 1
    assert onp.mixed_schedule(3, 0.5, 3, 2) == [3, 3, 2]
    assert onp.mixed_schedule(4, 2.0) == [4] * 4                  # clamped
    for n in (1, 7, 32, 80):
        for fr in (0.0, 0.125, 0.25, 0.5, 0.77, 1.0):
            b = onp.mixed_schedule(n, fr)
            assert len(b) == n and b == sorted(b, reverse=True)   # the wide layers come first
            assert abs(b.count(4) - fr * n) <= 0.5


def test_float_budget_of_table3(golden_dir):
    _, flt = _table3(golden_dir)
    block = _llama3_8b_block(golden_dir)
    factors = 32 * onp.factor_parameters(block, 128)
    blockwise = 32 * sum(N * K // 128 for N, K in block)
    assert round(factors / 2 ** 20) == flt["LowRankFactors"]
    assert round(blockwise / 2 ** 20) == flt["NormalFloat"]
    assert factors < blockwise                                   # the rank is a floor: never above the block-wise budget
    # a dropped term or a transposed shape moves the budget by more than the rounding hides
    assert round(32 * sum(onp.equivalent_rank(N, K, 128) * N for N, K in block) / 2 ** 20) != flt["LowRankFactors"]
