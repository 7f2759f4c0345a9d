"""Pins for the numpy replay of the paper's algorithm (Section IV-A) and its cost model (Section IV-B)."""
import os
from fractions import Fraction

import math

import numpy as np
import pytest

import oracle
from oracle import mma_reduction as mr

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "cost_model.txt")


@pytest.mark.parametrize("m", [2, 4, 16])
def test_first_mma_gives_row_sums_in_every_column(m):
    rng = np.random.default_rng(m)
    g = rng.integers(-50, 50, size=m * m).astype(np.float64)
    D, Dp = mr.group_reduce(g, m)
    rows = g.reshape(m, m).sum(axis=1)
    for j in range(m):
        assert np.array_equal(D[:, j], rows)          # first worked equation: each column = the m row sums
    assert np.all(Dp == g.sum())                      # second worked equation: every entry = the group total
    assert Dp.shape == (m, m)


def test_fill_order_last_slot_is_last_element():
    m = 4
    g = np.zeros(m * m)
    g[-1] = 7.0                                       # "A[m,m] is the m^2-th element of the group"
    D, _ = mr.group_reduce(g, m)
    assert np.array_equal(D[m - 1], np.full(m, 7.0)) and np.all(D[: m - 1] == 0)


@pytest.mark.parametrize("rows,depth", [(16, 32), (16, 64), (32, 16), (4, 4)])
def test_rectangular_tile(rows, depth):
    rng = np.random.default_rng(rows * depth)
    g = rng.integers(-128, 128, size=rows * depth).astype(np.float64)
    D, Dp = mr.group_reduce(g, rows, depth, cols=16)
    assert D.shape == (rows, 16)
    assert np.array_equal(D[:, 0], g.reshape(rows, depth).sum(axis=1))
    assert np.all(D == D[:, :1]) and np.all(Dp == g.sum())


@pytest.mark.parametrize("m", [2, 4, 16])
def test_zero_padding_of_a_short_group(m):
    rng = np.random.default_rng(99 + m)
    for k in range(0, m * m + 1):
        g = rng.integers(1, 9, size=k).astype(np.float64)
        _, Dp = mr.group_reduce(g, m)
        assert np.all(Dp == g.sum())


@pytest.mark.parametrize("m", [2, 4, 16])
@pytest.mark.parametrize("n", [1, 2, 3, 15, 16, 17, 255, 256, 257, 4095, 4096, 4097, 70000])
def test_hierarchy_reaches_the_plain_sum(m, n):
    rng = np.random.default_rng(n * 31 + m)
    x = rng.standard_normal(n).astype(np.float16)
    got, levels, sizes = mr.reduce_tc(x, m)
    # every partial sum here is a multiple of 2^-24 below 2^29, so binary64 regrouping is exact
    assert Fraction(got) == Fraction(oracle.sum_f16_exact(x)[2], 1 << 24)
    assert levels == mr.expected_levels(n, m * m)
    for a, b in zip(sizes, sizes[1:]):
        assert b == -(-a // (m * m))                  # each level divides the problem by m^2


def test_hierarchy_on_cdna_tile_and_empty_input():
    x = np.arange(1, 5001).astype(np.float16)[:2048]
    got, levels, sizes = mr.reduce_tc(x, 16, 32)
    assert got == 2048 * 2049 / 2 and levels == 2 and sizes == [2048, 4]
    assert mr.reduce_tc(np.zeros(0, np.float16), 16) == (0.0, 0, [])


def test_expected_levels_against_paper_recurrence():
    # T_tc(n) = 5 + T_tc(n/m^2), T_tc(m^2) = 5  =>  levels = log_{m^2} n when n is a power of m^2
    for m in (2, 4, 16):
        for k in range(1, 6):
            n = (m * m) ** k
            assert mr.expected_levels(n, m * m) == k
            assert mr.expected_levels(n + 1, m * m) == k + 1
            assert abs(mr.model_steps_tc(n, m) - 5 * k) < 1e-9
    assert mr.expected_levels(1 << 30, 256) == 4


def test_cost_model_values_printed_in_the_paper():
    rows = [l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    for kind, arg, val in rows:
        val = float(val)
        if kind == "speedup":
            m = int(arg.split("=")[1])
            assert abs(mr.model_speedup(m) - val) < 1e-12
            assert mr.model_speedup(m) > 1
            for n in (1 << 10, 1 << 20, 1 << 30):
                assert abs(mr.model_steps_classic(n) / mr.model_steps_tc(n, m) - val) < 1e-9
        elif kind == "steps_tc_at_group_size":
            m = int(arg.split("=")[1])
            assert abs(mr.model_steps_tc(m * m, m) - val) < 1e-12
        elif kind == "steps_classic_per_halving":
            assert mr.model_steps_classic(2) == val
        else:
            raise AssertionError(kind)


def test_partial_sums_stored_as_binary16_lose_precision_and_overflow():
    # Section IV-B writes each group's result back into X; if X stays binary16 the partial sums are
    # rounded to 11 bits at every level and saturate to infinity above 65504.
    x = np.random.default_rng(3).random(1 << 16).astype(np.float16)
    exact = oracle.sum_f16(x)[0]
    kept, _, _ = mr.reduce_tc(x, 16, acc_dtype=np.float32)
    assert abs(kept - exact) <= 1e-6 * exact
    rounded, _, _ = mr.reduce_tc(x, 16, acc_dtype=np.float32, store_dtype=np.float16)
    assert 1e-6 * exact < abs(rounded - exact) < 1e-2 * exact
    assert abs(rounded - exact) > 10 * abs(kept - exact)
    big = np.ones(1 << 17, dtype=np.float16)            # true sum 131072 > 65504
    assert mr.reduce_tc(big, 16, acc_dtype=np.float32)[0] == float(1 << 17)
    assert np.isinf(mr.reduce_tc(big, 16, acc_dtype=np.float32, store_dtype=np.float16)[0])


# ---- binary16 throughout: both MMA results and the stored partial sums rounded to binary16 ----------------------

HALF = dict(acc_dtype=np.float32, store_dtype=np.float16, mma_dtype=np.float16)


def test_binary16_throughout_closed_forms_and_overflow():
    """All-ones arrays have exact partial sums as long as they fit binary16: 65280 = 255 groups of 256 is representable
    (spacing 32 between 2^15 and 2^16), so the replay is exact there; 65520 and everything above rounds to infinity
    (the largest finite binary16 is 65504), so n = 65536 ones gives inf, and so does any longer array."""
    assert mr.reduce_tc(np.ones(65280, np.float16), 16, **HALF)[0] == 65280.0
    assert mr.reduce_tc(np.ones(256 * 100 + 7, np.float16), 16, **HALF)[0] == 25600.0    # 25607 rounds to 25600 (spacing 16 from 2^14 to 2^15)
    assert mr.reduce_tc(np.ones(65536, np.float16), 16, **HALF)[0] == math.inf
    assert mr.reduce_tc(np.ones(1 << 20, np.float16), 16, **HALF)[0] == math.inf
    assert mr.reduce_tc(-np.ones(1 << 17, np.float16), 16, **HALF)[0] == -math.inf
    # a group whose row sums are representable but whose total is not: 16 rows of 16 x 2049/2048-ish values
    g = np.full(256, 8.0, np.float16)
    g[0] = 8.0078125                                              # 8 + 2^-7: the row sum 128.0078125 needs 15 bits, rounds to 128
    D, Dp = mr.group_reduce(g, 16, acc_dtype=np.float32, mma_dtype=np.float16)
    assert D[0, 0] == 128.0 and Dp[0, 0] == 2048.0
    D, Dp = mr.group_reduce(g, 16, acc_dtype=np.float32)
    assert D[0, 0] == 128.0078125 and Dp[0, 0] == 2048.0078125


def test_binary16_throughout_error_is_of_binary16_size():
    rng = np.random.default_rng(3)
    for n in (300, 4096, 1 << 14):
        x = rng.random(n).astype(np.float16)
        exact = float(x.astype(np.float64).sum())
        half = mr.reduce_tc(x, 16, **HALF)[0]
        single = mr.reduce_tc(x, 16, acc_dtype=np.float32)[0]
        assert abs(single - exact) <= 4 * 2.0 ** -24 * exact
        assert abs(half - exact) <= 3 * 2.0 ** -11 * exact       # three roundings to 11 bits per level, two levels
        assert abs(half - exact) > abs(single - exact)
