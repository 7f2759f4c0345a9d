"""Numpy replay of the paper's tensor-core reduction (Section IV-A), for tests only.

TEST INFRASTRUCTURE: nothing in the product imports this file, and it shares
no code with the HIP kernels.

The algorithm, in the paper's order and notation:

1. take a group of m*m inputs and place them in A (m x m); B is all ones,
   C is all zeros;
2. first MMA, D = A x B + C: every column of D holds the m row sums of A
   (the first worked matrix equation of Section IV-A);
3. second MMA, D' = B x D + C with the all-ones matrix now on the left:
   every entry of D' is the sum of the m*m inputs (the second worked
   equation);
4. D'[0, 0] is written out as that group's entry of the array of partial sums;
5. the partial sums form a new problem of size n / m**2; repeat until the
   problem fits in one group, whose reduction is the result (the recurrence
   R_tc and its base case).

Readings where the paper is silent: a last group that is not full is padded
with zeros (zero is the identity of + and C is a zero matrix anyway); inputs
fill A row by row, so that A[m-1, m-1] is the m*m-th element of the group as
the text says.  The MMA itself is a library matmul.

A matrix unit whose tile is not square (CDNA4: 16 rows x 32 deep for binary16,
16 x 64 for int8) fits the same algebra with A of shape rows x depth, B all
ones of shape depth x cols, and an all-ones rows' x rows left operand in the
second step; ``rows``/``depth`` below generalise m x m to that.
"""
from __future__ import annotations

import math
from typing import List, Tuple

import numpy as np


def mma(A: np.ndarray, B: np.ndarray, C: np.ndarray) -> np.ndarray:
    """The one primitive of Section IV-A: D = A x B + C."""
    return A @ B + C


def group_reduce(group: np.ndarray, rows: int, depth: int | None = None, cols: int | None = None,
                 acc_dtype=np.float64, mma_dtype=None) -> Tuple[np.ndarray, np.ndarray]:
    """Two-MMA reduction M(x_1 .. x_{rows*depth}) of one group.

    Returns (D, D') where D = A x 1 + 0 and D' = 1 x D + 0.  ``group`` may be
    shorter than rows*depth: the rest of A is zero.

    ``mma_dtype``: the precision the result of an MMA is held in.  Section I-B says both that
    the multiply-accumulate works at half precision and that D can be kept in single precision;
    passing np.float16 replays the first statement literally (each of the two results is
    rounded to binary16 before anything else is done with it), None keeps acc_dtype.
    """
    depth = rows if depth is None else depth
    cols = rows if cols is None else cols
    g = np.asarray(group).reshape(-1)
    if g.size > rows * depth:
        raise ValueError("group of %d does not fit a %dx%d operand" % (g.size, rows, depth))
    A = np.zeros(rows * depth, dtype=acc_dtype)
    A[: g.size] = g.astype(acc_dtype)
    A = A.reshape(rows, depth)                       # row-major fill
    ones_B = np.ones((depth, cols), dtype=acc_dtype)
    zero_C = np.zeros((rows, cols), dtype=acc_dtype)
    D = mma(A, ones_B, zero_C)                       # first MMA: row sums in every column
    if mma_dtype is not None:
        with np.errstate(over="ignore"):
            D = D.astype(mma_dtype).astype(acc_dtype)
    ones_A = np.ones((rows, rows), dtype=acc_dtype)
    with np.errstate(invalid="ignore"):              # (an infinity in D times the ones stays an infinity)
        Dp = mma(ones_A, D, zero_C)                  # second MMA: the group total everywhere
    if mma_dtype is not None:
        with np.errstate(over="ignore"):
            Dp = Dp.astype(mma_dtype).astype(acc_dtype)
    return D, Dp


def reduce_level(x: np.ndarray, rows: int, depth: int | None = None, acc_dtype=np.float64,
                 store_dtype=None, mma_dtype=None) -> np.ndarray:
    """One level: every group of rows*depth inputs is replaced by its D'[0, 0].

    ``store_dtype`` is the type of the array the partial sums are written to.  The paper writes
    them back into X itself (Section IV-B), whose elements are binary16, while noting that D can
    be kept in FP32 (Section I-B); passing np.float16 here replays the first reading, None (keep
    acc_dtype) the second."""
    depth = rows if depth is None else depth
    gsz = rows * depth
    x = np.asarray(x).reshape(-1)
    ngroups = (x.size + gsz - 1) // gsz
    out = np.zeros(ngroups, dtype=acc_dtype)
    for k in range(ngroups):
        _, Dp = group_reduce(x[k * gsz: (k + 1) * gsz], rows, depth, acc_dtype=acc_dtype, mma_dtype=mma_dtype)
        out[k] = Dp[0, 0]
    if store_dtype is not None:
        with np.errstate(over="ignore"):
            out = out.astype(store_dtype).astype(acc_dtype)
    return out


def reduce_tc(x: np.ndarray, rows: int, depth: int | None = None, acc_dtype=np.float64,
              store_dtype=None, mma_dtype=None) -> Tuple[float, int, List[int]]:
    """R_tc(X): apply levels until one value is left.

    Returns (result, number of levels, problem size entering each level).
    An empty input is the empty sum: (0, 0, []).
    """
    x = np.asarray(x).reshape(-1)
    if x.size == 0:
        return acc_dtype(0).item(), 0, []
    sizes: List[int] = []
    cur = x
    while True:
        sizes.append(int(cur.size))
        cur = reduce_level(cur, rows, depth, acc_dtype=acc_dtype, store_dtype=store_dtype, mma_dtype=mma_dtype)
        if cur.size == 1:
            return cur[0].item(), len(sizes), sizes


def expected_levels(n: int, group: int) -> int:
    """ceil(log_group(n)) in exact integer arithmetic (at least one level for n >= 1).

    This is the number of recursion steps of T_tc(n) = 5 + T_tc(n / m**2) with
    group = m**2 (Section IV-B), counted on integers so that there is no
    floating-point logarithm to mis-round.
    """
    if n <= 0:
        return 0
    levels, cap = 1, group
    while cap < n:
        cap *= group
        levels += 1
    return levels


def model_steps_tc(n: int, m: int) -> float:
    """T_tc(n) = 5 log_{m^2} n of the simplified cost model (Section IV-B)."""
    return 5.0 * math.log(n) / math.log(m * m)


def model_steps_classic(n: int) -> float:
    """T(n) = 4 log_2 n of the same model."""
    return 4.0 * math.log2(n)


def model_speedup(m: int) -> float:
    """S = (4/5) log_2(m^2)."""
    return 0.8 * math.log2(m * m)
