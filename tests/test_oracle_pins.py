"""Pins for the CPU oracle (no GPU).

The paper prints no numeric example (Section V defers all experiments), so the
oracle is pinned to what the mathematics fixes: closed forms, an independent
library's binary16 decode, correctly-rounded and exact rational summation on
small inputs, and invariants of a sum.  Each pin is chosen so that a plausible
mistake (dropped element, wrong sign, wrong exponent bias, off-by-one split in
the pairwise recursion, ...) fails it.
"""
import itertools
import math
from fractions import Fraction

import numpy as np
import pytest

import oracle

F16_METHODS = [oracle.sum_f16, oracle.sum_f16_serial, oracle.sum_f16_neumaier,
               lambda x: oracle.sum_f16_exact(x)[:2]]


def frac_of_f16(a):
    """Exact rational value of each finite float16, via numpy's own decode (independent of the oracle)."""
    return [Fraction(float(v)) for v in np.asarray(a, dtype=np.float16).astype(np.float64)]


def ulp64(v):
    return math.ulp(abs(v)) if v != 0 else 5e-324


# ---- binary16 decode against an independent library -------------------------

def test_decode_all_patterns_match_numpy():
    pats = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    ref = pats.view(np.float16).astype(np.float64)
    got = np.array([oracle.f16_decode(int(p)) for p in pats])
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], ref[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(ref[~nan]))


def test_decode_known_values():
    # values fixed by the IEEE-754 binary16 format itself
    assert oracle.f16_decode(0x3C00) == 1.0
    assert oracle.f16_decode(0xC000) == -2.0
    assert oracle.f16_decode(0x7BFF) == 65504.0
    assert oracle.f16_decode(0x0001) == 2.0 ** -24
    assert oracle.f16_decode(0x0400) == 2.0 ** -14
    assert oracle.f16_decode(0x3555) == 0.333251953125
    assert oracle.f16_decode(0x7C00) == math.inf and oracle.f16_decode(0xFC00) == -math.inf
    assert math.isnan(oracle.f16_decode(0x7E00))


# ---- closed forms -----------------------------------------------------------

@pytest.mark.parametrize("n", list(range(0, 65)) + [1000, 1 << 20])
def test_ones_sum_to_n(n):
    x = np.ones(n, dtype=np.float16)
    for m in F16_METHODS:
        s, sa = m(x)
        assert s == float(n) and sa == float(n)
    xi = np.ones(n, dtype=np.int8)
    assert oracle.sum_i8(xi) == (n, n)


@pytest.mark.parametrize("n", [1 << 26, (1 << 30) + 12345])
def test_ones_sum_to_n_large(n):
    x = np.ones(n, dtype=np.float16)
    assert oracle.sum_f16(x) == (float(n), float(n))
    s, sa, units, nf = oracle.sum_f16_exact(x)
    assert units == n << 24 and s == float(n) and not nf
    del x
    xi = np.ones(n, dtype=np.int8)
    assert oracle.sum_i8(xi) == (n, n)


@pytest.mark.parametrize("c", [0.5, -1.5, 0.0999755859375, 65504.0, 2.0 ** -24, -(2.0 ** -14)])
@pytest.mark.parametrize("n", [0, 1, 7, 129, 4097, (1 << 20) + 3])
def test_constant_arrays(c, n):
    assert float(np.float16(c)) == c            # representable, so c*n is the exact answer
    x = np.full(n, c, dtype=np.float16)
    exact = Fraction(c) * n
    for m in F16_METHODS:
        s, sa = m(x)
        # c*n needs at most 11 + 21 significant bits: exactly representable in binary64
        assert Fraction(s) == exact
        assert Fraction(sa) == abs(exact)


@pytest.mark.parametrize("c", [-128, 127, 0, 1, -1])
@pytest.mark.parametrize("n", [0, 1, 255, 256, 65537, (1 << 24) + 5])
def test_constant_int8(c, n):
    x = np.full(n, c, dtype=np.int8)
    assert oracle.sum_i8(x) == (c * n, abs(c) * n)


@pytest.mark.parametrize("n", [0, 1, 2047, 2048, 2049, 100000, (1 << 22) + 777])
def test_f16_integer_ramp(n):
    # x_i = (i mod 2048) + 1: every value <= 2048 is exact in binary16; sum 1..k = k(k+1)/2
    i = np.arange(n, dtype=np.int64)
    x = ((i % 2048) + 1).astype(np.float16)
    q, r = divmod(n, 2048)
    expect = q * (2048 * 2049 // 2) + r * (r + 1) // 2
    for m in F16_METHODS:
        s, sa = m(x)
        assert s == float(expect) and sa == float(expect)
    assert oracle.sum_f16_exact(x)[2] == expect << 24


@pytest.mark.parametrize("n", [0, 1, 255, 256, 257, 1000, (1 << 22) + 131])
def test_i8_ramp(n):
    i = np.arange(n, dtype=np.int64)
    x = ((i % 256) - 128).astype(np.int8)
    q, r = divmod(n, 256)
    expect = -128 * q + sum(k - 128 for k in range(r))
    assert oracle.sum_i8(x)[0] == expect


@pytest.mark.parametrize("c", [1.0, 0.333251953125, 65504.0])
@pytest.mark.parametrize("n", [1, 2, 101, 4096, 100001])
def test_alternating_sign_cancels(c, n):
    x = np.full(n, c, dtype=np.float16)
    x[1::2] *= -1
    for m in F16_METHODS:
        s, sa = m(x)
        assert s == (c if n % 2 else 0.0)
        assert Fraction(sa) == Fraction(c) * n


# ---- brute force on tiny inputs ---------------------------------------------

def test_all_orderings_small():
    rng = np.random.default_rng(11)
    for n in range(1, 7):
        x = (rng.standard_normal(n) * 100).astype(np.float16)
        exact = sum(frac_of_f16(x), Fraction(0))
        for perm in itertools.permutations(range(n)):
            xp = x[list(perm)]
            for m in F16_METHODS:
                # every partial sum is a small multiple of 2^-24: exact in binary64
                assert Fraction(m(xp)[0]) == exact


@pytest.mark.parametrize("n", range(0, 65))
def test_brute_force_vs_fsum_and_fraction(n):
    rng = np.random.default_rng(1000 + n)
    scale = 10.0 ** rng.integers(-6, 4)
    x = (rng.standard_normal(n) * scale).astype(np.float16)
    vals = x.astype(np.float64)
    exact = sum(frac_of_f16(x), Fraction(0))
    exact_abs = sum((abs(f) for f in frac_of_f16(x)), Fraction(0))
    correctly_rounded = math.fsum(vals)
    assert correctly_rounded == float(exact)
    for m in F16_METHODS:
        s, sa = m(x)
        assert Fraction(s) == exact and Fraction(sa) == exact_abs
    units = oracle.sum_f16_exact(x)[2]
    assert Fraction(units, 1 << 24) == exact
    xi = rng.integers(-128, 128, size=n).astype(np.int8)
    assert oracle.sum_i8(xi) == (sum(int(v) for v in xi), sum(abs(int(v)) for v in xi))


# ---- the four summation methods agree (exactness invariant) ------------------

@pytest.mark.parametrize("n,dist", [(1 << 16, "u"), ((1 << 20) + 17, "n"), ((1 << 24) + 5, "wide")])
def test_methods_agree(n, dist):
    rng = np.random.default_rng(n)
    if dist == "u":
        x = rng.random(n).astype(np.float16)
    elif dist == "n":
        x = rng.standard_normal(n).astype(np.float16)
    else:  # full dynamic range of finite binary16, both signs
        pats = rng.integers(0, 0x7C00, size=n).astype(np.uint16) | (rng.integers(0, 2, size=n).astype(np.uint16) << 15)
        x = pats.view(np.float16)
    s_e, a_e, units, nf = oracle.sum_f16_exact(x)
    assert not nf
    assert s_e == float(Fraction(units, 1 << 24))   # one correct rounding of the exact total
    for m in (oracle.sum_f16, oracle.sum_f16_neumaier):
        s, a = m(x)
        assert abs(s - s_e) <= 2 * ulp64(s_e) + 2 * ulp64(a_e) * 2.0 ** -20
        assert abs(a - a_e) <= 1e-12 * a_e          # sum|x| is not compensated in the serial loops
    # numpy's own float64 pairwise sum: an independent implementation of the same definition
    s_np = float(np.sum(x.astype(np.float64)))
    assert abs(s_np - s_e) <= 1e-12 * a_e


# ---- invariants -----------------------------------------------------------------

def test_permutation_invariance():
    rng = np.random.default_rng(5)
    xi = rng.integers(-128, 128, size=100003).astype(np.int8)
    xf = rng.standard_normal(100003).astype(np.float16)
    ref_i = oracle.sum_i8(xi)
    ref_units = oracle.sum_f16_exact(xf)[2]
    ref_f = oracle.sum_f16(xf)[0]
    for _ in range(5):
        p = rng.permutation(xi.size)
        assert oracle.sum_i8(xi[p]) == ref_i
        assert oracle.sum_f16_exact(xf[p])[2] == ref_units
        assert abs(oracle.sum_f16(xf[p])[0] - ref_f) <= 2 * ulp64(ref_f) + 1e-13


def test_additivity_and_zero_padding():
    rng = np.random.default_rng(6)
    x = rng.standard_normal(50001).astype(np.float16)
    y = (rng.random(7777) * 1000).astype(np.float16)
    ux, uy = oracle.sum_f16_exact(x)[2], oracle.sum_f16_exact(y)[2]
    assert oracle.sum_f16_exact(np.concatenate([x, y]))[2] == ux + uy
    padded = np.concatenate([x, np.zeros(513, dtype=np.float16), -np.zeros(3, dtype=np.float16)])
    assert oracle.sum_f16_exact(padded)[2] == ux
    assert oracle.sum_f16(padded) == oracle.sum_f16(np.concatenate([x, np.zeros(516, dtype=np.float16)]))
    xi = rng.integers(-128, 128, size=4099).astype(np.int8)
    yi = rng.integers(-128, 128, size=17).astype(np.int8)
    assert oracle.sum_i8(np.concatenate([xi, yi]))[0] == oracle.sum_i8(xi)[0] + oracle.sum_i8(yi)[0]
    assert oracle.sum_i8(np.concatenate([xi, np.zeros(100, np.int8)])) == oracle.sum_i8(xi)


def test_pairwise_split_covers_every_element():
    # a single non-zero at each position of an array longer than the serial base case:
    # a wrong split (dropped or doubled element) shows up at some position
    for n in (129, 257, 300, 1025):
        for pos in list(range(0, n, 7)) + [n - 1, n // 2, n // 2 - 1, 127, 128]:
            x = np.zeros(n, dtype=np.float16)
            x[pos] = 3.0
            assert oracle.sum_f16(x) == (3.0, 3.0)


@pytest.mark.parametrize("nseg,seglen", [(0, 5), (5, 0), (1, 1), (7, 13), (33, 512), (16, 4096), (3, 5000)])
def test_segmented_equals_per_segment(nseg, seglen):
    rng = np.random.default_rng(nseg * 100003 + seglen)
    x = rng.standard_normal(nseg * seglen).astype(np.float16)
    s, sa = oracle.sum_segmented_f16(x, nseg, seglen)
    assert s.shape == (nseg,)
    for k in range(nseg):
        assert (s[k], sa[k]) == oracle.sum_f16(x[k * seglen:(k + 1) * seglen])
        exact = sum(frac_of_f16(x[k * seglen:(k + 1) * seglen]), Fraction(0)) if seglen <= 512 else None
        if exact is not None:
            assert Fraction(float(s[k])) == exact
    if nseg and seglen:
        assert abs(float(np.sum(s)) - oracle.sum_f16(x)[0]) <= 1e-9
    xi = rng.integers(-128, 128, size=nseg * seglen).astype(np.int8)
    si, sai = oracle.sum_segmented_i8(xi, nseg, seglen)
    assert np.array_equal(si, xi.reshape(nseg, seglen).astype(np.int64).sum(axis=1)) if nseg and seglen else np.all(si == 0)
    assert int(si.sum()) == oracle.sum_i8(xi)[0]


# ---- IEEE special values -----------------------------------------------------------

def test_nonfinite_semantics():
    base = np.array([1.0, 2.0, -0.5], dtype=np.float16)
    inf, nan = np.float16(np.inf), np.float16(np.nan)
    for m in (oracle.sum_f16, oracle.sum_f16_serial, oracle.sum_f16_neumaier):
        assert m(np.append(base, inf))[0] == math.inf
        assert m(np.append(base, -inf))[0] == -math.inf
        assert math.isnan(m(np.append(base, [inf, -inf]))[0])
        assert math.isnan(m(np.append(base, nan))[0])
        assert m(np.append(base, [inf, inf]))[0] == math.inf
    s, sa, units, nf = oracle.sum_f16_exact(np.append(base, inf))
    assert nf and units == int(2.5 * (1 << 24))


def test_subnormals_are_not_flushed():
    n = 1 << 20
    x = np.full(n, 2.0 ** -24, dtype=np.float16)          # smallest positive subnormal
    assert oracle.sum_f16(x) == (n * 2.0 ** -24, n * 2.0 ** -24)
    assert oracle.sum_f16_exact(x)[2] == n


def test_extremes_do_not_overflow():
    n = 1 << 20
    x = np.full(n, 65504.0, dtype=np.float16)
    assert oracle.sum_f16(x)[0] == 65504.0 * n
    x[::2] = -65504.0
    assert oracle.sum_f16(x) == (0.0, 65504.0 * n)


# ---- many-core form: contiguous chunks, one thread each, combined in chunk order ---------------------------

CHUNKS = [1, 2, 3, 7, 8, 64, 1000]


@pytest.mark.parametrize("chunks", CHUNKS)
def test_chunked_closed_forms_are_exact(chunks):
    """Closed forms whose every partial sum is representable: the chunked sums must be exact, and equal to the
    128-bit fixed-point sum."""
    for n in (0, 1, 5, 63, 1000, (1 << 20) + 3):
        ones = np.ones(n, dtype=np.float16)
        assert oracle.sum_f16_chunks(ones, chunks) == (float(n), float(n))
        ramp = ((np.arange(n) % 2048) + 1).astype(np.float16)                  # sum 1..k, all exact in binary16
        q, r = divmod(n, 2048)
        want = q * 2048 * 2049 // 2 + r * (r + 1) // 2
        assert oracle.sum_f16_chunks(ramp, chunks)[0] == float(want)
        assert oracle.sum_f16_chunks(ramp, chunks)[0] == oracle.sum_f16_exact(ramp)[0]
        alt = np.where(np.arange(n) % 2 == 0, 1.5, -1.5).astype(np.float16)
        assert oracle.sum_f16_chunks(alt, chunks) == (1.5 * (n % 2), 1.5 * n)
        i8 = ((np.arange(n) % 256) - 128).astype(np.int8)
        assert oracle.sum_i8_chunks(i8, chunks) == oracle.sum_i8(i8)
        assert oracle.sum_i8_chunks(np.full(n, -128, dtype=np.int8), chunks) == (-128 * n, 128 * n)


@pytest.mark.parametrize("chunks", CHUNKS)
def test_chunks_tile_the_array(chunks):
    """A single non-zero element at every position: a chunk boundary that drops or repeats an element shows."""
    for n in (1, 2, 7, 64, 129, 1001):
        x = np.zeros(n, dtype=np.float16)
        xi = np.zeros(n, dtype=np.int8)
        for i in range(n):
            x[i], xi[i] = 3.0, -7
            assert oracle.sum_f16_chunks(x, chunks) == (3.0, 3.0), (n, i)
            assert oracle.sum_i8_chunks(xi, chunks) == (-7, 7), (n, i)
            x[i], xi[i] = 0.0, 0


@pytest.mark.parametrize("chunks", CHUNKS)
def test_chunked_sum_agrees_with_single_thread_and_exact(chunks):
    rng = np.random.default_rng(chunks)
    for n in (10, 1000, 100003, (1 << 21) + 17):
        for x in (rng.random(n).astype(np.float16), rng.standard_normal(n).astype(np.float16),
                  (rng.standard_normal(n) * 1000).astype(np.float16)):
            s, a = oracle.sum_f16_chunks(x, chunks)
            s1, a1 = oracle.sum_f16(x)
            se, ae = oracle.sum_f16_exact(x)[:2]
            assert abs(s - s1) <= 2 * ulp64(a1) and abs(a - a1) <= 2 * ulp64(a1)
            assert abs(s - se) <= 2 * ulp64(ae) and abs(a - ae) <= 2 * ulp64(ae)
        xi = rng.integers(-128, 128, n, dtype=np.int8)
        assert oracle.sum_i8_chunks(xi, chunks) == (int(xi.astype(np.int64).sum()), int(np.abs(xi.astype(np.int64)).sum()))


def test_chunked_sum_brute_force_against_fractions():
    rng = np.random.default_rng(5)
    for n in (1, 2, 3, 17, 64):
        x = (rng.standard_normal(n) * 8).astype(np.float16)
        want = sum(frac_of_f16(x), Fraction(0))
        for chunks in (1, 2, 5, 64, 100):
            assert Fraction(oracle.sum_f16_chunks(x, chunks)[0]) == want       # small sums of binary16 are exact in binary64


@pytest.mark.parametrize("chunks", [1, 3, 8, 50])
def test_chunked_segmented_equals_single_thread(chunks):
    rng = np.random.default_rng(9)
    for nseg, seglen in ((1, 10), (7, 1), (33, 129), (100, 1000), (5, 0)):
        x = rng.standard_normal(nseg * seglen).astype(np.float16)
        s, a = oracle.sum_segmented_f16_chunks(x, nseg, seglen, chunks)
        s1, a1 = oracle.sum_segmented_f16(x, nseg, seglen)
        assert np.array_equal(s, s1) and np.array_equal(a, a1)


def test_chunk_count_is_checked_and_default_uses_every_thread():
    x = np.ones(100, dtype=np.float16)
    assert oracle.max_threads() >= 1
    assert oracle.sum_f16_chunks(x) == (100.0, 100.0)
    with pytest.raises(RuntimeError):
        oracle.sum_f16_chunks(x, 5000)
    with pytest.raises(RuntimeError):
        oracle.sum_i8_chunks(np.ones(3, dtype=np.int8), -1)
