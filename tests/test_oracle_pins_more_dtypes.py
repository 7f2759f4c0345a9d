"""Pins for the oracle's bfloat16 / binary32 / 8-bit floating-point sums (no GPU): decodes against
independent libraries (numpy bit views, torch's float8 types), closed forms, exact rational brute force."""
import math
from fractions import Fraction

import numpy as np
import pytest

import oracle
from oracle import BF16, F32, F8E4M3, F8E5M2

torch = pytest.importorskip("torch")


def ref_values(pats, dtype):
    """binary64 values of raw patterns, decoded by numpy / torch (not by the oracle)."""
    if dtype == BF16:
        return (pats.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    if dtype == F32:
        return pats.view(np.float32).astype(np.float64)
    tdt = torch.float8_e4m3fn if dtype == F8E4M3 else torch.float8_e5m2
    return torch.from_numpy(pats.copy()).view(tdt).to(torch.float64).numpy()


def encode(vals, dtype):
    """Raw patterns of exactly representable values (checked by decoding them back)."""
    v = np.asarray(vals, dtype=np.float64)
    if dtype == BF16:
        p = (v.astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)
    elif dtype == F32:
        p = v.astype(np.float32).view(np.uint32)
    else:
        tdt = torch.float8_e4m3fn if dtype == F8E4M3 else torch.float8_e5m2
        p = torch.from_numpy(v).to(tdt).view(torch.uint8).numpy()
    assert np.array_equal(ref_values(p, dtype), v), "value not representable"
    return p


ALL = [BF16, F32, F8E4M3, F8E5M2]


@pytest.mark.parametrize("dtype", [BF16, F8E4M3, F8E5M2])
def test_decode_every_pattern(dtype):
    nbits = 16 if dtype == BF16 else 8
    pats = np.arange(1 << nbits, dtype=np.uint32).astype(np.uint16 if nbits == 16 else np.uint8)
    ref = ref_values(pats, dtype)
    got = np.array([oracle.decode(int(p), dtype) for p in pats])
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], ref[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(ref[~nan]))


def test_decode_f32_patterns():
    rng = np.random.default_rng(1)
    pats = np.concatenate([rng.integers(0, 1 << 32, size=200000, dtype=np.uint64).astype(np.uint32),
                           np.array([0, 1, 0x007fffff, 0x00800000, 0x3f800000, 0x7f7fffff, 0x7f800000, 0xff800000,
                                     0x7fc00000, 0x80000000, 0x80000001], dtype=np.uint32)])
    ref = ref_values(pats, F32)
    got = np.array([oracle.decode(int(p), F32) for p in pats])
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan) and np.array_equal(got[~nan], ref[~nan])


def test_format_constants():
    # fixed by the format definitions
    assert oracle.decode(0x3F80, BF16) == 1.0 and oracle.decode(0x0001, BF16) == 2.0 ** -133
    assert oracle.decode(0x7F7F, BF16) == (2 - 2.0 ** -7) * 2.0 ** 127
    assert oracle.decode(0x38, F8E4M3) == 1.0 and oracle.decode(0x7E, F8E4M3) == 448.0
    assert oracle.decode(0x01, F8E4M3) == 2.0 ** -9 and math.isnan(oracle.decode(0x7F, F8E4M3))
    assert oracle.decode(0x78, F8E4M3) == 256.0                      # no infinity in E4M3
    assert oracle.decode(0x3C, F8E5M2) == 1.0 and oracle.decode(0x7B, F8E5M2) == 57344.0
    assert oracle.decode(0x01, F8E5M2) == 2.0 ** -16 and oracle.decode(0x7C, F8E5M2) == math.inf
    assert math.isnan(oracle.decode(0x7D, F8E5M2))


@pytest.mark.parametrize("dtype", ALL)
@pytest.mark.parametrize("n", [0, 1, 2, 63, 64, 127, 128, 129, 257, 4097, (1 << 20) + 3])
def test_constants_and_ones(dtype, n):
    for c in (1.0, -1.5, 0.5, 0.0078125):
        x = encode(np.full(n, c), dtype)
        for method in ("pairwise", "neumaier"):
            s, a = oracle.sum_any(x, dtype, method)
            assert s == c * n and a == abs(c) * n


@pytest.mark.parametrize("dtype", ALL)
@pytest.mark.parametrize("n", [1, 15, 16, 17, 1000, 100003])
def test_integer_ramp_and_alternation(dtype, n):
    period = 16 if dtype in (F8E4M3, F8E5M2) else 256          # every integer below is exactly representable
    i = np.arange(n)
    x = encode((i % period) + 1.0, dtype) if dtype != F8E5M2 else encode((i % 8) + 1.0, dtype)
    per = period if dtype != F8E5M2 else 8
    q, r = divmod(n, per)
    expect = q * per * (per + 1) // 2 + r * (r + 1) // 2
    assert oracle.sum_any(x, dtype)[0] == float(expect)
    alt = np.full(n, 1.25)
    alt[1::2] = -1.25
    s, a = oracle.sum_any(encode(alt, dtype), dtype)
    assert s == (1.25 if n % 2 else 0.0) and a == 1.25 * n


@pytest.mark.parametrize("dtype", ALL)
@pytest.mark.parametrize("n", list(range(0, 40)) + [64, 129, 300])
def test_brute_force_exact(dtype, n):
    rng = np.random.default_rng(7 * n + dtype)
    if dtype in (BF16, F32):
        raw = (rng.standard_normal(n) * 10.0 ** rng.integers(-3, 4)).astype(np.float32)
        pats = (raw.view(np.uint32) >> 16).astype(np.uint16) if dtype == BF16 else raw.view(np.uint32)
    else:
        pats = rng.integers(0, 256, size=n).astype(np.uint8)
        pats = pats[np.isfinite(ref_values(pats, dtype))]
    vals = ref_values(pats, dtype)
    exact = sum((Fraction(float(v)) for v in vals), Fraction(0))
    exact_abs = sum((abs(Fraction(float(v))) for v in vals), Fraction(0))
    for method in ("pairwise", "neumaier"):
        s, a = oracle.sum_any(pats, dtype, method)
        assert s == math.fsum(vals) or abs(Fraction(s) - exact) <= Fraction(math.ulp(float(exact_abs) + 1e-300)) * 4
        assert abs(Fraction(a) - exact_abs) <= Fraction(math.ulp(float(exact_abs) + 1e-300)) * 4
    if dtype in (F8E4M3, F8E5M2):
        u, ua, scale, nf = oracle.sum_f8_exact(pats, dtype)
        assert not nf and Fraction(u) * Fraction(scale) == exact and Fraction(ua) * Fraction(scale) == exact_abs
        assert Fraction(oracle.sum_any(pats, dtype)[0]) == exact      # small multiples of 2^-16: exact in binary64


@pytest.mark.parametrize("dtype", ALL)
def test_methods_agree_permutation_additivity_segments(dtype):
    rng = np.random.default_rng(dtype)
    n = 200003
    if dtype in (BF16, F32):
        raw = rng.standard_normal(n).astype(np.float32)
        pats = (raw.view(np.uint32) >> 16).astype(np.uint16) if dtype == BF16 else raw.view(np.uint32)
    else:
        pats = rng.integers(0, 256, size=n).astype(np.uint8)
        pats = pats[np.isfinite(ref_values(pats, dtype))]
        n = pats.size
    s, a = oracle.sum_any(pats, dtype)
    s2, a2 = oracle.sum_any(pats, dtype, "neumaier")
    assert abs(s - s2) <= 1e-12 * a and abs(a - a2) <= 1e-12 * a
    assert abs(s - math.fsum(ref_values(pats, dtype))) <= 1e-12 * a
    p = rng.permutation(n)
    assert abs(oracle.sum_any(pats[p], dtype)[0] - s) <= 1e-12 * a
    k = n // 3
    assert abs(oracle.sum_any(pats[:k], dtype)[0] + oracle.sum_any(pats[k:], dtype)[0] - s) <= 1e-12 * a
    nseg, seglen = 37, n // 37
    seg, sega = oracle.sum_segmented_any(pats[: nseg * seglen], nseg, seglen, dtype)
    for j in (0, 5, 36):
        assert (seg[j], sega[j]) == oracle.sum_any(pats[j * seglen:(j + 1) * seglen], dtype)
    if dtype in (F8E4M3, F8E5M2):
        u, ua, scale, _ = oracle.sum_f8_exact(pats, dtype)
        assert s == u * scale and a == ua * scale
        up, _, _, _ = oracle.sum_f8_exact(pats[p], dtype)
        assert up == u


@pytest.mark.parametrize("dtype", [BF16, F32, F8E5M2])
def test_nonfinite(dtype):
    base = encode(np.array([1.0, 2.0, -0.5]), dtype)
    inf = {BF16: 0x7F80, F32: 0x7F800000, F8E5M2: 0x7C}[dtype]
    ninf = {BF16: 0xFF80, F32: 0xFF800000, F8E5M2: 0xFC}[dtype]
    nan = {BF16: 0x7FC0, F32: 0x7FC00000, F8E5M2: 0x7E}[dtype]
    mk = lambda *extra: np.concatenate([base, np.array(extra, dtype=base.dtype)])
    assert oracle.sum_any(mk(inf), dtype)[0] == math.inf
    assert oracle.sum_any(mk(ninf), dtype)[0] == -math.inf
    assert math.isnan(oracle.sum_any(mk(inf, ninf), dtype)[0])
    assert math.isnan(oracle.sum_any(mk(nan), dtype)[0])


def test_e4m3_nan_and_extremes():
    x = np.array([0x38, 0x7F], dtype=np.uint8)
    assert math.isnan(oracle.sum_any(x, F8E4M3)[0])
    u, ua, scale, nf = oracle.sum_f8_exact(x, F8E4M3)
    assert nf and u * scale == 1.0
    big = np.full(1 << 20, 0x7E, dtype=np.uint8)
    assert oracle.sum_any(big, F8E4M3)[0] == 448.0 * (1 << 20)
