"""The seeded input generators: C fast path against the numpy recipes, ranges, chunkability."""
import numpy as np
import pytest

from paper_1903_03640_amd import workloads as w


def test_mix64_published_vectors():
    # first two outputs of SplitMix64 seeded with 0 (its published reference sequence)
    z = w._z_numpy(1, np.array([0, w.GOLDEN], dtype=np.uint64))
    assert int(z[0]) == 0xE220A8397B1DCDAF and int(z[1]) == 0x6E789E6AA1B965F4


@pytest.mark.parametrize("seed,start,n", [(0, 0, 4099), (2, (1 << 30) + 100, 1000), (4, 12345, 70001)])
def test_uniform_f16_c_equals_numpy(seed, start, n):
    for sym in (False, True):
        a = w.uniform_f16(seed, n, start, symmetric=sym)
        b = w.uniform_f16_numpy(seed, n, start, symmetric=sym)
        assert np.array_equal(a.view(np.uint16), b.view(np.uint16))
        lo = -1.0 if sym else 0.0
        assert a.min() >= lo and a.max() < 1.0


@pytest.mark.parametrize("seed,start,n", [(1, 0, 50001), (1, (1 << 26) - 7, 64)])
def test_normal_f16_c_equals_numpy(seed, start, n):
    a = w.normal_f16(seed, n, start)
    b = w.normal_f16_numpy(seed, n, start)
    assert np.array_equal(a.view(np.uint16), b.view(np.uint16))
    assert np.isfinite(a.astype(np.float64)).all()


@pytest.mark.parametrize("seed,start,n", [(3, 0, 65537), (3, (1 << 30) - 5, 5)])
def test_uniform_i8_c_equals_numpy(seed, start, n):
    assert np.array_equal(w.uniform_i8(seed, n, start), w.uniform_i8_numpy(seed, n, start))


def test_chunks_concatenate_to_the_whole():
    whole = w.uniform_f16(2, 10000)
    parts = np.concatenate([w.uniform_f16(2, 3333, 0), w.uniform_f16(2, 6667, 3333)])
    assert np.array_equal(whole.view(np.uint16), parts.view(np.uint16))
    assert w.checksum(whole) == int(whole.view(np.uint16).astype(np.uint64).sum())
    i8 = w.uniform_i8(3, 1001)
    assert w.checksum(i8) == int(i8.view(np.uint8).astype(np.uint64).sum())


def test_distribution_sanity():
    n = 1 << 20
    u = w.uniform_f16(0, n).astype(np.float64)
    assert abs(u.mean() - 0.5) < 5 * (1 / 12 / n) ** 0.5 + 1e-3
    g = w.normal_f16(1, n).astype(np.float64)
    assert abs(g.mean()) < 5 / n ** 0.5 and abs(g.std() - 1) < 0.01
    assert abs(np.abs(g).mean() - 0.7979) < 0.01
    s = w.uniform_f16(4, n, symmetric=True).astype(np.float64)
    assert abs(s.mean()) < 5 * (1 / 3 / n) ** 0.5 + 1e-3
    i = w.uniform_i8(3, n).astype(np.float64)
    assert abs(i.mean() + 0.5) < 5 * 73.9 / n ** 0.5
    assert i.min() == -128 and i.max() == 127


def test_config_table():
    c = w.CONFIGS
    assert c["C3"].n == (1 << 30) + 12345 and c["C3"].nbytes == 2147508338
    assert c["C5"].nseg * c["C5"].seglen == c["C5"].n == 1 << 28
    assert c["C4"].nbytes == 1 << 30
    x = w.make(c["C1"])
    assert x.dtype == np.float16 and x.size == 1 << 20
    assert np.array_equal(w.make(c["C3"], n=100, start=5).view(np.uint16), w.uniform_f16(2, 100, 5).view(np.uint16))
