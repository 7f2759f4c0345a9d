"""Precision of the binary16 -> binary32 MMA reduction against the exact sum.

Section V of the paper leaves open how much precision a reduction loses when it is done with
half-precision tensor-core inputs.  This measures it on the real matrix unit, for the kernels of
this library and (on the CPU) for the two ways the paper's text can be read:

  gpu mfma         redux_sum, MMA family, default chain bound (256 iterations)
  gpu mfma long    the same with one block and no chain bound: every accumulator entry is a
                   single binary32 running sum over its whole share of the array
  gpu classic      redux_sum, classic family
  gpu multipass    redux_sum_multipass: groups of 256, binary32 partial sums in memory
  replay f32       numpy replay of the published algorithm with binary32 partial sums
  replay f16       the same with the partial sums written back into a binary16 array, as
                   Section IV-B literally says (small n only; it overflows above 65504)

The reference is the oracle's exact 128-bit fixed-point sum.  Errors are reported relative to
sum|x|; run with -s to see the table.

Bound asserted for the default path: every accumulator entry is a chain of at most
2 * max_chain MFMAs, each adding 32 products to the running value, so
|err| <= (2 * max_chain + 32 + 64) * 2^-24 * sum|x|  (first-order bound of recursive summation,
plus the folds), which for max_chain = 256 is 3.7e-5 < 1e-4.
"""
import math

import numpy as np
import pytest

import oracle
from oracle import mma_reduction as mr
from paper_1903_03640_amd import redux, workloads

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

U32 = 2.0 ** -24


def make(dist, n, seed):
    if dist == "uniform01":
        return workloads.uniform_f16(seed, n)
    if dist == "normal":
        return workloads.normal_f16(seed, n)
    if dist == "tenth":
        return np.full(n, 0.1, dtype=np.float16)
    if dist == "wide":                                   # magnitudes log-uniform over 2^-14 .. 2^10, random sign
        u = workloads.uniform_f16(seed, n).astype(np.float64)
        s = workloads.uniform_f16(seed + 1, n, symmetric=True).astype(np.float64)
        return (np.sign(s) * 2.0 ** (24 * u - 14)).astype(np.float16)
    raise ValueError(dist)


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available()
    redux.load()
    torch.cuda.set_device(0)
    yield torch.device("cuda:0")
    redux.set_variant("auto")
    redux.set_param("max_chain", 256)
    redux.set_param("max_grid", 16384)


@pytest.mark.parametrize("dist", ["uniform01", "normal", "tenth", "wide"])
def test_precision_table(dev, dist):
    rows = []
    for lg in (12, 16, 20, 24, 27):
        n = 1 << lg
        x = make(dist, n, 40 + lg)
        _, sum_abs, units, nonfinite = oracle.sum_f16_exact(x)
        assert not nonfinite
        exact = units / float(1 << 24)                   # correctly rounded binary64 of the exact total
        xd = torch.from_numpy(x).to(dev)
        res = {}
        redux.set_variant("mfma")
        res["mfma"] = redux.sum(xd).item()
        redux.set_param("max_chain", 65536)
        redux.set_param("max_grid", 1)
        res["mfma long"] = redux.sum(xd).item()
        redux.set_param("max_chain", 256)
        redux.set_param("max_grid", 16384)
        redux.set_variant("classic")
        res["classic"] = redux.sum(xd).item()
        redux.set_variant("auto")
        res["multipass"] = redux.sum_multipass(xd)[0].item()
        torch.cuda.synchronize()
        if lg <= 20:
            with np.errstate(invalid="ignore", over="ignore"):
                res["replay f32"] = mr.reduce_tc(x, 16, acc_dtype=np.float32)[0]
                res["replay f16"] = mr.reduce_tc(x, 16, acc_dtype=np.float32, store_dtype=np.float16)[0]
        rel = {k: (abs(v - exact) / sum_abs if math.isfinite(v) else math.inf) for k, v in res.items()}
        rows.append((lg, sum_abs, exact, rel))
        # the default path: the derived first-order bound, and the library's stated tolerance
        assert rel["mfma"] <= (2 * 256 + 96) * U32
        assert rel["classic"] <= 1e-4 and rel["multipass"] <= 1e-4
    print("\n%s: |error| / sum|x|   (2^-24 = %.2e)" % (dist, U32))
    names = ["mfma", "mfma long", "classic", "multipass", "replay f32", "replay f16"]
    print("  log2 n  sum|x|      exact sum      " + "".join("%-12s" % k for k in names))
    for lg, sum_abs, exact, rel in rows:
        print("  %-6d  %-10.4g  %-13.6g  " % (lg, sum_abs, exact) +
              "".join("%-12s" % ("%.2e" % rel[k] if k in rel else "-") for k in names))


def test_error_of_final_rounding_only(dev):
    """Small exact cases: when every partial sum is representable in binary32 the result is the exact sum."""
    for n in (1, 100, 4096, 1 << 16):
        x = (np.arange(n) % 7 - 3).astype(np.float16)
        exact = float(np.sum(x.astype(np.float64)))
        xd = torch.from_numpy(x).to(dev)
        for variant in ("mfma", "classic"):
            redux.set_variant(variant)
            assert redux.sum(xd).item() == exact
        redux.set_variant("auto")
        assert redux.sum_multipass(xd)[0].item() == exact


def test_error_vs_chain_length(dev):
    """How long a binary32 accumulator chain may get before it is folded into the binary64 total: one block reads
    2^27 elements (8192 loop iterations), with the fold every `max_chain` iterations.  Every accumulator entry then
    adds at most 2 * max_chain MFMA results in a row; the first-order bound (2 * max_chain + 96) * 2^-24 * sum|x|
    must hold, and the error grows with the chain (run with -s for the table)."""
    n = 1 << 27
    redux.set_variant("mfma")
    redux.set_param("max_grid", 1)
    print("\n|error| / sum|x| by chain length (one block, n = 2^27; 2^-24 = %.2e)" % U32)
    print("  dist       " + "".join("%-11d" % c for c in (1, 4, 16, 64, 256, 1024, 8192)))
    for dist in ("uniform01", "tenth", "normal"):
        x = make(dist, n, 77)
        _, sum_abs, units, nonfinite = oracle.sum_f16_exact(x)
        assert not nonfinite
        exact = units / float(1 << 24)
        xd = torch.from_numpy(x).to(dev)
        rels = []
        for chain in (1, 4, 16, 64, 256, 1024, 8192):
            redux.set_param("max_chain", chain)
            got = redux.sum(xd).item()
            rel = abs(got - exact) / sum_abs
            assert rel <= (2 * chain + 96) * U32, (dist, chain, rel)
            rels.append(rel)
        print("  %-10s " % dist + "".join("%-11s" % ("%.2e" % r) for r in rels))
        assert rels[0] <= 2 * U32                          # folded every iteration: only the final rounding is left
    redux.set_param("max_chain", 256)
    redux.set_param("max_grid", 16384)
