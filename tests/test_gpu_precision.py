"""Precision of the binary16 -> binary32 MMA reduction against the exact sum.

Section V of the paper leaves open how much precision a reduction loses when it is done with
half-precision tensor-core inputs.  This measures it on the real matrix unit, for the kernels of
this library and (on the CPU) for the two ways the paper's text can be read:

  gpu mfma         redux_sum, MMA family, default chain bound (256 iterations)
  gpu mfma long    the same with one block and no chain bound: every accumulator entry is a
                   single binary32 running sum over its whole share of the array
  gpu classic      redux_sum, classic family
  gpu multipass    redux_sum_multipass: groups of 256, binary32 partial sums in memory
  gpu half         redux_sum_multipass with "lit_half": both MMA results rounded to binary16, partial sums stored as
                   binary16 -- what the paper's wording describes when it is taken literally
  gpu comp         redux_sum with "compensated": first MMA with C = 0, row sums added with a two-sum on the vector ALU
  gpu comp long    the same with one block and no chain bound
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
    redux.set_param("lit_half", 0)
    redux.set_param("compensated", 0)


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
        redux.set_param("lit_half", 1)
        res["half"] = redux.sum_multipass(xd)[0].item()
        redux.set_param("lit_half", 0)
        redux.set_variant("mfma")
        redux.set_param("compensated", 1)
        res["comp"] = redux.sum(xd).item()
        redux.set_param("max_chain", 65536)
        redux.set_param("max_grid", 1)
        res["comp long"] = redux.sum(xd).item()
        redux.set_param("max_chain", 256)
        redux.set_param("max_grid", 16384)
        redux.set_param("compensated", 0)
        redux.set_variant("auto")
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
        # compensation: within two roundings of the binary32 result whatever the chain length is
        assert rel["comp"] <= 2 * U32 and rel["comp long"] <= 2 * U32
        # binary16 throughout: of binary16 size while everything fits, infinite (or NaN: inf - inf) once a partial sum does not
        if math.isfinite(res["half"]):
            assert rel["half"] <= 4 * 2.0 ** -11, (dist, lg, rel["half"])
            assert rel["half"] >= rel["multipass"]
        else:
            assert dist != "normal" and sum_abs > 65504
    print("\n%s: |error| / sum|x|   (2^-24 = %.2e)" % (dist, U32))
    names = ["mfma", "mfma long", "comp", "comp long", "classic", "multipass", "half", "replay f32", "replay f16"]
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


def test_binary16_throughout_pins_and_replay(dev):
    """The binary16-throughout form of the level-by-level sum: closed forms with exact partial sums, the overflow at
    65504, and agreement with the numpy replay of the same reading (both round each MMA result and each stored partial
    sum to binary16; the matrix unit adds a row's sixteen products in binary32 in its own order, the replay in numpy's,
    so the two can differ by one binary16 rounding per level where a sum falls next to a rounding boundary)."""
    redux.set_param("lit_half", 1)
    ones = lambda n, v=1.0: torch.full((n,), v, dtype=torch.float16, device=dev)
    assert redux.sum_multipass(ones(65280))[0].item() == 65280.0          # 255 x 256: representable (spacing 32)
    assert redux.sum_multipass(ones(25607))[0].item() == 25600.0          # rounds down (spacing 16)
    assert redux.sum_multipass(ones(65536))[0].item() == math.inf         # 65520 and above round to infinity
    assert redux.sum_multipass(ones(1 << 24))[0].item() == math.inf
    assert redux.sum_multipass(ones(1 << 17, -1.0))[0].item() == -math.inf
    out, levels = redux.sum_multipass(ones(1 << 17, 0.25))
    assert out.item() == 32768.0 and levels == 3                          # same level count as the binary32 form
    g = np.full(256, 8.0, np.float16)
    g[0] = 8.0078125                                                      # the row sum 128.0078125 does not fit binary16
    assert redux.sum_multipass(torch.from_numpy(g).to(dev))[0].item() == 2048.0
    redux.set_param("lit_half", 0)
    assert redux.sum_multipass(torch.from_numpy(g).to(dev))[0].item() == 2048.0078125
    for n, seed in ((300, 1), (4096, 2), (1 << 14, 3), ((1 << 16) + 77, 4)):
        x = workloads.uniform_f16(seed, n)
        redux.set_param("lit_half", 1)
        got = redux.sum_multipass(torch.from_numpy(x).to(dev))[0].item()
        redux.set_param("lit_half", 0)
        want = mr.reduce_tc(x, 16, acc_dtype=np.float32, store_dtype=np.float16, mma_dtype=np.float16)[0]
        exact = float(x.astype(np.float64).sum())
        assert abs(got - want) <= 2 * 2.0 ** -11 * exact, (n, got, want)
        assert abs(got - exact) <= 4 * 2.0 ** -11 * exact
    # the form is for binary16 and m = 16 only
    redux.set_param("lit_half", 1)
    redux.set_param("lit_m", 4)
    with pytest.raises(redux.ReduxError):
        redux.sum_multipass(ones(1000))
    redux.set_param("lit_m", 16)
    with pytest.raises(redux.ReduxError):
        redux.sum_multipass(torch.ones(1000, dtype=torch.int8, device=dev))
    redux.set_param("lit_half", 0)


def test_compensation_gains_nothing_once_chains_are_bounded(dev):
    """|error| in units of the binary32 result's last place, against the exact sum: the bounded chain with its binary64
    cascade is already within one rounding of the output format, so a compensated chain has nothing left to gain; it
    only matters where the chain is not bounded (one block, 2^27 elements).  Run with -s for the table."""
    n = 1 << 27
    print("\n|error| / ulp(binary32 result), n = 2^27")
    print("  dist       default   compensated   one block, unbounded   one block, unbounded, compensated")
    for dist in ("uniform01", "tenth", "normal", "wide"):
        x = make(dist, n, 99)
        _, sum_abs, units, nonfinite = oracle.sum_f16_exact(x)
        assert not nonfinite
        exact = units / float(1 << 24)
        ulp = float(np.spacing(np.float32(abs(exact)))) if exact != 0 else 2.0 ** -149
        xd = torch.from_numpy(x).to(dev)
        redux.set_variant("mfma")
        res = []
        for comp, chain, grid in ((0, 256, 16384), (1, 256, 16384), (0, 65536, 1), (1, 65536, 1)):
            redux.set_param("compensated", comp)
            redux.set_param("max_chain", chain)
            redux.set_param("max_grid", grid)
            res.append(abs(redux.sum(xd).item() - exact) / ulp)
        redux.set_param("compensated", 0)
        redux.set_param("max_chain", 256)
        redux.set_param("max_grid", 16384)
        print("  %-10s %-9.2f %-13.2f %-22.1f %.2f" % (dist, res[0], res[1], res[2], res[3]))
        if dist != "normal" and dist != "wide":              # (cancelling sums: the result's ulp is far below sum|x| * 2^-24)
            assert res[0] <= 1.0 and res[1] <= 1.0           # one rounding of the output
            assert res[3] <= 1.0
        assert res[3] <= res[2] + 0.51
    redux.set_variant("auto")
