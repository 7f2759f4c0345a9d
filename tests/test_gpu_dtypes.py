"""GPU parity for the other element types (bfloat16, binary32, OCP E4M3 / E5M2): same bars as binary16 --
|gpu - oracle| <= 1e-4 * sum|x| -- on flat and segmented sums, both kernel families."""
import math

import numpy as np
import pytest

import oracle
from paper_1903_03640_amd import redux, workloads

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL = 1e-4
# The 8-bit MFMAs keep 14 bits below the largest of the eight products of a lane (measured on MI355X):
# terms more than 2^14 smaller than a neighbour are dropped, at most 7 per 8, so |err| <= 7 * 2^-14 * sum|x|.
TOL_F8_MFMA = 7 * 2.0 ** -14
VARIANTS = ("mfma", "classic", "auto")


def tol_of(kind, variant):
    return TOL_F8_MFMA if (variant == "mfma" and kind in ("e4m3", "e5m2")) else TOL
KINDS = ("bf16", "f32", "e4m3", "e5m2")
ODT = {"bf16": oracle.BF16, "f32": oracle.F32, "e4m3": oracle.F8E4M3, "e5m2": oracle.F8E5M2}


def tdt(kind):
    return {"bf16": torch.bfloat16, "f32": torch.float32, "e4m3": torch.float8_e4m3fn, "e5m2": torch.float8_e5m2}[kind]


def make(kind, seed, n):
    """raw storage patterns (numpy) of n finite values"""
    if kind == "bf16":
        return workloads.normal_bf16(seed, n)
    if kind == "f32":
        return workloads.normal_f32(seed, n).view(np.uint32)
    return workloads.finite_f8(seed, n, kind)


def to_dev(pats, kind, dev, offset_elems=0):
    """device tensor of the right dtype over the given raw patterns, optionally at a misaligned offset"""
    storage = {2: torch.int16, 4: torch.int32, 1: torch.uint8}[pats.dtype.itemsize]
    signed = pats.view({2: np.int16, 4: np.int32, 1: np.uint8}[pats.dtype.itemsize])
    t = torch.from_numpy(np.ascontiguousarray(signed))
    buf = torch.empty(t.numel() + offset_elems, dtype=storage, device=dev)
    buf[offset_elems:].copy_(t)
    return buf[offset_elems:].view(tdt(kind))


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available()
    redux.load()
    torch.cuda.set_device(0)
    yield torch.device("cuda:0")
    redux.set_variant("auto")


@pytest.fixture(autouse=True)
def reset():
    yield
    for name, val in (("unroll", 0), ("max_chain", 256), ("max_grid", 16384), ("seg_parts", 0)):
        redux.set_param(name, val)
    redux.set_variant("auto")


def check(got, pats, kind, variant="classic"):
    want, want_abs = oracle.sum_any(pats, ODT[kind])
    if math.isnan(want):
        assert math.isnan(got)
    elif math.isinf(want):
        assert got == want
    else:
        assert abs(got - want) <= tol_of(kind, variant) * want_abs, (kind, variant, got, want, want_abs)


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("kind", KINDS)
def test_flat_sizes(dev, kind, variant):
    redux.set_variant(variant)
    for n in (0, 1, 3, 4, 5, 15, 16, 17, 63, 64, 65, 255, 256, 257, 1023, 1024, 1025, 4097, 65537, (1 << 20) + 1,
              256 * 8 * 8 * 5 + 3, 3 * (1 << 20) + 777, (1 << 24) + 9):
        pats = make(kind, n % 101, n)
        x = to_dev(pats, kind, dev) if n else torch.empty(0, dtype=tdt(kind), device=dev)
        got = redux.sum(x)
        torch.cuda.synchronize()
        check(got.item(), pats, kind, variant)


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("kind", KINDS)
def test_flat_misaligned_and_launch_shapes(dev, kind, variant):
    redux.set_variant(variant)
    es = {"bf16": 2, "f32": 4, "e4m3": 1, "e5m2": 1}[kind]
    for off in range(1, 16 // es):
        for n in (1, 7, 70001):
            pats = make(kind, off, n)
            got = redux.sum(to_dev(pats, kind, dev, off))
            torch.cuda.synchronize()
            check(got.item(), pats, kind, variant)
    n = 5 * (1 << 20) + 12345
    pats = make(kind, 9, n)
    x = to_dev(pats, kind, dev)
    for unroll in (1, 2, 4, 8):
        for max_chain, max_grid in ((256, 16384), (1, 16384), (65536, 5)):
            redux.set_param("unroll", unroll)
            redux.set_param("max_chain", max_chain)
            redux.set_param("max_grid", max_grid)
            got = redux.sum(x)
            torch.cuda.synchronize()
            check(got.item(), pats, kind, variant)


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("kind", KINDS)
def test_closed_forms(dev, kind, variant):
    redux.set_variant(variant)
    for n in (1, 1000, (1 << 20) + 7, (1 << 24) - 3):
        ones = torch.ones(n, dtype=torch.float32, device=dev).to(tdt(kind))
        got = redux.sum(ones)
        torch.cuda.synchronize()
        assert got.item() == float(n)
        alt = torch.full((n,), 1.5, dtype=torch.float32, device=dev)
        alt[1::2] = -1.5
        got = redux.sum(alt.to(tdt(kind)))
        torch.cuda.synchronize()
        assert got.item() == (1.5 if n % 2 else 0.0)


@pytest.mark.parametrize("variant", VARIANTS)
def test_special_values(dev, variant):
    redux.set_variant(variant)
    for kind, inf, ninf, nan in (("bf16", 0x7F80, 0xFF80, 0x7FC0), ("f32", 0x7F800000, 0xFF800000, 0x7FC00000),
                                 ("e5m2", 0x7C, 0xFC, 0x7E)):
        base = make(kind, 3, 100000)
        for vals, want in (((inf,), math.inf), ((ninf,), -math.inf), ((nan,), math.nan), ((inf, ninf), math.nan)):
            p = base.copy()
            for k, v in enumerate(vals):
                p[(777 + 4097 * k) % p.size] = v
            got = redux.sum(to_dev(p, kind, dev)).item()
            assert (math.isnan(got) if math.isnan(want) else got == want), (kind, vals, got)
    p = make("e4m3", 3, 100000)
    p[4242] = 0x7F                                       # the E4M3 NaN pattern
    assert math.isnan(redux.sum(to_dev(p, "e4m3", dev)).item())
    big = np.full(1 << 20, 0x7E, dtype=np.uint8)         # 448, the largest E4M3 value
    assert redux.sum(to_dev(big, "e4m3", dev)).item() == 448.0 * (1 << 20)
    sub = np.full(1 << 20, 0x01, dtype=np.uint8)         # smallest subnormals of the 8-bit formats
    assert redux.sum(to_dev(sub, "e4m3", dev)).item() == 2.0 ** -9 * (1 << 20)
    assert redux.sum(to_dev(sub, "e5m2", dev)).item() == 2.0 ** -16 * (1 << 20)


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("kind", KINDS)
def test_segmented(dev, kind, variant):
    redux.set_variant(variant)
    for nseg, seglen, parts in ((1, 1, 0), (5, 8, 0), (64, 33, 0), (257, 512, 0), (100, 4099, 0), (3, (1 << 20) + 3, 0),
                                (7, 100003, 8), (2000, 64, 0), (1500, 2048, 0)):
        redux.set_param("seg_parts", parts)
        pats = make(kind, nseg + seglen, nseg * seglen)
        got = redux.sum_segmented(to_dev(pats, kind, dev), nseg, seglen)
        torch.cuda.synchronize()
        want, want_abs = oracle.sum_segmented_any(pats, nseg, seglen, ODT[kind])
        assert np.all(np.abs(got.cpu().numpy().astype(np.float64) - want) <= tol_of(kind, variant) * want_abs), (kind, nseg, seglen)


def test_f8_mfma_alignment_window(dev):
    """What the 8-bit MFMA drops, pinned on a constructed tile: one large value and 31 small ones in one row of A.
    The seven small values that share the large one's lane vanish once they are 2^14 times smaller; the 24 in
    other lanes survive.  The classic family adds all of them."""
    for kind, big_exp in (("e5m2", 15), ("e4m3", 8)):
        idx = [lane * 16 + j for lane in (0, 16, 32, 48) for j in range(8)]      # row 0 of the first MFMA
        for k, dropped in ((13, 0), (14, 7)):
            t = 2.0 ** (big_exp - k)
            vals = torch.zeros(1024, dtype=torch.float32)
            vals[idx[0]] = 2.0 ** big_exp
            for i in idx[1:]:
                vals[i] = t
            x = vals.to(tdt(kind)).to(dev)
            redux.set_variant("mfma")
            got = redux.sum(x).item()
            redux.set_variant("classic")
            ref = redux.sum(x).item()
            torch.cuda.synchronize()
            assert ref == 2.0 ** big_exp + 31 * t
            assert got == 2.0 ** big_exp + (31 - dropped) * t, (kind, k, got)
