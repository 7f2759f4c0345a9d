"""GPU parity of the contiguous-stream kernel for short segments -- 16-byte aligned powers of two from 16 B to
1 KiB, and its ragged form for any other length up to 1008 bytes at any element alignment: the two MMAs of
Section IV-A with 0/1 selection matrices (MFMA family) and the lane butterfly of Section III stopped early
(classic family), every element type, against the CPU oracle."""
import numpy as np
import pytest

import oracle
from paper_1903_03640_amd import redux, workloads

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL = 1e-4
TOL_F8_MFMA = 7 * 2.0 ** -14          # alignment window of the 8-bit MFMAs (see test_gpu_dtypes)
VARIANTS = ("mfma", "classic")
KINDS = ("f16", "bf16", "f32", "e4m3", "e5m2", "i8")
ESIZE = {"f16": 2, "bf16": 2, "f32": 4, "e4m3": 1, "e5m2": 1, "i8": 1}
ODT = {"bf16": oracle.BF16, "f32": oracle.F32, "e4m3": oracle.F8E4M3, "e5m2": oracle.F8E5M2}
CODE = {"f16": redux.F16, "bf16": redux.BF16, "f32": redux.F32, "e4m3": redux.F8E4M3, "e5m2": redux.F8E5M2, "i8": redux.I8}
SEG_BYTES = (16, 32, 64, 128, 256, 512, 1024, 2048, 4096)     # the last two: MMA family only (binary32 excepted)
# one wavefront's worth, a ragged count inside one slab, several slabs with a ragged last one, many slabs per block
NSEGS = (1, 3, 64, 1000, 4097, 70001)


def tdt(kind):
    return {"f16": torch.float16, "bf16": torch.bfloat16, "f32": torch.float32, "e4m3": torch.float8_e4m3fn,
            "e5m2": torch.float8_e5m2, "i8": torch.int8}[kind]


def patterns(kind, seed, n):
    """raw storage patterns of n finite values"""
    if kind == "f16":
        return workloads.normal_f16(seed, n)
    if kind == "i8":
        return workloads.uniform_i8(seed, n)
    if kind == "bf16":
        return workloads.normal_bf16(seed, n)
    if kind == "f32":
        return workloads.normal_f32(seed, n).view(np.uint32)
    return workloads.finite_f8(seed, n, kind)


def to_dev(pats, kind, dev):
    storage = {2: torch.int16, 4: torch.int32, 1: torch.int8}[pats.dtype.itemsize]
    signed = np.ascontiguousarray(pats).view({2: np.int16, 4: np.int32, 1: np.int8}[pats.dtype.itemsize])
    return torch.from_numpy(signed).to(dev).view(storage).view(tdt(kind))


def oracle_segmented(pats, kind, nseg, seglen):
    if kind == "f16":
        return oracle.sum_segmented_f16(pats, nseg, seglen)
    if kind == "i8":
        return oracle.sum_segmented_i8(pats, nseg, seglen)
    return oracle.sum_segmented_any(pats, nseg, seglen, ODT[kind])


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
    for name, val in (("max_grid", 16384), ("seg_blocks_per_cu", 0), ("layout", 2), ("nontemporal", 1), ("seg_short", 1), ("seg_short_pipe", -1), ("seg_ragged", 1)):
        redux.set_param(name, val)
    redux.set_variant("auto")


def expect_short(nseg, seglen, kind):
    """The plan for this shape under the current variant: the contiguous-stream kernel up to 1 KiB, and up to 4 KiB
    with the MMA family (binary32 excepted); the whole-tile kernel takes the rest if there are enough segments."""
    plan = redux.plan_sum_segmented(nseg, seglen, CODE[kind], x_address=0, compute_units=256)
    wide_ok = redux.get_variant() == redux.VARIANTS["mfma"] and kind != "f32"
    if seglen * ESIZE[kind] <= 1024 or wide_ok:
        assert plan.kernel == redux.KERNEL_SHORT, (kind, nseg, seglen, plan.kernel)
    else:
        assert plan.kernel in (redux.KERNEL_TILES, redux.KERNEL_RUNS), (kind, nseg, seglen, plan.kernel)


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("seg_bytes", SEG_BYTES)
@pytest.mark.parametrize("kind", KINDS)
def test_against_oracle(dev, kind, seg_bytes, variant):
    redux.set_variant(variant)
    seglen = seg_bytes // ESIZE[kind]
    tol = TOL_F8_MFMA if (variant == "mfma" and kind in ("e4m3", "e5m2")) else TOL
    for nseg in NSEGS:
        expect_short(nseg, seglen, kind)
        pats = patterns(kind, 7 * nseg + seg_bytes, nseg * seglen)
        got = redux.sum_segmented(to_dev(pats, kind, dev), nseg, seglen)
        torch.cuda.synchronize()
        want, want_abs = oracle_segmented(pats, kind, nseg, seglen)
        if kind == "i8":
            assert np.array_equal(got.cpu().numpy(), want), (nseg, seglen)
        else:
            err = np.abs(got.cpu().numpy().astype(np.float64) - want)
            assert np.all(err <= tol * want_abs), (kind, nseg, seglen, float(np.max(err / np.maximum(want_abs, 1e-300))))


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("seg_bytes", SEG_BYTES)
@pytest.mark.parametrize("kind", KINDS)
def test_every_segment_lands_in_its_own_slot(dev, kind, seg_bytes, variant):
    """Small integers are exact in every element type, so each result must equal its segment's integer sum
    bit for bit: any mix-up of rows, columns, loads or lanes shows."""
    redux.set_variant(variant)
    seglen = seg_bytes // ESIZE[kind]
    nseg = 3 * 2048 * 16 // (seg_bytes // 16) + 37          # three slabs and a ragged rest
    expect_short(nseg, seglen, kind)
    z = workloads.uniform_i8(seg_bytes, nseg * seglen).astype(np.int64)
    vals = z % 5 - 2                                        # -2 .. 2
    x = torch.from_numpy(vals.astype(np.float32)).to(dev).to(tdt(kind)) if kind != "i8" else torch.from_numpy(vals.astype(np.int8)).to(dev)
    want = vals.reshape(nseg, seglen).sum(axis=1)
    for max_grid, layout, pipe, nontemporal in ((16384, 2, -1, 1), (16384, 2, 0, 0), (16384, 2, 1, 1), (1, 2, 1, 0), (3, 0, 0, 1),
                                                (7, 1, 1, 1), (9, 2, 0, 1)):
        redux.set_param("max_grid", max_grid)
        redux.set_param("layout", layout)
        redux.set_param("seg_short_pipe", pipe)
        redux.set_param("nontemporal", nontemporal)
        got = redux.sum_segmented(x, nseg, seglen)
        torch.cuda.synchronize()
        assert np.array_equal(got.cpu().numpy().astype(np.int64), want), (kind, seg_bytes, max_grid, layout, pipe, nontemporal)


@pytest.mark.parametrize("variant", VARIANTS)
def test_matches_the_other_kernels_and_is_repeatable(dev, variant):
    """The same input through the contiguous-stream kernel and, with it switched off, through the kernels
    that handled these shapes before; and twice through itself, bit for bit."""
    redux.set_variant(variant)
    for seglen in (8, 64, 512):
        nseg = 50000
        pats = workloads.normal_f16(seglen, nseg * seglen)
        xd = to_dev(pats, "f16", dev)
        a = redux.sum_segmented(xd, nseg, seglen)
        b = redux.sum_segmented(xd, nseg, seglen)
        redux.set_param("seg_short", 0)
        c = redux.sum_segmented(xd, nseg, seglen)
        redux.set_param("seg_short", 1)
        torch.cuda.synchronize()
        assert torch.equal(a, b)
        want, want_abs = oracle.sum_segmented_f16(pats, nseg, seglen)
        for got in (a, c):
            assert np.all(np.abs(got.cpu().numpy().astype(np.float64) - want) <= TOL * want_abs)


def test_misaligned_or_odd_sizes_take_another_kernel(dev):
    redux.set_variant("classic")
    for seglen, addr in ((64, 2), (24, 0), (1024, 0), (4, 0)):
        plan = redux.plan_sum_segmented(1000, seglen, redux.F16, x_address=addr, compute_units=256)
        assert plan.kernel != redux.KERNEL_SHORT, (seglen, addr)
    redux.set_variant("auto")
    assert redux.plan_sum_segmented(1000, 4096, redux.F16, x_address=0, compute_units=256).kernel != redux.KERNEL_SHORT   # 8 KiB
    # and a misaligned base still gives the right sums
    nseg, seglen = 3000, 64
    pats = workloads.normal_f16(11, nseg * seglen)
    buf = torch.empty(nseg * seglen + 1, dtype=torch.float16, device=dev)
    buf[1:].copy_(to_dev(pats, "f16", dev))
    got = redux.sum_segmented(buf[1:], nseg, seglen)
    torch.cuda.synchronize()
    want, want_abs = oracle.sum_segmented_f16(pats, nseg, seglen)
    assert np.all(np.abs(got.cpu().numpy().astype(np.float64) - want) <= TOL * want_abs)


# ---- ragged form: any length up to 1008 bytes at any element alignment ---------------------------------------

def to_dev_at(pats, kind, dev, offset_elems):
    """the same patterns placed `offset_elems` elements past a 256-byte aligned allocation"""
    t = to_dev(pats, kind, dev)
    buf = torch.empty(t.numel() + offset_elems + 64, dtype=t.dtype, device=dev)      # room behind the end as well
    raw = buf.view(torch.uint8)
    raw.fill_(0xFF)                                      # what lies outside the array must never be added: all-ones bytes are NaN (or -1)
    view = buf[offset_elems:offset_elems + t.numel()]
    view.view(torch.uint8).copy_(t.view(torch.uint8))
    return view


RAGGED_BYTES = (1, 2, 3, 4, 6, 10, 14, 18, 30, 34, 66, 100, 130, 200, 258, 400, 514, 750, 1000, 1008)


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("kind", KINDS)
def test_ragged_against_oracle(dev, kind, variant):
    redux.set_variant(variant)
    es = ESIZE[kind]
    tol = TOL_F8_MFMA if (variant == "mfma" and kind in ("e4m3", "e5m2")) else TOL
    for seg_bytes in RAGGED_BYTES:
        if seg_bytes % es:
            continue
        seglen = seg_bytes // es
        for nseg, offset in ((1, 0), (37, 1), (5000, 3), (70001, 0)):
            x_addr_low = (offset * es) % 16
            plan = redux.plan_sum_segmented(nseg, seglen, CODE[kind], x_address=x_addr_low, compute_units=256)
            if plan.kernel in (redux.KERNEL_SHORT, redux.KERNEL_ROWS):
                continue                                  # an aligned shape another test covers
            assert plan.kernel == redux.KERNEL_RAGGED, (kind, seg_bytes, offset, plan.kernel)
            pats = patterns(kind, 3 * nseg + seg_bytes, nseg * seglen)
            xd = to_dev_at(pats, kind, dev, offset)
            assert xd.data_ptr() % 16 == x_addr_low
            got = redux.sum_segmented(xd, nseg, seglen)
            torch.cuda.synchronize()
            want, want_abs = oracle_segmented(pats, kind, nseg, seglen)
            if kind == "i8":
                assert np.array_equal(got.cpu().numpy(), want), (seg_bytes, nseg, offset)
            else:
                err = np.abs(got.cpu().numpy().astype(np.float64) - want)
                assert np.all(err <= tol * want_abs), (kind, seg_bytes, nseg, offset, float(np.max(err / np.maximum(want_abs, 1e-300))))


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("kind", KINDS)
def test_ragged_every_segment_lands_in_its_own_slot(dev, kind, variant):
    redux.set_variant(variant)
    es = ESIZE[kind]
    for seg_bytes, offset in ((es, 1), (es, 0), (4, 0), (8, 0), (8, 4 // es), (3 * es, 0), (20, 1), (52, 3), (236, 1), (1008, 0), (1008, 1), (48, 1), (1004, 0)):
        if seg_bytes % es:
            continue
        seglen = seg_bytes // es
        nseg = 5 * 2048 + 37
        vals = workloads.uniform_i8(seg_bytes + offset, nseg * seglen).astype(np.int64) % 5 - 2
        t = torch.from_numpy(vals.astype(np.float32)).to(tdt(kind)) if kind != "i8" else torch.from_numpy(vals.astype(np.int8))
        raw = t.view(torch.uint8).numpy().view({1: np.uint8, 2: np.uint16, 4: np.uint32}[es])
        xd = to_dev_at(raw, kind, dev, offset)
        want = vals.reshape(nseg, seglen).sum(axis=1)
        for max_grid, layout in ((16384, 2), (1, 2), (5, 0), (7, 1)):
            redux.set_param("max_grid", max_grid)
            redux.set_param("layout", layout)
            got = redux.sum_segmented(xd, nseg, seglen)
            torch.cuda.synchronize()
            assert np.array_equal(got.cpu().numpy().astype(np.int64), want), (kind, seg_bytes, offset, max_grid, layout)


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("kind", ("f16", "bf16", "f32", "e5m2", "e4m3"))
def test_non_finite_values_stay_in_their_segment(dev, kind, variant):
    """An infinity or NaN makes its own segment's sum non-finite and leaves every other segment exactly as it
    would be without it (a zero of a selection matrix times infinity must not leak into the neighbours)."""
    redux.set_variant(variant)
    es = ESIZE[kind]
    tol = TOL_F8_MFMA if (variant == "mfma" and kind in ("e4m3", "e5m2")) else TOL
    inf_bits = {"f16": 0x7C00, "bf16": 0x7F80, "f32": 0x7F800000, "e5m2": 0x7C, "e4m3": None}[kind]
    nan_bits = {"f16": 0x7E00, "bf16": 0x7FC0, "f32": 0x7FC00000, "e5m2": 0x7E, "e4m3": 0x7F}[kind]
    sign = {2: 0x8000, 4: 0x80000000, 1: 0x80}[es]
    for seg_bytes, offset in ((16, 0), (64, 0), (256, 0), (512, 0), (1024, 0), (2048, 0), (4096, 0), (40, 1), (200, 0), (1000, 1)):
        seglen = seg_bytes // es
        nseg = 3 * 2048 + 11
        pats = patterns(kind, seg_bytes, nseg * seglen).copy()
        bits = pats.view({1: np.uint8, 2: np.uint16, 4: np.uint32}[es])       # same memory, as storage patterns
        rng = np.random.default_rng(seg_bytes)
        hit = rng.choice(nseg, size=40, replace=False)
        for i, sg in enumerate(hit):
            pos = sg * seglen + int(rng.integers(seglen))
            if i % 3 == 0 or inf_bits is None:
                bits[pos] = nan_bits
            elif i % 3 == 1:
                bits[pos] = inf_bits
            else:
                bits[pos] = inf_bits | sign
        xd = to_dev_at(pats, kind, dev, offset)
        got = redux.sum_segmented(xd, nseg, seglen).cpu().numpy().astype(np.float64)
        torch.cuda.synchronize()
        want, want_abs = oracle_segmented(pats, kind, nseg, seglen)
        want = np.asarray(want, dtype=np.float64)
        finite = np.isfinite(want)
        assert finite.sum() == nseg - 40
        assert np.all(np.abs(got[finite] - want[finite]) <= tol * np.asarray(want_abs)[finite]), (kind, seg_bytes)
        nan = np.isnan(want)
        assert np.array_equal(np.isnan(got), nan), (kind, seg_bytes)
        assert np.array_equal(got[~finite & ~nan], want[~finite & ~nan]), (kind, seg_bytes)      # +inf and -inf
