"""GPU parity of the contiguous-stream kernel for short power-of-two segments (16 B .. 1 KiB, 16-byte
aligned): the two MMAs of Section IV-A with 0/1 selection matrices (MFMA family) and the lane butterfly
of Section III stopped early (classic family), every element type, against the CPU oracle."""
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
SEG_BYTES = (16, 32, 64, 128, 256, 512, 1024)
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
    for name, val in (("max_grid", 16384), ("seg_blocks_per_cu", 0), ("layout", 2), ("nontemporal", 1), ("seg_short", 1), ("seg_short_pipe", -1)):
        redux.set_param(name, val)
    redux.set_variant("auto")


def expect_short(nseg, seglen, kind):
    plan = redux.plan_sum_segmented(nseg, seglen, CODE[kind], x_address=0, compute_units=256)
    assert plan.kernel == redux.KERNEL_SHORT, (kind, nseg, seglen, plan.kernel)


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
    for seglen, addr in ((64, 2), (24, 0), (1024, 0), (4, 0)):
        plan = redux.plan_sum_segmented(1000, seglen, redux.F16, x_address=addr, compute_units=256)
        assert plan.kernel != redux.KERNEL_SHORT, (seglen, addr)
    # and a misaligned base still gives the right sums
    nseg, seglen = 3000, 64
    pats = workloads.normal_f16(11, nseg * seglen)
    buf = torch.empty(nseg * seglen + 1, dtype=torch.float16, device=dev)
    buf[1:].copy_(to_dev(pats, "f16", dev))
    got = redux.sum_segmented(buf[1:], nseg, seglen)
    torch.cuda.synchronize()
    want, want_abs = oracle.sum_segmented_f16(pats, nseg, seglen)
    assert np.all(np.abs(got.cpu().numpy().astype(np.float64) - want) <= TOL * want_abs)
