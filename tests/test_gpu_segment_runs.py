"""GPU parity of the run-of-segments kernel: segments from 1009 bytes to 256 KiB (by default it takes those below
8000 bytes) of any length at any element alignment, a run of up to sixteen whole segments per wavefront read as one contiguous piece of memory, each
segment owning one column of the MMA accumulator (first MMA of Section IV-A with a one-column selector, issued
once per side of a segment boundary; second MMA folds the rows), and its classic form; against the CPU oracle."""
import numpy as np
import pytest

import oracle
from paper_1903_03640_amd import redux, workloads
from test_gpu_short_segments import (CODE, ESIZE, KINDS, TOL, TOL_F8_MFMA, VARIANTS, oracle_segmented, patterns, tdt,
                                     to_dev_at)

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

# bytes per segment: just above the short kernels' limit, ragged at every scale, whole vectors, several iterations
# of 8 KiB per segment, up to the size the one-block-per-segment kernel takes over
RUN_BYTES = (1010, 1012, 1024 + 16, 1500, 2052, 3000, 4100, 5000, 8200, 12000, 16388, 30000, 32766)


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available()
    redux.load()
    torch.cuda.set_device(0)
    yield torch.device("cuda:0")
    redux.set_variant("auto")


@pytest.fixture(autouse=True)
def reset():
    redux.set_param("seg_runs_max", 1 << 18)                     # every size here through this kernel, not only what it takes by default
    redux.set_param("seg_block_bytes", 32768)
    yield
    redux.set_param("seg_runs_max", 0)
    redux.set_param("seg_runs_long", 36863)
    for name, val in (("max_grid", 16384), ("seg_blocks_per_cu", 0), ("unroll", 0), ("nontemporal", 1), ("seg_runs", 1), ("seg_run_len", 0), ("seg_runs_stream", 1),
                      ("seg_block_bytes", 28672), ("seg_parts", 0), ("seg_short", 1), ("seg_tiles", 1)):
        redux.set_param(name, val)
    redux.set_variant("auto")


def check(got, pats, kind, nseg, seglen, tol, what):
    want, want_abs = oracle_segmented(pats, kind, nseg, seglen)
    if kind == "i8":
        assert np.array_equal(got.cpu().numpy(), want), what
    else:
        err = np.abs(got.cpu().numpy().astype(np.float64) - want)
        assert np.all(err <= tol * want_abs), (what, float(np.max(err / np.maximum(want_abs, 1e-300))))


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("kind", KINDS)
def test_runs_against_oracle(dev, kind, variant):
    redux.set_variant(variant)
    es = ESIZE[kind]
    tol = TOL_F8_MFMA if (variant == "mfma" and kind in ("e4m3", "e5m2")) else TOL
    for seg_bytes in RUN_BYTES:
        if seg_bytes % es:
            continue
        seglen = seg_bytes // es
        # one segment, fewer than a run, a ragged number of runs; the base at several alignments
        for nseg, offset in ((1, 0), (5, 1), (37, 3), ((6 << 20) // seg_bytes + 3, 1)):
            x_addr_low = (offset * es) % 16
            redux.set_param("seg_parts", 1)                      # a few long segments would otherwise be cut into pieces
            plan = redux.plan_sum_segmented(nseg, seglen, CODE[kind], x_address=x_addr_low, compute_units=256)
            assert plan.kernel == redux.KERNEL_RUNS and 1 <= plan.vectors <= 16, (kind, seg_bytes, nseg, plan.kernel)
            pats = patterns(kind, 5 * nseg + seg_bytes, nseg * seglen)
            xd = to_dev_at(pats, kind, dev, offset)
            assert xd.data_ptr() % 16 == x_addr_low
            got = redux.sum_segmented(xd, nseg, seglen)
            torch.cuda.synchronize()
            check(got, pats, kind, nseg, seglen, tol, (kind, seg_bytes, nseg, offset))


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("kind", KINDS)
def test_runs_every_segment_lands_in_its_own_slot(dev, kind, variant):
    """Small integers are exact in every element type: each result must equal its segment's integer sum bit for
    bit, for every run length, so a byte on the wrong side of a boundary or a column mix-up shows."""
    redux.set_variant(variant)
    es = ESIZE[kind]
    for seg_bytes, offset in ((1012, 1), (1024, 1), (1028, 0), (2000, 3), (4100, 1), (8192 + 4, 0), (20000, 2)):
        if seg_bytes % es:
            continue
        seglen = seg_bytes // es
        nseg = (3 << 20) // seg_bytes + 5
        vals = workloads.uniform_i8(seg_bytes + offset, nseg * seglen).astype(np.int64) % 5 - 2
        t = torch.from_numpy(vals.astype(np.float32)).to(tdt(kind)) if kind != "i8" else torch.from_numpy(vals.astype(np.int8))
        raw = t.view(torch.uint8).numpy().view({1: np.uint8, 2: np.uint16, 4: np.uint32}[es])
        xd = to_dev_at(raw, kind, dev, offset)
        want = vals.reshape(nseg, seglen).sum(axis=1)
        redux.set_param("seg_parts", 1)                          # a few long segments would otherwise be cut into pieces
        for run_len, max_grid, nontemporal in ((0, 16384, 1), (1, 16384, 1), (2, 3, 0), (7, 16384, 1), (16, 1, 1), (16, 16384, 0)):
            redux.set_param("seg_run_len", run_len)
            redux.set_param("max_grid", max_grid)
            redux.set_param("nontemporal", nontemporal)
            plan = redux.plan_sum_segmented(nseg, seglen, CODE[kind], x_address=xd.data_ptr() % 16, compute_units=256)
            assert plan.kernel == redux.KERNEL_RUNS and (run_len == 0 or plan.vectors == run_len), (seg_bytes, plan.kernel, plan.vectors)
            got = redux.sum_segmented(xd, nseg, seglen)
            torch.cuda.synchronize()
            assert np.array_equal(got.cpu().numpy().astype(np.int64), want), (kind, seg_bytes, offset, run_len, max_grid)


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("kind", ("f16", "bf16", "f32", "e5m2", "e4m3"))
def test_runs_non_finite_values_stay_in_their_segment(dev, kind, variant):
    """An infinity or NaN makes its own segment's sum non-finite and leaves every other segment of its run exactly as it
    would be without it (a zero of the column selector times infinity must not leak into the neighbours)."""
    redux.set_variant(variant)
    es = ESIZE[kind]
    tol = TOL_F8_MFMA if (variant == "mfma" and kind in ("e4m3", "e5m2")) else TOL
    inf_bits = {"f16": 0x7C00, "bf16": 0x7F80, "f32": 0x7F800000, "e5m2": 0x7C, "e4m3": None}[kind]
    nan_bits = {"f16": 0x7E00, "bf16": 0x7FC0, "f32": 0x7FC00000, "e5m2": 0x7E, "e4m3": 0x7F}[kind]
    sign = {2: 0x8000, 4: 0x80000000, 1: 0x80}[es]
    redux.set_param("seg_parts", 1)                              # a few long segments would otherwise be cut into pieces
    for seg_bytes, offset in ((1012, 1), (3000, 0), (8200, 1)):
        seglen = seg_bytes // es
        nseg = 2000
        pats = patterns(kind, seg_bytes, nseg * seglen).copy()
        bits = pats.view({1: np.uint8, 2: np.uint16, 4: np.uint32}[es])
        rng = np.random.default_rng(seg_bytes)
        hit = rng.choice(nseg, size=40, replace=False)
        for i, sg in enumerate(hit):
            # first and last element of a segment too: the bytes right next to a boundary
            pos = sg * seglen + (0 if i % 5 == 0 else seglen - 1 if i % 5 == 1 else int(rng.integers(seglen)))
            if i % 3 == 0 or inf_bits is None:
                bits[pos] = nan_bits
            elif i % 3 == 1:
                bits[pos] = inf_bits
            else:
                bits[pos] = inf_bits | sign
        xd = to_dev_at(pats, kind, dev, offset)
        assert redux.plan_sum_segmented(nseg, seglen, CODE[kind], x_address=xd.data_ptr() % 16, compute_units=256).kernel == redux.KERNEL_RUNS
        got = redux.sum_segmented(xd, nseg, seglen).cpu().numpy().astype(np.float64)
        torch.cuda.synchronize()
        want, want_abs = oracle_segmented(pats, kind, nseg, seglen)
        want = np.asarray(want, dtype=np.float64)
        finite = np.isfinite(want)
        assert finite.sum() == nseg - 40
        assert np.all(np.abs(got[finite] - want[finite]) <= tol * np.asarray(want_abs)[finite]), (kind, seg_bytes)
        nan = np.isnan(want)
        assert np.array_equal(np.isnan(got), nan), (kind, seg_bytes)
        assert np.array_equal(got[~finite & ~nan], want[~finite & ~nan]), (kind, seg_bytes)


@pytest.mark.parametrize("variant", VARIANTS)
def test_runs_int8_extremes_and_largest_segment(dev, variant):
    """All elements at an extreme in the largest segment the kernel takes (256 KiB): the int32 accumulator columns and the
    exact second MMA hold; and the same sums as the one-wavefront-per-segment kernel gives."""
    redux.set_variant(variant)
    redux.set_param("seg_block_bytes", 0)                        # never one block per segment
    redux.set_param("seg_parts", 1)
    seglen, nseg = 256 << 10, 9
    for value in (-128, 127):
        x = torch.full((nseg * seglen + 3,), value, dtype=torch.int8, device=dev)[3:]
        assert redux.plan_sum_segmented(nseg, seglen, redux.I8, x_address=x.data_ptr() % 16, compute_units=256).kernel == redux.KERNEL_RUNS
        got = redux.sum_segmented(x, nseg, seglen)
        torch.cuda.synchronize()
        assert got.cpu().tolist() == [value * seglen] * nseg
    pats = workloads.normal_f16(3, 300 * 4100)
    xd = to_dev_at(pats, "f16", dev, 1)
    a = redux.sum_segmented(xd, 300, 4100)
    b = redux.sum_segmented(xd, 300, 4100)
    redux.set_param("seg_runs", 0)
    assert redux.plan_sum_segmented(300, 4100, redux.F16, x_address=2, compute_units=256).kernel == redux.KERNEL_WAVE
    c = redux.sum_segmented(xd, 300, 4100)
    torch.cuda.synchronize()
    assert torch.equal(a, b)                                     # repeatable bit for bit
    want, want_abs = oracle.sum_segmented_f16(pats, 300, 4100)
    for got in (a, c):
        assert np.all(np.abs(got.cpu().numpy().astype(np.float64) - want) <= TOL * want_abs)


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("kind", ("f16", "i8"))
def test_runs_take_segments_just_above_32_kib_by_default(dev, kind, variant):
    """With every setting at its default, many segments of a little more than 32 KiB go through this kernel (few of them, or
    longer ones, through one block per segment); the wavefronts' last, shorter runs are part of what is checked."""
    redux.set_variant(variant)
    redux.set_param("seg_runs_max", 0)
    es = ESIZE[kind]
    for seg_bytes, nseg, offset, kernel in ((36002, 2100, 1, redux.KERNEL_RUNS), (33000, 2048, 0, redux.KERNEL_RUNS),
                                            (36002, 2047, 1, redux.KERNEL_BLOCK), (36864, 2100, 0, redux.KERNEL_BLOCK), (40000, 2100, 1, redux.KERNEL_BLOCK)):
        seglen = seg_bytes // es
        pats = patterns(kind, seg_bytes + nseg, nseg * seglen)
        xd = to_dev_at(pats, kind, dev, offset)
        assert redux.plan_sum_segmented(nseg, seglen, CODE[kind], x_address=xd.data_ptr() % 16, compute_units=256).kernel == kernel
        got = redux.sum_segmented(xd, nseg, seglen)
        torch.cuda.synchronize()
        check(got, pats, kind, nseg, seglen, TOL, (kind, seg_bytes, nseg, offset))


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("kind", KINDS)
def test_rolling_and_plain_form_give_the_same_bits(dev, kind, variant):
    """Both families have two forms of this kernel: loads rolling across the ends of runs (the default) and run by run.
    Given the same grid and run length both issue the same MMAs on the same data in the same order, so every result must
    be the same bit for bit: small and large shapes, every run length, tiny grids.  A run with a non-finite value is summed again by the classic form in
    both, run by run (the rolling form keeps one bit for each of a wavefront's first 64 runs), so with NaNs in the data
    and at most 64 runs per wavefront the two still agree bit for bit (the classic family never mixes segments and has
    nothing to sum again)."""
    redux.set_variant(variant)
    es = ESIZE[kind]
    redux.set_param("seg_parts", 1)
    redux.set_param("seg_blocks_per_cu", 3)                      # the same grid, and so the same runs, for both forms
    redux.set_param("unroll", 4)                                 # (and the same loads per iteration, which the run length is chosen by)
    for seg_bytes, nseg, offset in ((1012, 1, 0), (1012, 5, 1), (1040, 37, 3), (2000, 1000, 1), (3000, 70001, 0), (4100, 333, 5), (8200, 64, 1),
                                    (20000, 17, 2), (1016, 30000, 1), (32766, 9, 3)):
        if seg_bytes % es:
            continue
        seglen = seg_bytes // es
        for with_nan in (False, True):
            if with_nan and (kind == "i8" or nseg < 5):
                continue
            pats = patterns(kind, seg_bytes + nseg, nseg * seglen).copy()
            if with_nan:
                bits = pats.view({1: np.uint8, 2: np.uint16, 4: np.uint32}[es])
                nan = {"f16": 0x7E00, "bf16": 0x7FC0, "f32": 0x7FC00000, "e5m2": 0x7E, "e4m3": 0x7F}[kind]
                bits[seglen + 3] = nan
                bits[(nseg - 1) * seglen] = nan
            xd = to_dev_at(pats, kind, dev, offset)
            # (with NaNs only shapes of at most 64 runs per wavefront: the default grid, or few segments)
            for run_len, max_grid in ((0, 16384), (1, 16384), (16, 16384)) + (((3, 2), (16, 1)) if not with_nan or nseg <= 64 else ()):
                redux.set_param("seg_run_len", run_len)
                redux.set_param("max_grid", max_grid)
                assert redux.plan_sum_segmented(nseg, seglen, CODE[kind], x_address=xd.data_ptr() % 16, compute_units=256).kernel == redux.KERNEL_RUNS
                redux.set_param("seg_runs_stream", 0)
                plain = redux.sum_segmented(xd, nseg, seglen)
                redux.set_param("seg_runs_stream", 1)
                rolling = redux.sum_segmented(xd, nseg, seglen)
                torch.cuda.synchronize()
                a, b = plain.cpu().numpy(), rolling.cpu().numpy()
                assert np.array_equal(a.view(np.uint8), b.view(np.uint8)), (variant, kind, seg_bytes, nseg, offset, with_nan, run_len, max_grid)


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("kind", ("f16", "i8"))
def test_plain_form_against_oracle(dev, kind, variant):
    """The run-by-run form is no longer what runs by default: its own pass against the oracle."""
    redux.set_variant(variant)
    redux.set_param("seg_runs_stream", 0)
    redux.set_param("seg_parts", 1)
    es = ESIZE[kind]
    for seg_bytes, nseg, offset in ((1010, 37, 1), (3000, 5000, 0), (8200, 300, 3), (30000, 40, 1)):
        if seg_bytes % es:
            continue
        seglen = seg_bytes // es
        pats = patterns(kind, seg_bytes, nseg * seglen)
        xd = to_dev_at(pats, kind, dev, offset)
        got = redux.sum_segmented(xd, nseg, seglen)
        torch.cuda.synchronize()
        check(got, pats, kind, nseg, seglen, TOL, (kind, seg_bytes, nseg, offset))
