"""Host logic without a GPU: the launch plans the library computes (grid, unroll, finish, pieces) and
the slab schedule of the flat kernel.  These are the numbers the kernels index memory with, so their
invariants are checked here over many shapes before anything runs on a device."""
import os

import pytest
from hypothesis import given, settings, strategies as st

from paper_1903_03640_amd import redux

pytestmark = pytest.mark.skipif(not os.path.exists(redux.LIB_PATH), reason="libredux.so not built")

ES = {redux.F16: 2, redux.I8: 1, redux.BF16: 2, redux.F32: 4, redux.F8E4M3: 1, redux.F8E5M2: 1}
DTYPES = sorted(ES)
PARAMS = ("blocks_per_cu", "seg_blocks_per_cu", "max_grid", "unroll", "finish", "seg_finish", "rows_max_vec", "seg_parts", "seg_tiles", "seg_block_bytes", "layout", "seg_short", "seg_ragged", "seg_runs", "seg_run_len", "seg_runs_max", "seg_runs_long", "seg_balance", "seg_runs_stream")


@pytest.fixture(autouse=True)
def restore_params():
    keep = {k: redux.get_param(k) for k in PARAMS}
    yield
    for k, v in keep.items():
        redux.set_param(k, v)


@settings(max_examples=400, deadline=None)
@given(n=st.one_of(st.integers(0, 5000), st.integers(0, 1 << 40)), dtype=st.sampled_from(DTYPES),
       mis=st.integers(0, 15), cus=st.sampled_from([1, 8, 104, 256, 304]),
       bpc=st.integers(1, 16), max_grid=st.sampled_from([1, 7, 256, 16384]), unroll=st.sampled_from([0, 1, 2, 4, 8]))
def test_flat_plan_invariants(n, dtype, mis, cus, bpc, max_grid, unroll):
    es = ES[dtype]
    addr = 4096 + (mis // es) * es                       # aligned to the element size, any 16-byte phase
    redux.set_param("blocks_per_cu", bpc)
    redux.set_param("max_grid", max_grid)
    redux.set_param("unroll", unroll)
    p = redux.plan_sum(n, dtype, addr, cus)
    per_vec = 16 // es
    # geometry: head + vectors + tail tile the array exactly; head ends on a 16-byte boundary
    assert p.head + p.vectors * per_vec + p.tail == n
    assert p.head < per_vec and p.tail < per_vec
    if p.vectors or p.tail:
        assert (addr + p.head * es) % 16 == 0
    assert p.unroll in (1, 2, 4, 8) and (unroll == 0 or p.unroll == unroll)
    nslab = p.vectors // (256 * p.unroll)
    assert 1 <= p.grid <= min(cus * bpc, max_grid, 16384)
    assert p.grid <= max(nslab, 1)
    assert p.finish in (5, 8) if dtype == redux.I8 else p.finish in (4, 6, 7) and (p.finish == 4) == (p.grid > 2048)
    assert (p.finish in (7, 8)) == (2 << 20 < p.vectors * 16 < 256 << 20) or p.finish == 4
    assert 1 <= p.chain <= 256                                       # the default max_chain, possibly lowered for int8
    assert p.kernel == redux.KERNEL_FLAT


def test_flat_plan_defaults_on_mi355x():
    c3 = redux.plan_sum((1 << 30) + 12345, redux.F16, 0, 256)
    assert (c3.unroll, c3.grid, c3.finish) == (8, 256, 6)           # one block per CU, 8 loads per lane, one kernel per call
    assert (c3.head, c3.tail, c3.vectors) == (0, 1, 134219271)      # the last 16-byte vector holds one element
    c1 = redux.plan_sum(1 << 20, redux.F16, 0, 256)
    assert (c1.unroll, c1.grid, c1.finish) == (8, 64, 6)            # small: few blocks, finishes in the same kernel
    assert redux.plan_sum(1 << 26, redux.F16, 0, 256).finish == 7   # 128 MiB: all blocks arrive together, so by die first
    assert redux.plan_sum(0, redux.I8, 0, 256).grid == 1
    for n, f in ((1 << 20, 5), (1 << 26, 8), (1 << 30, 5)):          # int8: block totals are added and counted by one atomic addition (mid sizes: by die first)
        assert redux.plan_sum(n, redux.I8, 0, 256).finish == f
    assert redux.plan_sum((1 << 40) + 4096, redux.I8, 0, 256).finish == 4   # beyond the 49 bits the counted word gives the sum
    assert redux.plan_sum(1 << 21, redux.F16, 0, 256).finish == 7             # 4 MiB: 128 blocks arrive together
    assert redux.plan_sum(1 << 20, redux.F16, 0, 256).finish == 6
    assert redux.plan_sum(1 << 27, redux.F16, 0, 256).finish == 6             # 256 MiB: they no longer do


@settings(max_examples=300, deadline=None)
@given(layout=st.integers(0, 2), nslab=st.integers(0, 5000), grid=st.integers(1, 600))
def test_slab_schedule_covers_every_slab_once(layout, nslab, grid):
    seen = bytearray(nslab)
    for b in range(grid):
        start, stride, count = redux.plan_block_slabs(layout, nslab, grid, b)
        assert count == 0 or stride >= 1
        for k in range(count):
            s = start + k * stride
            assert s < nslab and not seen[s]
            seen[s] = 1
    assert all(seen)


def test_slab_schedule_is_balanced_and_die_blocked():
    nslab, grid = 65537, 256
    for layout in (0, 1, 2):
        counts = [redux.plan_block_slabs(layout, nslab, grid, b)[2] for b in range(grid)]
        assert sum(counts) == nslab and max(counts) - min(counts) <= 2
    # layout 2: the blocks of die d (block % 8 == d) stay inside the d-th eighth of the array
    for b in range(grid):
        start, stride, count = redux.plan_block_slabs(2, nslab, grid, b)
        d = b % 8
        lo, hi = nslab * d // 8, nslab * (d + 1) // 8
        assert lo <= start and start + (count - 1) * stride < hi


@settings(max_examples=200, deadline=None)
@given(layout=st.integers(0, 2), nseg=st.one_of(st.integers(1, 40), st.integers(1, 60000)), per_run=st.integers(1, 16),
       grid=st.one_of(st.integers(1, 40), st.sampled_from([8, 16, 64, 256])))
def test_run_share_covers_every_segment_once_and_is_balanced(layout, nseg, per_run, grid):
    seen = bytearray(nseg)
    work = []
    for b in range(grid):
        for w in range(4):
            first, stride, rounds, tail_first, tail_count = redux.plan_run_share(layout, nseg, per_run, grid, b, w)
            assert 0 <= tail_count <= per_run
            runs = [(first + k * stride, per_run) for k in range(rounds)] + ([(tail_first, tail_count)] if tail_count else [])
            for s0, c in runs:
                assert s0 + c <= nseg and not any(seen[s0:s0 + c])
                seen[s0:s0 + c] = b"\x01" * c
            work.append(rounds * per_run + tail_count)
    assert all(seen)
    # the eight dies differ by at most one segment in what they own, the wavefronts of a die by one more
    assert max(work) - min(work) <= (2 if layout == 2 and grid % 8 == 0 else 1)


def test_run_share_extremes():
    # the largest grid (65536 wavefronts) and the longest runs: the 32-bit arithmetic of the last run's share holds
    nseg, per_run, grid = (1 << 20) * 16 - 1, 16, 16384
    for b in (0, 1, 7, 8191, 16383):
        for w in range(4):
            first, stride, rounds, tail_first, tail_count = redux.plan_run_share(0, nseg, per_run, grid, b, w)
            assert stride == grid * 4 * per_run and rounds == nseg // stride and tail_count in (15, 16)
            j = b * 4 + w
            rest = nseg - rounds * stride
            assert tail_first == rounds * stride + rest * j // (grid * 4) and first == j * per_run
    # a part gets whole rounds only while it has enough segments; 2^40 segments do not overflow anything
    first, stride, rounds, tail_first, tail_count = redux.plan_run_share(2, 1 << 40, 16, 768, 767, 3)
    lo, hi = (1 << 40) * 7 // 8, 1 << 40
    assert lo <= first < hi and stride == 96 * 4 * 16 and rounds == (hi - lo) // stride and tail_first + tail_count <= hi
    with pytest.raises(redux.ReduxError):
        redux.plan_run_share(0, 10, 17, 4, 0, 0)
    with pytest.raises(redux.ReduxError):
        redux.plan_run_share(0, 10, 4, 4, 0, 4)


@settings(max_examples=500, deadline=None)
@given(nseg=st.one_of(st.integers(1, 300), st.integers(1, 1 << 24)), seglen=st.one_of(st.integers(1, 3000), st.integers(1, 1 << 26), st.sampled_from([4, 8, 16, 32, 64, 128, 256, 512, 1024, 2048])),
       dtype=st.sampled_from(DTYPES), aligned=st.booleans(), cus=st.sampled_from([1, 104, 256]),
       seg_parts=st.sampled_from([0, 0, 0, 2, 8, 64, 4096]), rows_max=st.sampled_from([64, 64, 0, 5]),
       seg_bpc=st.integers(0, 16), unroll=st.sampled_from([0, 1, 2, 4, 8]), block_bytes=st.sampled_from([32768, 32768, 0, 1000]),
       seg_short=st.sampled_from([1, 1, 0]), seg_ragged=st.sampled_from([1, 1, 0]), seg_runs=st.sampled_from([1, 1, 0]),
       run_len=st.sampled_from([0, 0, 0, 1, 5, 16]), runs_max=st.sampled_from([0, 0, 7999, 1 << 18]),
       runs_long=st.sampled_from([36863, 36863, 0, 1 << 18]))
def test_segmented_plan_invariants(nseg, seglen, dtype, aligned, cus, seg_parts, rows_max, seg_bpc, unroll, block_bytes, seg_short, seg_ragged,
                                   seg_runs, run_len, runs_max, runs_long):
    es = ES[dtype]
    addr = 4096 if aligned else 4096 + es
    redux.set_param("seg_parts", seg_parts)
    redux.set_param("rows_max_vec", rows_max)
    redux.set_param("seg_blocks_per_cu", seg_bpc)
    redux.set_param("unroll", unroll)
    redux.set_param("seg_block_bytes", block_bytes)
    redux.set_param("seg_short", seg_short)
    redux.set_param("seg_ragged", seg_ragged)
    redux.set_param("seg_runs", seg_runs)
    redux.set_param("seg_run_len", run_len)
    redux.set_param("seg_runs_max", runs_max)
    runs_max = runs_max or (28671 if redux.resolved_variant(dtype, True) == "mfma" else 7999)   # 0 = by family
    redux.set_param("seg_runs_long", runs_long)
    p = redux.plan_sum_segmented(nseg, seglen, dtype, addr, cus)
    assert 1 <= p.grid <= 16 * cus
    limit = 4096 if dtype not in (redux.F32, redux.F8E4M3, redux.F8E5M2) else 1024    # variant auto: MMA family except for the 8-bit floats
    pow2_short = aligned and 16 <= seglen * es <= limit and (seglen * es) & (seglen * es - 1) == 0
    assert (p.kernel == redux.KERNEL_SHORT) == bool(seg_short and pow2_short)
    if p.kernel == redux.KERNEL_SHORT:
        assert p.vectors == seglen * es // 16 and p.unroll == 8 and p.parts == 1
        assert p.grid <= max(1, -(-(nseg * p.vectors) // 2048))            # never more blocks than 32 KiB slabs
    elif p.kernel == redux.KERNEL_RAGGED:
        sb = seglen * es
        assert seg_ragged and sb <= 1008 and p.unroll == 8 and p.parts == 1
        lanes = p.vectors
        assert lanes in (1, 2, 4, 8, 16, 32, 64)
        # every placement of a segment fits its lane group: first byte at most 16 - es bytes into a vector
        worst = addr % 16 if sb % 16 == 0 else (16 - sb if 16 % sb == 0 and addr % sb == 0 else 16 - es)
        assert lanes * 16 >= worst + sb and (lanes == 1 or (lanes // 2) * 16 < worst + sb)
        assert p.grid <= max(1, -(-(nseg * lanes) // 2048))
    elif p.kernel == redux.KERNEL_ROWS:
        assert dtype in (redux.F16, redux.I8) and aligned and (seglen * es) % 16 == 0
        assert not (seg_ragged and seglen * es <= 1008)              # only where the ragged form is off (or does not reach)
        assert p.vectors == seglen * es // 16 and 1 <= p.vectors <= rows_max
        assert p.unroll in (1, 2, 4, 8) and (p.vectors <= 4 * p.unroll or p.unroll == 8)
        waves = p.grid * 4
        super_groups = -(-(-(-nseg // 16)) // (8 // p.unroll))
        assert p.grid <= max(1, -(-super_groups // 4)) and waves >= 1
    elif p.kernel == redux.KERNEL_TILES:
        assert aligned and seglen * es == 1024 * p.unroll and p.unroll in (1, 2, 4, 8) and nseg >= 4 * cus
        assert p.parts == 1 and p.grid <= -(-nseg // 4)
    elif p.kernel == redux.KERNEL_BLOCK:
        assert block_bytes and seglen * es >= block_bytes and p.unroll in (1, 2, 4, 8)
        # pieces per segment: a power of two, or what makes exactly one round over one or two blocks per compute unit
        assert p.parts & (p.parts - 1) == 0 or (seg_parts == 0 and any(0 <= full - p.parts <= 2 for full in (cus // nseg, 2 * cus // nseg)))
        assert p.parts * p.part_len >= seglen
        if p.parts > 1:
            assert nseg * p.parts <= 16384 and p.part_len % 512 == 0
            # piece totals meet in a second kernel (2) or in the same one (5: int8, counted; 6: floating point, slots), and
            # in the same one only if no block has a second piece to go on to
            assert p.finish in ((2, 5) if dtype == redux.I8 else (2, 6))
            assert (p.finish != 2) == (nseg * p.parts <= p.grid)
        else:
            assert p.part_len == seglen and p.finish == 0
        assert p.grid <= nseg * p.parts
    elif p.kernel == redux.KERNEL_RUNS:
        sb = seglen * es
        long_range = 32768 < sb <= runs_long and nseg >= 8 * cus
        assert seg_runs and (1008 < sb <= runs_max or long_range) and p.parts == 1 and p.unroll in (4, 8) and p.finish == 0
        assert long_range or not (block_bytes and sb >= block_bytes)
        assert 1 <= p.vectors <= 16 and (run_len == 0 or p.vectors == run_len)
        assert run_len or p.vectors <= nseg
        nruns = -(-nseg // p.vectors)
        assert p.grid <= max(1, -(-nruns // 4))                 # never more wavefronts than runs
        assert 15 + p.vectors * sb < 1 << 32                    # a run's byte positions fit 32 bits
    else:
        assert p.unroll in (1, 2, 4, 8)
        assert not (seg_ragged and seglen * es <= 1008)
        if seg_runs and 1008 < seglen * es <= runs_max:          # whole segments of this size go to the run kernel
            assert p.kernel == redux.KERNEL_PIECES
        if p.kernel == redux.KERNEL_PIECES:
            assert p.parts > 1 and p.parts & (p.parts - 1) == 0
            assert nseg * p.parts <= 16384                      # piece totals fit the workspace
            assert p.part_len % 512 == 0 and p.parts * p.part_len >= seglen
            assert p.finish == 2
        else:
            assert p.kernel == redux.KERNEL_WAVE and p.parts == 1 and p.part_len == seglen
        assert p.grid <= max(1, -(-(nseg * p.parts) // 4))


def test_segmented_plan_defaults_on_mi355x():
    c5 = redux.plan_sum_segmented(65536, 4096, redux.F16, 0, 256)
    assert (c5.kernel, c5.unroll, c5.grid, c5.parts) == (redux.KERNEL_TILES, 8, 256, 1)      # 8 KiB segments: pipelined
    two_k = redux.plan_sum_segmented(65536, 1024, redux.F16, 0, 256)
    assert (two_k.kernel, two_k.vectors, two_k.grid) == (redux.KERNEL_SHORT, 128, 256)          # 2 KiB: contiguous stream, two loads per segment
    assert redux.plan_sum_segmented(65536, 512, redux.F32, 0, 256).grid == 768                  # binary32, 2 KiB: whole-tile kernel, three blocks per CU
    redux.set_param("seg_tiles", 0)
    c5 = redux.plan_sum_segmented(65536, 4096, redux.F16, 0, 256)
    assert (c5.kernel, c5.unroll, c5.grid, c5.parts) == (redux.KERNEL_RUNS, 4, 512, 1)            # runs of whole segments, rolling loads, two blocks per CU
    redux.set_param("seg_runs", 0)
    c5 = redux.plan_sum_segmented(65536, 4096, redux.F16, 0, 256)
    assert (c5.kernel, c5.unroll, c5.grid, c5.parts) == (redux.KERNEL_WAVE, 2, 1024, 1)           # 512 vectors: two loads per lane, four blocks per CU
    redux.set_param("seg_runs", 1)
    redux.set_param("seg_tiles", 1)
    assert redux.plan_sum_segmented(1023, 4096, redux.F16, 0, 256).kernel == redux.KERNEL_RUNS    # too few segments for the whole-tile kernel
    assert redux.plan_sum_segmented(65536, 4096 + 8, redux.F16, 0, 256).kernel == redux.KERNEL_RUNS   # 8208 B: the rolling form reaches up to 28 KiB
    assert redux.plan_sum_segmented(65536, 14000, redux.F16, 0, 256).kernel == redux.KERNEL_RUNS      # 28000 B
    assert redux.plan_sum_segmented(65536, 14336, redux.F16, 0, 256).kernel == redux.KERNEL_BLOCK     # 28 KiB
    redux.set_variant("classic")
    assert redux.plan_sum_segmented(65536, 4096 + 8, redux.F16, 0, 256).kernel == redux.KERNEL_WAVE   # the run-by-run forms stop below 8000 B
    redux.set_variant("auto")
    redux.set_param("seg_runs_stream", 0)
    assert redux.plan_sum_segmented(65536, 4096 + 8, redux.F16, 0, 256).kernel == redux.KERNEL_WAVE
    redux.set_param("seg_runs_stream", 1)
    three = redux.plan_sum_segmented(65536, 3 * 512, redux.F16, 0, 256)                           # 3 KiB: not a power of two
    assert (three.kernel, three.vectors, three.unroll, three.grid) == (redux.KERNEL_RUNS, 13, 4, 512)   # 32 segments per wavefront on two blocks per CU: two runs of 13 and a last one of 6 (runs of 16 would be 48 KiB: in step with the memory channels)
    few = redux.plan_sum_segmented(40, 2050, redux.F16, 0, 256)
    assert (few.kernel, few.vectors, few.grid) == (redux.KERNEL_RUNS, 1, 10)                      # few segments: one per run
    redux.set_variant("classic")
    three = redux.plan_sum_segmented(65536, 3 * 512, redux.F16, 0, 256)
    assert (three.kernel, three.unroll, three.grid) == (redux.KERNEL_RUNS, 4, 2 * 256)               # rolling: four loads, two blocks per CU
    assert redux.plan_sum_segmented(65536, 1000, redux.F16, 0, 256).grid == 3 * 256                 # 2000 B: three
    redux.set_param("seg_runs_stream", 0)
    three = redux.plan_sum_segmented(65536, 3 * 512, redux.F16, 0, 256)
    assert (three.kernel, three.unroll) == (redux.KERNEL_RUNS, 8) and three.grid in (4 * 256, 8 * 256)   # run by run: eight loads, more wavefronts
    redux.set_param("seg_runs_stream", 1)
    redux.set_variant("auto")
    redux.set_param("seg_runs_stream", 0)                                                          # the plain form wants three blocks per CU
    assert redux.plan_sum_segmented(65536, 3 * 512, redux.F16, 0, 256).grid == 768
    redux.set_param("seg_runs_stream", 1)
    assert redux.plan_sum_segmented(65536, 600, redux.F16, 0, 256).grid == 768                     # 1200 B: three also for the rolling form
    redux.set_param("seg_runs", 0)
    assert redux.plan_sum_segmented(65536, 3 * 512, redux.F16, 0, 256).kernel == redux.KERNEL_WAVE
    redux.set_param("seg_runs", 1)
    redux.set_param("seg_runs_max", 7999)
    assert redux.plan_sum_segmented(65536, 4096 + 8, redux.F16, 0, 256).kernel == redux.KERNEL_WAVE
    redux.set_param("seg_runs_max", 0)
    # just above 32 KiB a block's second pass would be mostly idle: runs, while every wavefront can have a segment of its own
    assert redux.plan_sum_segmented(2048, 18000, redux.F16, 0, 256).kernel == redux.KERNEL_RUNS
    assert redux.plan_sum_segmented(2047, 18000, redux.F16, 0, 256).kernel == redux.KERNEL_BLOCK
    assert redux.plan_sum_segmented(2048, 16384, redux.F16, 0, 256).kernel == redux.KERNEL_BLOCK     # 32 KiB exactly
    assert redux.plan_sum_segmented(4096, 18432, redux.F16, 0, 256).kernel == redux.KERNEL_BLOCK     # 36 KiB and up
    redux.set_param("seg_runs_long", 0)
    assert redux.plan_sum_segmented(2048, 18000, redux.F16, 0, 256).kernel == redux.KERNEL_BLOCK
    redux.set_param("seg_runs_long", 36863)
    # 1072 segments of 500000 bytes on 512 blocks would be 2.1 rounds: four pieces each make it 8.4
    cut = redux.plan_sum_segmented(1072, 250000, redux.F16, 0, 256)
    assert (cut.kernel, cut.parts, cut.grid, cut.finish) == (redux.KERNEL_BLOCK, 4, 512, 2) and cut.part_len * 2 >= 65536
    # where the pieces of a segment meet: in the same kernel wherever there is a block for every piece, in a second
    # kernel where a block has a second piece to go on to
    for shape, want in (((2, 1 << 20, redux.F16), (64, 128, 6)), ((128, 1 << 19, redux.F16), (2, 256, 6)), ((16, 1 << 22, redux.F16), (16, 256, 6)),
                        ((16, 1 << 23, redux.I8), (16, 256, 5)), ((2, 1 << 26, redux.I8), (128, 256, 5)), ((100, 2621440, redux.F16), (64, 512, 2)),
                        ((2, 1 << 27, redux.F16), (128, 256, 6))):
        q = redux.plan_sum_segmented(shape[0], shape[1], shape[2], 0, 256)
        assert (q.kernel, q.parts, q.grid, q.finish) == (redux.KERNEL_BLOCK,) + want, (shape, q.parts, q.grid, q.finish)
    redux.set_param("seg_finish", 0)
    assert redux.plan_sum_segmented(2, 1 << 20, redux.F16, 0, 256).finish == 2
    redux.set_param("seg_finish", 1)
    assert redux.plan_sum_segmented(100, 2621440, redux.F16, 0, 256).finish == 6
    redux.set_param("seg_finish", -1)
    redux.set_param("seg_balance", 0)
    assert redux.plan_sum_segmented(1072, 250000, redux.F16, 0, 256).parts == 1
    redux.set_param("seg_balance", 1)
    assert redux.plan_sum_segmented(1024, 250000, redux.F16, 0, 256).parts == 1                  # two whole rounds: nothing to gain
    short = redux.plan_sum_segmented(1 << 22, 64, redux.F16, 0, 256)
    assert (short.kernel, short.vectors, short.unroll, short.grid) == (redux.KERNEL_SHORT, 8, 8, 256)   # 128 B: contiguous stream
    assert redux.plan_sum_segmented(1 << 22, 64, redux.BF16, 0, 256).kernel == redux.KERNEL_SHORT     # every dtype
    assert redux.plan_sum_segmented(100, 64, redux.F16, 0, 256).grid == 1                             # 12.5 KiB: one slab
    rag = redux.plan_sum_segmented(1 << 22, 72, redux.F16, 0, 256)
    assert (rag.kernel, rag.vectors) == (redux.KERNEL_RAGGED, 16)                                     # 144 B: 9 of 16 lanes busy
    redux.set_param("seg_ragged", 0)
    rows = redux.plan_sum_segmented(1 << 22, 72, redux.F16, 0, 256)
    assert (rows.kernel, rows.vectors, rows.unroll) == (redux.KERNEL_ROWS, 9, 4)
    redux.set_param("seg_ragged", 1)
    redux.set_param("seg_short", 0)
    for dt in (redux.F16, redux.BF16):
        ragged = redux.plan_sum_segmented(1 << 22, 64, dt, 0, 256)                                    # full lane groups: the ragged form
        assert (ragged.kernel, ragged.vectors) == (redux.KERNEL_RAGGED, 8)
    redux.set_param("seg_ragged", 0)
    short = redux.plan_sum_segmented(1 << 22, 64, redux.F16, 0, 256)
    assert (short.kernel, short.vectors, short.unroll) == (redux.KERNEL_ROWS, 8, 2)
    assert redux.plan_sum_segmented(1 << 22, 64, redux.BF16, 0, 256).kernel == redux.KERNEL_WAVE      # rows: binary16 and int8 only
    redux.set_param("seg_ragged", 1)
    redux.set_param("seg_short", 1)
    ragged = redux.plan_sum_segmented(1 << 22, 64, redux.F16, 2, 256)                                 # misaligned base: 9 vectors
    assert (ragged.kernel, ragged.vectors, ragged.grid) == (redux.KERNEL_RAGGED, 16, 2 * 256)            # 9 of 16 lanes busy: two blocks per CU
    ragged = redux.plan_sum_segmented(1 << 20, 100, redux.BF16, 0, 256)                               # 200 B anywhere: 14 vectors
    assert (ragged.kernel, ragged.vectors) == (redux.KERNEL_RAGGED, 16)
    assert redux.plan_sum_segmented(1 << 20, 3, redux.F8E4M3, 0, 256).vectors == 2                    # 3 B can straddle two vectors
    assert redux.plan_sum_segmented(1 << 20, 2, redux.F16, 0, 256).vectors == 1                       # 4 B on a 4-byte boundary cannot
    assert redux.plan_sum_segmented(1 << 20, 2, redux.F16, 2, 256).vectors == 2
    longest = redux.plan_sum_segmented(1 << 20, 504, redux.F16, 0, 256)                               # 1008 B: the longest
    assert (longest.vectors, longest.grid) == (64, 256)                                               # 63 of 64 lanes busy: one block per CU
    assert redux.plan_sum_segmented(1 << 20, 252, redux.F32, 0, 256).grid == 512                      # binary32 runs the classic family: one block more
    assert redux.plan_sum_segmented(1 << 20, 253, redux.F32, 0, 256).kernel == redux.KERNEL_RUNS
    redux.set_param("seg_ragged", 0)
    assert redux.plan_sum_segmented(1 << 22, 64, redux.F16, 2, 256).kernel == redux.KERNEL_WAVE
    redux.set_param("seg_ragged", 1)
    long_ = redux.plan_sum_segmented(256, 1 << 20, redux.F16, 0, 256)
    assert (long_.kernel, long_.parts, long_.part_len, long_.unroll, long_.grid) == (redux.KERNEL_BLOCK, 1, 1 << 20, 8, 256)    # a block each, one round
    long_ = redux.plan_sum_segmented(64, 1 << 22, redux.F16, 0, 256)
    assert (long_.kernel, long_.parts, long_.part_len, long_.unroll, long_.grid) == (redux.KERNEL_BLOCK, 4, 1 << 20, 8, 256)    # four pieces each make it 256
    assert redux.plan_sum_segmented(4096, 65536, redux.F16, 0, 256).kernel == redux.KERNEL_BLOCK      # 128 KiB each, no pieces
    redux.set_param("seg_block_bytes", 0)
    long_ = redux.plan_sum_segmented(256, 1 << 20, redux.F16, 0, 256)
    assert (long_.kernel, long_.parts, long_.part_len) == (redux.KERNEL_PIECES, 8, 131072)
    redux.set_param("seg_block_bytes", 28672)
    assert redux.plan_sum_segmented(1, 100, redux.I8, 0, 256).kernel == redux.KERNEL_RAGGED
    assert redux.plan_sum_segmented(1, 2000, redux.I8, 0, 256).kernel == redux.KERNEL_RUNS


def test_plan_argument_errors():
    import ctypes
    lib = redux.load()
    p = redux.Plan()
    assert lib.redux_plan_sum(8, 9, 0, 256, ctypes.byref(p)) == -2
    assert lib.redux_plan_sum(8, redux.F16, 0, 0, ctypes.byref(p)) == -8
    assert lib.redux_plan_sum(8, redux.F16, 0, 256, None) == -1
    assert lib.redux_plan_sum(1 << 63, redux.F32, 0, 256, ctypes.byref(p)) == -3
    assert lib.redux_plan_sum_segmented(0, 8, redux.F16, 0, 256, ctypes.byref(p)) == -8
    assert lib.redux_plan_sum_segmented(1 << 40, 1 << 40, redux.F16, 0, 256, ctypes.byref(p)) == -3
    with pytest.raises(redux.ReduxError):
        redux.plan_block_slabs(3, 10, 4, 0)
    with pytest.raises(redux.ReduxError):
        redux.plan_block_slabs(0, 10, 4, 4)


@settings(max_examples=300, deadline=None)
@given(max_chain=st.sampled_from([1, 100, 256, 4096, 16384, 32768, 65536]), unroll=st.sampled_from([0, 1, 2, 4, 8]),
       variant=st.sampled_from(["mfma", "classic"]), n=st.integers(1, 1 << 36), seg=st.booleans(),
       block_bytes=st.sampled_from([0, 32768]))
def test_int8_chain_never_lets_an_int32_accumulator_wrap(max_chain, unroll, variant, n, seg, block_bytes):
    """chain x (largest magnitude one loop iteration can add to an accumulator entry) stays below 2^31:
    an int8 MFMA adds at most 64 x 128 per entry, the classic dot product at most 4 x 128 per running sum and vector."""
    keep = redux.get_param("max_chain"), redux.get_variant()
    redux.set_param("max_chain", max_chain)
    redux.set_param("unroll", unroll)
    redux.set_param("seg_block_bytes", block_bytes)
    redux.set_variant(variant)
    try:
        if seg:
            p = redux.plan_sum_segmented(3, n, redux.I8, 0, 256)
            chains = 4 if p.kernel == redux.KERNEL_BLOCK else 1
        else:
            p = redux.plan_sum(n, redux.I8, 0, 256)
            chains = 4
        assert 1 <= p.chain <= max_chain
        if p.kernel in (redux.KERNEL_FLAT, redux.KERNEL_BLOCK, redux.KERNEL_WAVE, redux.KERNEL_PIECES):
            per_iter = 8192 * -(-p.unroll // chains) if variant == "mfma" else 512 * p.unroll
            assert p.chain * per_iter < 2 ** 31
        # floating point: the setting is taken as it is
        assert redux.plan_sum(n, redux.F16, 0, 256).chain == max_chain
    finally:
        redux.set_param("max_chain", keep[0])
        redux.set_variant(keep[1])
