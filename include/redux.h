/*
 * redux.h -- C ABI of libredux: arithmetic reduction of n numbers to one sum on
 * an AMD MI355X (gfx950), with the additions encoded as chains of
 * matrix-multiply-accumulate (MMA) operations against an all-ones operand.
 *
 * Method: the tensor-core reduction of Section IV-A of "Analyzing GPU Tensor
 * Core Potential for Fast Reductions" (Carrasco, Vega, Navarro; arXiv
 * 1903.03640).  The problem solved is the arithmetic reduction of Section III,
 *      R(X) = sum_{i=1..n} x_i .
 *
 * Conventions that hold for every entry point
 *   - Plain C types only.  No exceptions cross this boundary; every function
 *     that can fail returns a redux_status (0 = success, negative = error).
 *   - "device pointer" = memory the current HIP device can read (hipMalloc,
 *     or PyTorch device tensors).  "host pointer" = ordinary process memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Work is enqueued asynchronously on it; the library never synchronises
 *     the device.  Results are valid once the stream has reached that point.
 *   - Inputs are never modified (the paper reduces in place inside X; this
 *     library does not).  Outputs are written only by kernels.
 *   - All argument checks happen before the first HIP call, so the error
 *     returns for bad arguments can be exercised on a machine without a GPU.
 *   - The library owns one small workspace (block partials, slots, ticket
 *     counters: 320 KiB) per (device, stream); it is created by the first
 *     call on that stream (one hipMalloc, so not during stream capture) and
 *     released by redux_shutdown().  Two calls on the same stream are ordered
 *     by the stream; calls on different streams use different workspaces, and host threads
 *     calling on different streams do not wait for each other's launches.
 *   - HIP graphs: a captured call holds the addresses of the library's buffers as they were at capture.
 *     They stay valid until redux_shutdown(); a graph captured before redux_shutdown() must not be
 *     replayed after it (capture it again).
 *   - Determinism: for a given input, device, variant and launch parameters
 *     the result is bit-identical from call to call (partials are combined in
 *     a fixed order; no floating-point atomics unless "finish" = 3 is asked for).
 */
#ifndef REDUX_H
#define REDUX_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Element type of the input array. */
typedef enum {
    REDUX_F16    = 0, /* IEEE binary16 in, binary32 MMA accumulation, one binary32 result (the paper's case) */
    REDUX_I8     = 1, /* int8 in, int32 MMA accumulation flushed to int64, one int64 result */
    REDUX_BF16   = 2, /* bfloat16 in (v_mfma_f32_16x16x32_bf16), binary32 accumulation and result */
    REDUX_F32    = 3, /* binary32 in (v_mfma_f32_16x16x4_f32, four K-slices per 16-byte load), binary32 result */
    REDUX_F8E4M3 = 4, /* OCP 8-bit E4M3 in (v_mfma_f32_16x16x32_fp8_fp8), binary32 accumulation and result */
    REDUX_F8E5M2 = 5  /* OCP 8-bit E5M2 in (v_mfma_f32_16x16x32_bf8_bf8), binary32 accumulation and result */
} redux_dtype;

typedef enum {
    REDUX_OK        =  0,
    REDUX_ERR_NULL  = -1, /* x is NULL with a non-empty input, or out is NULL */
    REDUX_ERR_DTYPE = -2, /* dtype is not a redux_dtype */
    REDUX_ERR_SIZE  = -3, /* nseg*seglen (or the byte count) overflows size_t / exceeds 2^62 */
    REDUX_ERR_ALIGN = -4, /* x not aligned to its element size, or out not aligned to its result size */
    REDUX_ERR_HIP   = -5, /* a HIP call failed; see redux_last_hip_error() */
    REDUX_ERR_NOMEM = -6, /* the workspace could not be allocated */
    REDUX_ERR_ALIAS = -7, /* out lies inside the input range */
    REDUX_ERR_PARAM = -8, /* unknown name or out-of-range value in redux_set_param / redux_set_variant */
    REDUX_ERR_SCRATCH = -9 /* redux_sum_static: the launch would write more than 2048 block partials, or the current
                              device's ordinal is 64 or higher */
} redux_status;

/* Which kernel family computes the sum. */
typedef enum {
    REDUX_VARIANT_AUTO    = 0, /* MFMA (as fast as CLASSIC on the flat sum, with the vector ALU idle; faster on segmented
                                  sums) -- except CLASSIC for the 8-bit floats, whose MFMAs drop bits, and for binary32,
                                  whose MMA needs four MFMAs per load and measures 5 % (flat sum) to 25 % (segmented
                                  sums) slower */
    REDUX_VARIANT_MFMA    = 1, /* MMA encoding: data tile x all-ones, accumulator chained through C   */
    REDUX_VARIANT_CLASSIC = 2  /* per-lane serial accumulation + wavefront tree (Section III)         */
} redux_variant;

/*
 * redux_sum -- R(X) = sum of n numbers (Section III, definition of the arithmetic
 * reduction; computed by the MMA scheme of Section IV-A, or by the classic tree
 * scheme of Section III when the classic variant is selected).
 *
 *   x      device pointer, read only, n contiguous elements of `dtype`; must be
 *          aligned to the element size only (1, 2 or 4 bytes).  May be NULL iff n == 0.
 *   n      number of elements; 0 is allowed and yields the empty sum 0.
 *   dtype  a redux_dtype.
 *   out    device pointer owned by the caller: one int64_t (I8, 8-byte aligned) or one float (every
 *          floating-point dtype, 4-byte aligned).  Must not lie inside [x, x + n*elemsize).
 *   stream hipStream_t or NULL.
 *
 * Floating-point dtypes: elements past the end of the last MMA tile count as zeros; binary32 partial
 * sums are combined across wavefronts and blocks in binary64 and rounded once to
 * binary32.  IEEE semantics for Inf/NaN; subnormal inputs are not flushed.
 * I8: the result is exact for any n that fits in device memory.
 * F8E4M3 / F8E5M2 with the MFMA family: the matrix unit keeps only 14 bits below the largest of the
 * eight products a lane contributes to one MFMA, so the error can reach 7 * 2^-14 (4.3e-4) of sum|x|
 * when values differ by more than 2^14 in magnitude; the classic family (the default for these two
 * dtypes) adds in binary32 and stays within 1e-4 of sum|x| like the others.
 */
int redux_sum(const void *x, size_t n, int dtype, void *out, void *stream);

/*
 * redux_sum_static -- redux_sum for callers that must not allocate: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, same kernels, same result bit for bit as redux_sum with
 * the same settings; the only difference is where the block partials and the ticket live: not in the per-stream
 * workspace that redux_sum allocates on first use, but in a static array in device memory (18 688 bytes per device,
 * held from the moment the library's code is loaded on a device until the process ends).
 *
 *   - Calls no hipMalloc, hipFree or any other allocating routine, on any call.  The first call on a device asks the
 *     runtime for the array's address on that device (hipGetSymbolAddress); make that call outside stream capture.
 *   - Limit: the launch may write at most 2048 block partials.  A default launch writes one per compute unit (256 on
 *     an MI355X); more than 2048 can only come from "blocks_per_cu" above 8 on such a device.  A call beyond the limit
 *     returns REDUX_ERR_SCRATCH and launches nothing ("max_grid" = 2048 keeps any setting inside it).  Device
 *     ordinals 0 .. 63.
 *   - The array is shared by every call on a device and keeps what the last call left in it.  Each call clears the
 *     ticket (and, where the finish reads the partials as they arrive, marks the slots of its blocks empty) with a
 *     small fill kernel ahead of the sum (no memset node, so it can be captured).  Calls on ONE stream are ordered by the stream and are safe back to back.  Calls that overlap on one
 *     device -- different streams, or different host threads on different streams -- race on the array and give
 *     wrong sums: use redux_sum there, which keeps one workspace per stream.
 */
int redux_sum_static(const void *x, size_t n, int dtype, void *out, void *stream);

/*
 * redux_sum_segmented -- nseg independent reductions: out[s] = sum_{k<seglen} x[s*seglen + k]
 * (the same R(X), applied to each array of a batch; the first MMA of Section IV-A
 * already yields independent row sums).
 *
 *   x       device pointer, row-major [nseg][seglen], read only; may be NULL iff nseg*seglen == 0.
 *   out     device pointer to nseg results (int64_t for I8, float for every floating-point dtype).
 *   nseg == 0 is a no-op; seglen == 0 writes nseg zeros.
 *
 *   x needs the alignment of its element type only, and seglen may be any number of elements.
 *
 * The kernel is chosen from (nseg, seglen, alignment); redux_plan_sum_segmented reports the choice.
 * Segments of up to 1 KiB (aligned powers of two: 4 KiB) are read as one contiguous stream, a group of 2^k lanes
 * per segment, and the constant operands of the two MMAs become 0/1 selection matrices, so that one MMA pair yields
 * many sums; longer segments, up to 28 KiB, are taken a run of up to sixteen at a time by one wavefront, which
 * streams the run as one contiguous piece of memory (first MMA with a one-column selector per segment, issued twice
 * for a load that holds a segment boundary; second MMA to fold the rows of all columns at once), with a leaner form
 * for aligned segments of exactly 1, 2, 4 or 8 KiB; segments of 28 KiB and more take a whole block each; a few long
 * segments are cut into pieces whose totals (in the workspace) a second kernel adds per segment.
 *
 * Reads outside x: segments that do not start or end on a 16-byte boundary are read as the 16-byte aligned vectors
 * that overlap them, so up to 15 bytes before x and after x + nseg*seglen*elemsize may be read (never written).  They
 * share a 16-byte granule, hence a page, with bytes of x, and they never enter a sum.
 * Non-finite values stay in their segment: an infinity or NaN affects out[s] of its own segment only.
 */
int redux_sum_segmented(const void *x, size_t nseg, size_t seglen, int dtype, void *out, void *stream);

/*
 * redux_sum_multipass -- the same sum computed exactly as Sections IV-A and IV-B lay the algorithm out,
 * level by level: the input is cut into contiguous groups of m*m numbers (m = 16 unless the "lit_m"
 * parameter says 4 or 32; int8: always 512 on the first level, the narrowest int8 tile being 16 x 32,
 * then 256); every group goes through both MMAs with C = 0
 * (D = A x 1, D' = 1 x D) and the thread in charge writes D'[1,1] into an array of partial sums in
 * global memory; each level is one kernel launch and the partial sums are the next level's input,
 * until one value is left (recurrence R_tc; ceil(log_{m*m} n) levels for binary16).  A last group that
 * is not full is zero padded.  Binary16: partial sums are binary32 at every level.  Int8: int32 inside
 * the first MMA, int64 partial sums, later levels in binary64 (exact below 2^53).
 *
 *   x, n, dtype, out, stream   as for redux_sum; dtype REDUX_F16 or REDUX_I8 only (REDUX_ERR_DTYPE otherwise).
 *   levels   host pointer or NULL; receives the number of levels (= kernel launches); 0 for n == 0.
 *
 * The arrays of partial sums (n/256 and n/65536 entries) are library-owned per (device, stream) and grow
 * on demand (hipMalloc, so not during stream capture; an outgrown buffer is kept until redux_shutdown, because a
 * captured graph may still hold its address).
 * This entry point exists to measure the algorithm as published against redux_sum, which chains the
 * accumulator through C and makes one pass; it is not the fast path.
 */
int redux_sum_multipass(const void *x, size_t n, int dtype, void *out, int *levels, void *stream);

/*
 * redux_mma_group_probe -- the two MMA steps of Section IV-A on ONE group, with both
 * result matrices written out (for checking the encoding, not for speed).
 *
 *   x      device pointer to `count` elements, count <= 512 (F16: a 16 x 32 operand A,
 *          filled row by row) or <= 1024 (I8: 16 x 64); missing elements are zeros.
 *   D      device pointer to 256 results, row-major 16 x 16: D = A x 1 + 0
 *          (float for F16, int32_t for I8).  Every column holds the 16 row sums of A.
 *   Dprime device pointer to 256 results, row-major 16 x 16: D' = 1 x D + 0
 *          (float for F16, double for I8 -- the int32 matrix is widened exactly and the
 *          second MMA runs in binary64).  Every entry is the sum of the group.
 */
int redux_mma_group_probe(const void *x, size_t count, int dtype, void *D, void *Dprime, void *stream);

/*
 * redux_calibration_copy -- plain device-to-device copy of nbytes (a multiple of 16; both pointers
 * 16-byte aligned) by a 16-byte-per-lane kernel.  Not part of the reduction: it is the kernel of
 * exactly known traffic (nbytes read, nbytes written) against which hardware byte counters are
 * calibrated when the reduction's HBM traffic is measured.
 */
int redux_calibration_copy(void *dst, const void *src, size_t nbytes, void *stream);

/*
 * Launch plans -- what the library would launch for a given problem, computed on the host with no HIP
 * call (so it works, and is tested, on a machine without a GPU).  `compute_units` stands for the device's
 * compute-unit count (256 on an MI355X); `x_address` is the address the input would have (only its low
 * four bits matter: alignment decides head/tail elements and whether the short-segment kernel applies).
 * The current redux_set_param settings apply.
 */
typedef enum {
    REDUX_KERNEL_FLAT   = 0, /* redux_sum */
    REDUX_KERNEL_ROWS   = 1, /* redux_sum_segmented, sixteen short segments per wavefront */
    REDUX_KERNEL_WAVE   = 2, /* redux_sum_segmented, one wavefront per segment */
    REDUX_KERNEL_PIECES = 3, /* redux_sum_segmented, long segments cut into pieces, one wavefront per piece, + a per-segment finish
                                kernel: only with "seg_block_bytes" = 0 (from 32 KiB on) or "seg_parts" above 1 */
    REDUX_KERNEL_TILES  = 4, /* redux_sum_segmented, segments of exactly 1, 2, 4 or 8 KiB: one wavefront per
                                segment with the next segment's loads issued ahead */
    REDUX_KERNEL_BLOCK  = 5, /* redux_sum_segmented, long segments: one block per segment or per piece of one
                                (parts > 1: the piece totals are added per segment, see "seg_finish") */
    REDUX_KERNEL_SHORT  = 6, /* redux_sum_segmented, 16-byte aligned segments of 16, 32, ... 1024 bytes (MMA family, except
                                binary32: ... 4096 bytes): the array is
                                read as one contiguous stream and 0/1 selection matrices in the two MMAs (or a
                                shortened lane butterfly) yield every segment's sum */
    REDUX_KERNEL_RAGGED = 7, /* redux_sum_segmented, any other segment of up to 1008 bytes: the same kernel, each group
                                of `vectors` lanes reading the aligned vectors that overlap its segment */
    REDUX_KERNEL_RUNS   = 8  /* redux_sum_segmented, segments from 1009 to 28671 bytes (classic family: 7999; and from 32769 to 36863 when there
                                are many) of any length and alignment: one
                                wavefront streams a run of `vectors` (1 .. 16) consecutive whole segments, every lane of
                                every load busy; each segment of the run owns one column of the MMA accumulator */
} redux_kernel;

typedef struct {
    int      kernel;   /* a redux_kernel */
    int      unroll;   /* 16-byte loads in flight per lane (ROWS: per row group) */
    unsigned grid;     /* 256-thread blocks of the main kernel */
    int      finish;   /* FLAT: the value of "finish" that is used (2 = second kernel; 4, 5, 6 = in the same kernel); segmented:
                          0 if parts == 1, else where the piece totals meet: 2 = second kernel, 5 (int8) / 6 = same kernel */
    uint64_t parts;    /* pieces per segment (above 1 only for PIECES and BLOCK) */
    uint64_t part_len; /* elements per piece */
    unsigned head;     /* FLAT: elements before the first 16-byte aligned vector */
    unsigned tail;     /* FLAT: elements after the last whole vector */
    uint64_t vectors;  /* FLAT: whole 16-byte vectors; ROWS: vectors per segment */
    unsigned chain;    /* loop iterations between folds of the MMA accumulators: "max_chain", lowered for int8 so that
                          no int32 accumulator can pass 2^31 whatever the input holds */
} redux_plan;

int redux_plan_sum(size_t n, int dtype, uintptr_t x_address, int compute_units, redux_plan *plan);
int redux_plan_sum_segmented(size_t nseg, size_t seglen, int dtype, uintptr_t x_address, int compute_units,
                             redux_plan *plan); /* nseg, seglen >= 1 */
/* The slabs (block-sized runs of unroll x 4 KiB) that block `block` of `grid` reads under `layout`:
 * start, start + stride, ... (count of them).  Over all blocks they cover 0 .. nslab-1 exactly once. */
int redux_plan_block_slabs(int layout, uint64_t nslab, uint64_t grid, uint64_t block,
                           uint64_t *start, uint64_t *stride, uint64_t *count);
/* The segments that wavefront `wave` (0 .. 3) of block `block` of `grid` sums in the RUNS kernel under `layout`:
 * `rounds` whole runs of per_run (1 .. 16) segments starting at first, first + stride, ..., then one last run of
 * tail_count (0 .. per_run) segments starting at tail_first.  Over all wavefronts they cover 0 .. nseg-1 exactly once,
 * and no two wavefronts differ by more than one run of the same length plus one segment. */
int redux_plan_run_share(int layout, uint64_t nseg, unsigned per_run, uint64_t grid, uint64_t block, unsigned wave,
                         uint64_t *first, uint64_t *stride, uint64_t *rounds, uint64_t *tail_first, unsigned *tail_count);

/* Select the kernel family for subsequent calls (process-wide). Also read once from the
 * environment variable REDUX_VARIANT = auto | mfma | classic. */
int redux_set_variant(int variant);
int redux_get_variant(void);
/* The family (REDUX_VARIANT_MFMA or _CLASSIC) that a redux_sum (segmented == 0) or redux_sum_segmented (!= 0) call on
 * `dtype` runs with under the current setting; a negative redux_status for an unknown dtype. */
int redux_resolved_variant(int dtype, int segmented);

/*
 * Launch parameters (process-wide; for tuning and tests).  Names:
 *   "blocks_per_cu"     1..16   256-thread blocks per compute unit for the flat sum (default 1)
 *   "seg_blocks_per_cu" 0..16   the same for the segmented sum; 0 = from the segment length (default 0)
 *   "max_grid"          1..16384 upper limit on the number of blocks (default 16384)
 *   "unroll"            0,1,2,4,8   16-byte loads in flight per lane; 0 = chosen from the size (default 0)
 *   "nontemporal"       0/1     use non-temporal (streaming) loads (default 1)
 *   "pause"             -1..64  flat sum: every loop iteration of a wavefront ends with this many 64-cycle sleeps;
 *                               -1 = the measured best (8 for the MMA family on binary16, bfloat16 and int8 runs of
 *                               512 MiB and more, else 0) (default -1)
 *   "stagger"           0..64   flat sum, blocks that run at least 32 loop iterations (256 MiB and up): wavefront w of a
 *                               block starts w x stagger x 64 cycles late, worth 1-2 us per call (default 4)
 *   "rows_max_vec"      0..64   segmented sum, binary16 and int8, only where "seg_short" / "seg_ragged" do not apply:
 *                               segments of at most this many 16-byte vectors (and 16-byte aligned) take the
 *                               sixteen-segments-per-wavefront kernel; 0 = never (default 64)
 *   "seg_block_bytes"   0..2^40 segmented sum: segments of at least this many bytes take one 256-thread block
 *                               each (or one per piece) and are streamed like the flat sum; 0 = never (default 28672: measured, from
 *                               there on a block is ahead of one wavefront per segment)
 *   "seg_short"         0/1     segmented sum: 16-byte aligned segments of a power-of-two size from 16 to 1024 bytes (4096
 *                               with the MMA family, binary32 excepted) take the contiguous-stream kernel (default 1)
 *   "seg_ragged"        0/1     segmented sum: every other segment of up to 1008 bytes takes that kernel's ragged form
 *                               (default 1)
 *   "seg_runs"          0/1     segmented sum: segments of more than 1008 and at most "seg_runs_max" bytes (and less than
 *                               "seg_block_bytes") that are not cut into pieces take the run-of-segments kernel; 0 = one
 *                               wavefront per segment instead (default 1)
 *   "seg_runs_max"      0, 1009..2^18  largest segment in bytes that kernel takes; 0 = by family (default): 28671 for the
 *                               MMA family's rolling form (up to where one block per segment takes over), 7999 for the
 *                               run-by-run forms (measured: from 8000 bytes on one wavefront per segment is ahead of them)
 *   "seg_runs_long"     0..2^18 that kernel also takes segments of more than 32768 bytes up to this size when there are
 *                               at least eight per compute unit (default 36863: measured, one block per segment leaves
 *                               most of its second 32 KiB pass idle there; 0 = none)
 *   "seg_runs_stream"   0/1     that kernel: 1 = every register is loaded again, with what the wavefront's next
 *                               iteration (of this run or of its next one) needs, right after it has been used, so the
 *                               loads stay in flight across the end of a run; 0 = load, work, fold, store, run by run
 *                               (default 1: measured 2-4 % ahead; on the same grid with the same run length the results are the same bit for bit)
 *   "seg_balance"       0..99   segmented sum, one block per segment: into how many pieces (a power of two, of at least 64 KiB)
 *                               a segment is cut.  1 = the number with the lowest modelled time: whole rounds of pieces
 *                               over the grid at full time, a last round that fills a fraction f of the grid at sqrt(f) of
 *                               one (at least half), plus what adding the piece totals costs; 2 .. 99 = the first number
 *                               that uses that percentage of its rounds' slots; 0 = only as many as it takes to have
 *                               two pieces per compute unit (default 1)
 *   "seg_run_len"       0..16   that kernel: segments per run; 0 = the length with the lowest cost per wavefront
 *                               (iterations, of which a run's last is partly idle, plus a fixed cost per run; every
 *                               wavefront takes the same number of whole runs and a share of what is left) (default 0)
 *   "seg_short_pipe"    -1,0,1  that kernel: 1 = every register is reloaded from the block's next 32 KiB as soon as it has
 *                               been consumed, 0 = plain load-then-work loop, -1 = the measured best for the shape (default -1)
 *   "seg_tiles"         0/1     segmented sum: 16-byte aligned segments of exactly 1, 2, 4 or 8 KiB, at least
 *                               four per compute unit, take the pipelined one-wavefront-per-segment kernel (default 1)
 *   "seg_parts"         0..4096 segmented sum: pieces a long segment is cut into; 0 = from the
 *                               shape (default 0); ignored if nseg * pieces exceeds the workspace (16384)
 *   "seg_finish"        -1,0,1  segmented sum, long segments cut into pieces, one block per piece: 1 = the block of a
 *                               segment that arrives last adds the segment's piece totals in the same kernel (floating
 *                               point: totals in slots that read empty between launches, arrivals counted by a ticket
 *                               per segment; int8: one 64-bit atomic addition per piece that adds and counts), 0 = a
 *                               second kernel adds them; same order, same bits.  -1 = the measured best: the same
 *                               kernel wherever there is a block for every piece (a block that goes on to another
 *                               piece would wait for its ticket first).  Up to 28 segments of 32 or more pieces
 *                               count their arrivals in two levels, as "finish" 7 and 8 do (default -1)
 *   "compensated"       0/1     redux_sum, binary16, MMA family: the first MMA runs with C = 0 and its row sums are added to the
 *                               running sums with a two-sum on the vector ALU, the lost parts kept in a second
 *                               accumulator (for the precision study: it buys nothing once chains are bounded, and costs
 *                               vector instructions) (default 0)
 *   "lit_m"             4,16,32 redux_sum_multipass, binary16: linear size m of the MMA matrices (default 16)
 *   "lit_half"          0/1     redux_sum_multipass, binary16, m = 16 (REDUX_ERR_PARAM from the call otherwise): the result of
 *                               each of the two MMAs is rounded to binary16 and the partial sums are stored as binary16,
 *                               Section I-B's half-precision multiply-accumulate and Section IV-B's results written back
 *                               into X, both taken literally; the
 *                               final value is that binary16 number widened (an infinity once a partial sum passes
 *                               65504).  For measuring what that reading costs in accuracy, nothing else (default 0)
 *   "lit_unroll"        0,1,2,4,8,16  redux_sum_multipass: wavefront steps per loop iteration; 0 = the
 *                               measured best for the shape (default 0)
 *   "lit_blocks_per_cu" 0..16   redux_sum_multipass: 256-thread blocks per compute unit; 0 = the measured
 *                               best for the shape (default 0)
 *   "layout"            0..2    which part of the array a block reads: 0 = blocks interleaved over the
 *                               whole array, 1 = one contiguous share per block, 2 = one contiguous
 *                               eighth per accelerator die, interleaved among that die's blocks (default 2)
 *   "finish"            -1..8   how block partials become the result: 0/1/4 = the block that arrives last
 *                               sums them in the same kernel (0: acquire+release on every block's ticket,
 *                               1: release only, acquire in the last block, 4: no release fence at all -- the
 *                               partial is published by a device-scope atomic exchange whose completion the
 *                               ticket waits for), 2 = a second one-block kernel
 *                               on the same stream, 3 = every block adds its total to the result atomically
 *                               (the atomic scheme of Section II, for comparison: a fill kernel clears the
 *                               result first, and floating-point results then depend on the order of arrival
 *                               in their last bits), 5 = int8 only: every block adds its total to one 64-bit word
 *                               with a single atomic addition that also counts the blocks (sum above bit 15,
 *                               count below), and the block that completes the count writes the result: exact,
 *                               independent of the order, no partials and no clearing kernel (other types: taken
 *                               as 4), 6 = floating point only: as 4, but no block waits for its partial to have
 *                               arrived before it draws its ticket; the partials go to slots that read empty
 *                               between launches, and the last block reads each slot until it is filled, then
 *                               empties it again (grids above 2048 blocks and int8: taken as 4),
 *                               7 = as 6 and 8 = as 5, with the arrivals counted in two levels: the blocks of an
 *                               accelerator die (block b runs on die b mod 8) meet at a word of the die's own, the
 *                               last of each die at the common one, so that no word has more than gridDim / 8
 *                               read-modify-writes queueing at it,
 *                               -1 = the measured best for the input: 5 or 8 for int8, else 6 or 7; the two-level
 *                               forms for inputs above 2 MiB and below 256 MiB, whose blocks all arrive within a
 *                               microsecond (default -1)
 *   "max_chain"         1..65536 loop iterations between folds of the MMA accumulators into the wide
 *                               per-wavefront total (bounds binary32 chain length).  For int8 the library lowers
 *                               it where needed so that an int32 accumulator stays below 2^31 for any input
 *                               (redux_plan.chain reports the value used)
 * Returns REDUX_ERR_PARAM for an unknown name or a value out of range.
 */
int redux_set_param(const char *name, long value);
long redux_get_param(const char *name); /* LONG_MIN for an unknown name */

const char *redux_strerror(int status);
int redux_last_hip_error(void); /* raw hipError_t behind the last REDUX_ERR_HIP/NOMEM on this thread */
void redux_shutdown(void);      /* frees every workspace; the library can be used again afterwards   */
const char *redux_version(void);

#ifdef __cplusplus
}
#endif
#endif /* REDUX_H */
