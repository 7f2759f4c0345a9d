// redux_api.hip -- the C ABI of libredux (see include/redux.h): argument checks, variant and
// launch-shape selection, workspace ownership, kernel launches.  No compute happens on the host.
#include "../../include/redux.h"
#include "redux_kernels.h"
#include "redux_literal.h"
#include "redux_short.h"
#include "redux_runs.h"

#include <climits>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <map>
#include <mutex>
#include <utility>
#include <vector>

using namespace redux;

// ---- scratch memory of redux_sum_static: nothing is ever allocated for it ------------------------------------------
// Block partials (8 bytes each) followed by the ticket on its own 256-byte line.  Every device the library runs on
// holds its own copy of this array from the moment the code object is loaded until the process ends.
constexpr int kScratchSlots = 2048;                              // block partials a launch may write
constexpr size_t kScratchTicketOffset = (size_t)kScratchSlots * sizeof(u64);
constexpr size_t kScratchLeavesOffset = kScratchTicketOffset + 256;   // eight second-level tickets, 256 bytes apart
constexpr size_t kScratchBytes = kScratchLeavesOffset + 8 * 256;      // 18 688 bytes
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {

// ---- process-wide settings --------------------------------------------------------------------
struct Settings {
    int variant = REDUX_VARIANT_AUTO;
    long blocks_per_cu = 1;
    long seg_blocks_per_cu = 0;   // 0 = from the segment length
    long unroll = 0;          // 0 = from the problem size
    long nontemporal = 1;
    long max_chain = 256;
    long max_grid = kMaxGrid;
    long layout = 2;
    long rows_max_vec = 64;       // short-segment kernel up to this many 16-byte vectors per segment (0 = off)
    long seg_parts = 0;           // 0 = pieces per long segment chosen from the shape
    long stagger = 4;             // flat sum: wavefront w of a block starts w x stagger x 64 cycles late (long runs only)
    long seg_short_pipe = -1;     // that kernel: 1 = refill each register as soon as it is consumed, 0 = plain loop, -1 = measured best
    long seg_ragged = 1;          // use that kernel's ragged form for all other segments of up to 1008 bytes
    long seg_short = 1;           // use the contiguous-stream kernel for aligned power-of-two segments of 16 B .. 1 KiB
    long seg_tiles = 1;           // use the pipelined kernel for segments of 1, 2, 4 or 8 whole tiles
    long seg_runs = 1;            // use the run-of-segments kernel for segments above 1008 bytes that are not cut into pieces
    long seg_run_len = 0;         // segments per run (0 = from the shape)
    long seg_runs_max = 0;        // largest segment (bytes) that kernel takes (0 = by family: 28671 MMA rolling form, else 7999)
    long seg_runs_stream = 1;     // run-of-segments kernel: 1 = every register reloaded right after its use
    long seg_balance = 1;         // long segments are cut into more pieces when the last round of pieces would be mostly empty
    long seg_runs_long = 36863;   // it also takes segments of more than 32 KiB up to this size (0 = none)
    long seg_block_bytes = 28672; // segments of at least this many bytes take one block each (0 = never); measured: from
                                  // 28 KiB on a block is ahead of one wavefront per segment (7.05 against 6.7 TB/s), at 24 KiB behind
    long lit_unroll = 0;          // groups per wavefront iteration of the level-by-level form (0 = per dtype)
    long lit_blocks_per_cu = 0;
    long lit_m = 16;              // linear size m of the MMA matrices of the level-by-level form
    long compensated = 0;         // flat sum, binary16, MMA family: two-sum compensated chain (precision study)
    long lit_half = 0;            // level-by-level form, binary16, m = 16: both MMA results and the partial sums in binary16
    long finish = -1;             // -1 = from the input size
    long seg_finish = -1;         // segments cut into pieces, one block each: 1 = the last block of a segment to arrive adds its piece
                                  // totals, 0 = a second kernel does, -1 = measured best
    long pause = -1;              // flat sum: 64-cycle sleeps at the end of every loop iteration (-1 = measured best)
};
Settings g_set;
std::once_flag g_env_once;
std::mutex g_mu;

thread_local int t_last_hip = 0;

void read_env()
{
    const char *v = std::getenv("REDUX_VARIANT");
    if (!v) return;
    if (!std::strcmp(v, "mfma")) g_set.variant = REDUX_VARIANT_MFMA;
    else if (!std::strcmp(v, "classic")) g_set.variant = REDUX_VARIANT_CLASSIC;
    else g_set.variant = REDUX_VARIANT_AUTO;
}

int hip_fail(hipError_t e, int status = REDUX_ERR_HIP)
{
    t_last_hip = (int)e;
    return status;
}

// ---- per (device, stream) workspace -----------------------------------------------------------
struct Workspace {
    u64 *partials = nullptr;    // kMaxGrid slots
    unsigned *ticket = nullptr; // behind the partials, on its own 256-byte line
    u64 *slots = nullptr;       // behind the ticket: kMaxGrid slots that read empty between launches (flat sum, finish 6 and 7: the
                                // first kWorkspaceSlots; segments cut into pieces that finish in the kernel: one per piece)
    u64 *counted = nullptr;     // behind the slots: 64 KiB of words that read zero between launches.  Flat sum, finish 7 and 8: the
                                // eight second-level tickets, a 256-byte line each.  Segments cut into pieces: a word per segment
                                // (floating point: its ticket; int8: its counted sum), a line apart while they fit; nine lines per
                                // segment where the arrivals are counted in two levels
};
constexpr unsigned kWorkspaceSlots = 2048;
constexpr size_t kTicketOffset = (size_t)kMaxGrid * sizeof(u64);
constexpr size_t kSlotsOffset = kTicketOffset + 256;
constexpr size_t kCountedOffset = kSlotsOffset + (size_t)kMaxGrid * sizeof(u64);
constexpr size_t kWorkspaceBytes = kCountedOffset + (size_t)(kMaxGrid / 2) * sizeof(u64);

std::map<std::pair<int, hipStream_t>, Workspace> g_ws;

// In host code `scratch` is only a handle for the symbol, not an address in device memory: what kernels and fills get
// is the address hipGetSymbolAddress returns for the device that is current, asked for once per device and kept here.
constexpr int kStaticDevices = 64;
void *g_scratch_ptr[kStaticDevices] = {};
int g_static_cus[kStaticDevices] = {};
std::map<int, int> g_cus;

int device_cus(int dev, int *cus)
{
    auto it = g_cus.find(dev);
    if (it == g_cus.end()) {
        int n = 0;
        hipError_t e = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess) return hip_fail(e);
        if (n <= 0) n = 1;
        it = g_cus.emplace(dev, n).first;
    }
    *cus = it->second;
    return REDUX_OK;
}

int get_workspace(int dev, hipStream_t st, Workspace *out)
{
    auto key = std::make_pair(dev, st);
    auto it = g_ws.find(key);
    if (it == g_ws.end()) {
        void *p = nullptr;
        hipError_t e = hipMalloc(&p, kWorkspaceBytes);
        if (e != hipSuccess) return hip_fail(e, REDUX_ERR_NOMEM);
        Workspace w;
        w.partials = (u64 *)p;
        w.ticket = (unsigned *)((char *)p + kTicketOffset);
        // the ticket must read zero before the first launch; a fill kernel on the caller's
        // stream keeps the ordering without a device-wide synchronisation
        w.slots = (u64 *)((char *)p + kSlotsOffset);
        w.counted = (u64 *)((char *)p + kCountedOffset);
        hipLaunchKernelGGL(empty_slots_kernel, dim3(1), dim3(256), 0, st, w.slots, (unsigned)kMaxGrid, w.ticket, 64u, (unsigned *)nullptr);
        hipLaunchKernelGGL(fill_zero_words_kernel, dim3(kMaxGrid / 256), dim3(256), 0, st, (unsigned *)w.counted, (unsigned)kMaxGrid);
        e = hipGetLastError();
        if (e != hipSuccess) { (void)hipFree(p); return hip_fail(e); }
        it = g_ws.emplace(key, w).first;
    }
    *out = it->second;
    return REDUX_OK;
}

// ---- per (device, stream) buffers for the arrays of partial sums of the level-by-level form ----------
struct LevelBuffers {
    void *buf[2] = {nullptr, nullptr};
    size_t bytes[2] = {0, 0};
};
std::map<std::pair<int, hipStream_t>, LevelBuffers> g_levels;

// Buffers that were outgrown.  A captured graph holds the addresses that were current when it was captured, so nothing
// is freed (and the device is never waited for) before redux_shutdown.
std::vector<void *> g_retired;

int get_level_buffers(int dev, hipStream_t st, size_t bytes0, size_t bytes1, LevelBuffers *out)
{
    LevelBuffers &lb = g_levels[std::make_pair(dev, st)];
    const size_t want[2] = {bytes0, bytes1};
    for (int i = 0; i < 2; ++i) {
        if (lb.bytes[i] >= want[i]) continue;
        // at least double, so that a slowly growing input retires a bounded total (less than the final size)
        const size_t bytes = want[i] > 2 * lb.bytes[i] ? want[i] : 2 * lb.bytes[i];
        void *p = nullptr;
        hipError_t e = hipMalloc(&p, bytes);
        if (e != hipSuccess) return hip_fail(e, REDUX_ERR_NOMEM);
        if (lb.buf[i]) g_retired.push_back(lb.buf[i]);
        lb.buf[i] = p;
        lb.bytes[i] = bytes;
    }
    *out = lb;
    return REDUX_OK;
}

template <int M, int U>
void launch_literal_f16(bool first, bool fast, const void *in, u64 n, void *outp, unsigned grid, hipStream_t st)
{
    if (first) {
        if (fast) hipLaunchKernelGGL((literal_level_kernel<M, true, U, true>), dim3(grid), dim3(kBlock), 0, st, in, n, outp, 1);
        else      hipLaunchKernelGGL((literal_level_kernel<M, true, U, false>), dim3(grid), dim3(kBlock), 0, st, in, n, outp, 1);
    } else {
        // (sixteen 32 x 32 tiles of binary32 per wavefront step would not fit the register file; the kernel loops over
        // its own batches, so any grid fits any U)
        constexpr int UL = (M == 32 && U > 8) ? 8 : U;
        hipLaunchKernelGGL((literal_level_kernel<M, false, UL, true>), dim3(grid), dim3(kBlock), 0, st, in, n, outp, 1);
    }
}

// the binary16-throughout form (m = 16): every level reads binary16; `last` says whether outp is the caller's binary32 result
template <int U>
void launch_literal_half(bool fast, bool last, const void *in, u64 n, void *outp, unsigned grid, hipStream_t st)
{
    if (fast) hipLaunchKernelGGL((literal_level_kernel<16, true, U, true, true>), dim3(grid), dim3(kBlock), 0, st, in, n, outp, last ? 1 : 0);
    else      hipLaunchKernelGGL((literal_level_kernel<16, true, U, false, true>), dim3(grid), dim3(kBlock), 0, st, in, n, outp, last ? 1 : 0);
}

template <int U>
void launch_literal_i8(bool first, bool fast, const void *in, u64 n, void *outp, unsigned grid, hipStream_t st)
{
    if (first) {
        if (fast) hipLaunchKernelGGL((literal_level_i8_kernel<U, true>), dim3(grid), dim3(kBlock), 0, st, (const signed char *)in, n, (i64 *)outp);
        else      hipLaunchKernelGGL((literal_level_i8_kernel<U, false>), dim3(grid), dim3(kBlock), 0, st, (const signed char *)in, n, (i64 *)outp);
    } else {
        hipLaunchKernelGGL((literal_level_i64_kernel<U>), dim3(grid), dim3(kBlock), 0, st, (const i64 *)in, n, (i64 *)outp);
    }
}

// ---- kernel dispatch ----------------------------------------------------------------------------
template <class F, int U>
void launch_flat_u(bool nt, unsigned grid, hipStream_t st, const FlatArgs &a)
{
    if (nt) hipLaunchKernelGGL((sum_flat_kernel<F, U, true>), dim3(grid), dim3(kBlock), 0, st, a);
    else    hipLaunchKernelGGL((sum_flat_kernel<F, U, false>), dim3(grid), dim3(kBlock), 0, st, a);
}

template <class F>
void launch_flat(int unroll, bool nt, unsigned grid, hipStream_t st, const FlatArgs &a)
{
    switch (unroll) {
    case 8: launch_flat_u<F, 8>(nt, grid, st, a); break;
    case 4: launch_flat_u<F, 4>(nt, grid, st, a); break;
    case 2: launch_flat_u<F, 2>(nt, grid, st, a); break;
    default: launch_flat_u<F, 1>(nt, grid, st, a); break;
    }
}

template <class F, int U>
void launch_seg_u(bool nt, unsigned grid, hipStream_t st, const SegArgs &a)
{
    if (nt) hipLaunchKernelGGL((sum_segmented_kernel<F, U, true>), dim3(grid), dim3(kBlock), 0, st, a);
    else    hipLaunchKernelGGL((sum_segmented_kernel<F, U, false>), dim3(grid), dim3(kBlock), 0, st, a);
}

template <class F>
void launch_seg(int unroll, bool nt, unsigned grid, hipStream_t st, const SegArgs &a)
{
    switch (unroll) {
    case 8: launch_seg_u<F, 8>(nt, grid, st, a); break;
    case 4: launch_seg_u<F, 4>(nt, grid, st, a); break;
    case 2: launch_seg_u<F, 2>(nt, grid, st, a); break;
    default: launch_seg_u<F, 1>(nt, grid, st, a); break;
    }
}

// ---- argument checks shared by the entry points ---------------------------------------------------
// element size and result size of a dtype; 0 for an unknown dtype
size_t elem_size_of(int dtype)
{
    switch (dtype) {
    case REDUX_F16: case REDUX_BF16: return 2;
    case REDUX_I8: case REDUX_F8E4M3: case REDUX_F8E5M2: return 1;
    case REDUX_F32: return 4;
    default: return 0;
    }
}
size_t out_size_of(int dtype) { return dtype == REDUX_I8 ? 8 : 4; }

int check_common(const void *x, size_t count, int dtype, const void *out, size_t nout, size_t *elem_size)
{
    const size_t es = elem_size_of(dtype);
    if (es == 0) return REDUX_ERR_DTYPE;
    const size_t os = out_size_of(dtype);
    if (count > ((size_t)1 << 62) / es) return REDUX_ERR_SIZE;
    if (!out && nout) return REDUX_ERR_NULL;
    if (!x && count) return REDUX_ERR_NULL;
    if ((uintptr_t)x % es) return REDUX_ERR_ALIGN;
    if ((uintptr_t)out % os) return REDUX_ERR_ALIGN;
    if (count && nout) {
        uintptr_t xb = (uintptr_t)x, xe = xb + count * es;
        uintptr_t ob = (uintptr_t)out, oe = ob + nout * os;
        if (ob < xe && xb < oe) return REDUX_ERR_ALIAS;
    }
    *elem_size = es;
    return REDUX_OK;
}

// the kernel family of (dtype, variant), handed to a generic callable
template <class Fn>
void with_flat_family(int dtype, bool mfma, Fn &&fn)
{
    switch (dtype) {
    case REDUX_F16:    if (mfma) fn(FloatMfmaT<kF16, 4>());  else fn(FloatClassic<kF16>());  break;
    case REDUX_BF16:   if (mfma) fn(FloatMfmaT<kBF16, 4>()); else fn(FloatClassic<kBF16>()); break;
    case REDUX_F32:    if (mfma) fn(FloatMfmaT<kF32, 4>());  else fn(FloatClassic<kF32>());  break;
    case REDUX_F8E4M3: if (mfma) fn(FloatMfmaT<kE4M3, 4>()); else fn(FloatClassic<kE4M3>()); break;
    case REDUX_F8E5M2: if (mfma) fn(FloatMfmaT<kE5M2, 4>()); else fn(FloatClassic<kE5M2>()); break;
    default:           if (mfma) fn(I8Mfma());               else fn(I8Classic());           break;
    }
}

template <class Fn>
void with_seg_family(int dtype, bool mfma, Fn &&fn)
{
    switch (dtype) {
    case REDUX_F16:    if (mfma) fn(FloatMfmaT<kF16, 1>());  else fn(FloatClassic<kF16>());  break;
    case REDUX_BF16:   if (mfma) fn(FloatMfmaT<kBF16, 1>()); else fn(FloatClassic<kBF16>()); break;
    case REDUX_F32:    if (mfma) fn(FloatMfmaT<kF32, 1>());  else fn(FloatClassic<kF32>());  break;
    case REDUX_F8E4M3: if (mfma) fn(FloatMfmaT<kE4M3, 1>()); else fn(FloatClassic<kE4M3>()); break;
    case REDUX_F8E5M2: if (mfma) fn(FloatMfmaT<kE5M2, 1>()); else fn(FloatClassic<kE5M2>()); break;
    default:           if (mfma) fn(I8MfmaSeg());            else fn(I8Classic());           break;
    }
}

template <class Fn>
void with_short_family(int dtype, Fn &&fn)
{
    switch (dtype) {
    case REDUX_F16:    fn(ShortFloat<kF16>());  break;
    case REDUX_BF16:   fn(ShortFloat<kBF16>()); break;
    case REDUX_F32:    fn(ShortFloat<kF32>());  break;
    case REDUX_F8E4M3: fn(ShortFloat<kE4M3>()); break;
    case REDUX_F8E5M2: fn(ShortFloat<kE5M2>()); break;
    default:           fn(ShortI8());           break;
    }
}

// The family a call runs with.  `flat`: redux_sum (otherwise redux_sum_segmented).
int effective_variant(const Settings &S, int dtype, bool flat = false)
{
    int v = S.variant;
    if (v != REDUX_VARIANT_AUTO) return v;
    // The 8-bit floating-point MFMAs align the eight products of a lane to the largest of them and keep
    // only 14 bits below it (measured), so small terms next to a large one are dropped: up to
    // 7 * 2^-14 of sum|x|, above the 1e-4 this library promises.  Their default is the classic family.
    if (dtype == REDUX_F8E4M3 || dtype == REDUX_F8E5M2) return REDUX_VARIANT_CLASSIC;
    // Everything else: the MMA family.  Flat sums of 1-2 GiB: both families move the same bytes in the same time
    // (interleaved runs of 100 calls: 289.8 +- 0.4 against 289.2 +- 0.3 us on 2 GiB of binary16), so the tie goes to the
    // family that keeps the vector ALU idle (2.9 % against 21.5 % busy); after an idle period the MMA family is also
    // 3 % faster for the first forty calls (294 against 304 us).  Segmented sums: as fast (8 KiB segments) or 5-30 %
    // faster (short and ragged segments).  Binary32 is the exception: its MMA takes four K-slices, hence four 8-pass
    // MFMAs, per 16-byte load, and measures 5 % behind the classic family on the flat sum (306 against 290 us on 2 GiB)
    // and up to 25 % behind on segmented sums (2 KiB segments 5.5 against 7.0 TB/s, 1.5 KB 4.9 against 6.7, 32 KiB 5.7
    // against 7.1; ahead only on 16-byte aligned power-of-two segments of 64 B - 1 KiB, by 3-6 %).
    (void)flat;
    if (dtype == REDUX_F32) return REDUX_VARIANT_CLASSIC;
    return REDUX_VARIANT_MFMA;
}

long *param_slot(const char *name, long *lo, long *hi)
{
    if (!name) return nullptr;
    if (!std::strcmp(name, "blocks_per_cu")) { *lo = 1; *hi = 16; return &g_set.blocks_per_cu; }
    if (!std::strcmp(name, "seg_blocks_per_cu")) { *lo = 0; *hi = 16; return &g_set.seg_blocks_per_cu; }
    if (!std::strcmp(name, "unroll")) { *lo = 0; *hi = 8; return &g_set.unroll; }
    if (!std::strcmp(name, "nontemporal")) { *lo = 0; *hi = 1; return &g_set.nontemporal; }
    if (!std::strcmp(name, "max_chain")) { *lo = 1; *hi = 65536; return &g_set.max_chain; }
    if (!std::strcmp(name, "max_grid")) { *lo = 1; *hi = kMaxGrid; return &g_set.max_grid; }
    if (!std::strcmp(name, "rows_max_vec")) { *lo = 0; *hi = 64; return &g_set.rows_max_vec; }
    if (!std::strcmp(name, "seg_block_bytes")) { *lo = 0; *hi = (long)1 << 40; return &g_set.seg_block_bytes; }
    if (!std::strcmp(name, "stagger")) { *lo = 0; *hi = 64; return &g_set.stagger; }
    if (!std::strcmp(name, "seg_short_pipe")) { *lo = -1; *hi = 1; return &g_set.seg_short_pipe; }
    if (!std::strcmp(name, "seg_ragged")) { *lo = 0; *hi = 1; return &g_set.seg_ragged; }
    if (!std::strcmp(name, "seg_short")) { *lo = 0; *hi = 1; return &g_set.seg_short; }
    if (!std::strcmp(name, "seg_runs")) { *lo = 0; *hi = 1; return &g_set.seg_runs; }
    if (!std::strcmp(name, "seg_runs_max")) { *lo = 0; *hi = 1 << 18; return &g_set.seg_runs_max; }
    if (!std::strcmp(name, "seg_runs_long")) { *lo = 0; *hi = 1 << 18; return &g_set.seg_runs_long; }
    if (!std::strcmp(name, "seg_balance")) { *lo = 0; *hi = 99; return &g_set.seg_balance; }
    if (!std::strcmp(name, "seg_runs_stream")) { *lo = 0; *hi = 1; return &g_set.seg_runs_stream; }
    if (!std::strcmp(name, "seg_run_len")) { *lo = 0; *hi = 16; return &g_set.seg_run_len; }
    if (!std::strcmp(name, "seg_tiles")) { *lo = 0; *hi = 1; return &g_set.seg_tiles; }
    if (!std::strcmp(name, "seg_parts")) { *lo = 0; *hi = 4096; return &g_set.seg_parts; }
    if (!std::strcmp(name, "seg_finish")) { *lo = -1; *hi = 1; return &g_set.seg_finish; }
    if (!std::strcmp(name, "compensated")) { *lo = 0; *hi = 1; return &g_set.compensated; }
    if (!std::strcmp(name, "lit_half")) { *lo = 0; *hi = 1; return &g_set.lit_half; }
    if (!std::strcmp(name, "lit_m")) { *lo = 4; *hi = 32; return &g_set.lit_m; }
    if (!std::strcmp(name, "lit_unroll")) { *lo = 0; *hi = 16; return &g_set.lit_unroll; }
    if (!std::strcmp(name, "lit_blocks_per_cu")) { *lo = 0; *hi = 16; return &g_set.lit_blocks_per_cu; }
    if (!std::strcmp(name, "layout")) { *lo = 0; *hi = 2; return &g_set.layout; }
    if (!std::strcmp(name, "pause")) { *lo = -1; *hi = 64; return &g_set.pause; }
    if (!std::strcmp(name, "finish")) { *lo = -1; *hi = 8; return &g_set.finish; }
    return nullptr;
}

// ---- launch plans: pure host arithmetic, shared by the entry points and by redux_plan_* ---------------------
struct FlatPlan { int unroll; unsigned grid; int finish; unsigned chain; unsigned pause; };

// Launch shape of the flat sum.  Measured on MI355X: read bandwidth peaks with about 8 MiB in flight
// (one 256-thread block per compute unit, eight 16-byte loads per lane) and drops by several percent
// when more blocks are resident.  Small inputs keep the deep unroll as long as that leaves 64 blocks.
// Loop iterations between folds of the MMA accumulators into the wide per-wavefront total: the "max_chain" setting, lowered
// for int8 where an int32 accumulator could otherwise pass 2^31.  One int8 MFMA adds at most 64 x 128 = 2^13 in magnitude to an
// accumulator entry and an iteration issues `unroll` of them over `chains` accumulators; the classic family adds at most
// 4 x 128 = 2^9 per running sum per 16-byte vector.
unsigned chain_length(const Settings &S, int dtype, bool mfma, int unroll, int chains)
{
    u64 chain = (u64)S.max_chain;
    if (dtype == REDUX_I8) {
        const u64 per_iter = mfma ? (u64)8192 * (u64)((unroll + chains - 1) / chains) : (u64)512 * (u64)unroll;
        const u64 cap = (((u64)1 << 31) - 1) / per_iter;
        if (chain > cap) chain = cap;
    }
    return (unsigned)chain;
}

FlatPlan plan_flat(const Settings &S, u64 nvec, int cus, int dtype)
{
    FlatPlan p;
    u64 gmax = (u64)cus * (u64)S.blocks_per_cu;
    if (gmax > (u64)S.max_grid) gmax = (u64)S.max_grid;
    if (gmax < 1) gmax = 1;
    p.unroll = (int)S.unroll;
    if (p.unroll == 0) {
        const u64 want = gmax < 64 ? gmax : 64;
        p.unroll = 8;
        while (p.unroll > 1 && nvec / ((u64)kBlock * p.unroll) < want) p.unroll >>= 1;
    }
    const u64 nslab = nvec / ((u64)kBlock * p.unroll);
    p.grid = (unsigned)(nslab < 1 ? 1 : (nslab < gmax ? nslab : gmax));
    // How the block totals meet (all in the same kernel; us per whole call, back to back, binary16 / int8):
    //   floating point: every block sends its partial to a slot and draws a ticket, the last one adds the slots (finish 6);
    //   int8: one atomic addition per block adds its total to a word and counts it (finish 5).
    //   Read-modify-writes of one line of memory are served one after the other, about 8 ns each.  From 4 to 128 MiB all blocks arrive
    //   within a microsecond and the last waits for a queue of 256, so there the blocks of a die meet at the die's own word
    //   first and the eight dies at the common one (finish 7 / 8): 8 MiB 5.2 / 4.5 against 7.1 / 6.6 in one level (and
    //   6.4 - 7.0 with a second one-block kernel, finish 2), 32 MiB 8.5 / 7.6 against 10.2 / 9.5 (8.8), 128 MiB 22.4 / 21.5
    //   against 23.6 / 22.8 (22.4).  Up to 2 MiB (64 blocks) and from 256 MiB on (arrivals spread out) one level is level
    //   or ahead by the second level's round trip: 2 GiB 289.0 / 288.9 against 289.4 / 289.1 (second kernel 289.1 / 290.4).
    // What an input cannot take falls back to the plain ticket finish (4): int8 beyond 2^40 elements (the counted
    // word's sum has 49 bits), floating point on more blocks than there are slots.
    const bool together = nvec > ((u64)2 << 20) / 16 && nvec < ((u64)256 << 20) / 16;
    const bool is_int = dtype == REDUX_I8;
    int finish = (int)S.finish;
    if (finish < 0) finish = is_int ? (together ? 8 : 5) : (together ? 7 : 6);
    if ((finish == 5 || finish == 8) && !(is_int && nvec <= ((u64)1 << 36))) finish = 4;
    if ((finish == 6 || finish == 7) && (is_int || p.grid > kWorkspaceSlots)) finish = 4;
    p.finish = finish;
    const bool mfma = effective_variant(S, dtype, true) == REDUX_VARIANT_MFMA;
    p.chain = chain_length(S, dtype, mfma, p.unroll, 4);
    // Measured on 0.5 - 4 GiB of binary16, bfloat16 and int8: a wavefront of the MMA family that sleeps about 500 cycles
    // between its last MMA and its next eight loads finishes the call 0.5 - 1.5 % earlier (2 GiB: 290.4 against 293.1 us),
    // level with the classic family, whose conversions and additions take about as long.  Eight loads per lane on every
    // compute unit are slightly more than the memory system needs in flight; the sleep shortens its queues.  Runs of
    // 256 MiB and less gain nothing or lose, and binary32 (four MMAs per load) and the 8-bit floats (two) lose.
    const bool one_mma_per_load = dtype == REDUX_F16 || dtype == REDUX_BF16 || dtype == REDUX_I8;
    p.pause = S.pause >= 0 ? (unsigned)S.pause : (mfma && one_mma_per_load && nslab / p.grid >= 64 ? 8u : 0u);
    return p;
}

struct SegPlan {
    int kernel;          // REDUX_KERNEL_SHORT, _ROWS, _RAGGED, _TILES, _BLOCK, _WAVE or _PIECES
    int unroll;          // rows: loads per row group per iteration; otherwise 16-byte loads in flight per lane
    unsigned grid;
    u64 parts, part_len; // pieces per segment and elements per piece (parts == 1: the whole segment)
    unsigned nvec;       // short, rows: 16-byte vectors per segment; ragged: lanes per segment
    unsigned chain;      // loop iterations between folds (the kernels that loop over a segment)
};

SegPlan plan_segmented_shape(const Settings &S, u64 nseg, u64 seglen, int dtype, size_t es, uintptr_t x_addr, int cus)
{
    SegPlan p;
    p.parts = 1;
    p.part_len = seglen;
    p.nvec = 0;
    const u64 seg_bytes = seglen * es;
    // aligned power-of-two segments of 16 B .. 1 KiB (4 KiB): read as one contiguous stream, 0/1 selection matrices in the MMAs
    // (measured: with the MMA family also 2 KiB, +7 %, and 4 KiB, +3 %, against one wavefront per segment; 8 KiB is slower)
    const u64 short_limit = effective_variant(S, dtype) == REDUX_VARIANT_MFMA && dtype != REDUX_F32 ? 4096 : 1024;
    if (S.seg_short && x_addr % 16 == 0 && seg_bytes >= 16 && seg_bytes <= short_limit && (seg_bytes & (seg_bytes - 1)) == 0) {
        p.kernel = REDUX_KERNEL_SHORT;
        p.nvec = (unsigned)(seg_bytes / 16);
        p.unroll = kShortLoads;
        const u64 nslab = (nseg * p.nvec + kShortSlab - 1) / kShortSlab;
        // measured: one block per compute unit for the MMA family, two for the classic one (its conversions are longer)
        const long best_bpc = effective_variant(S, dtype) == REDUX_VARIANT_MFMA ? 1 : 2;
        u64 gmax = (u64)cus * (u64)(S.seg_blocks_per_cu ? S.seg_blocks_per_cu : best_bpc);
        if (gmax > (u64)S.max_grid) gmax = (u64)S.max_grid;
        if (gmax < 1) gmax = 1;
        p.grid = (unsigned)(nslab < gmax ? nslab : gmax);
        return p;
    }
    // short segments: sixteen per wavefront, one per row of the A operand
    // (only when the ragged form below is switched off: measured, that form is as fast or faster at every size)
    const auto ragged_lanes = [](u64 cover) { u64 l = 1; while (l < cover) l *= 2; return l; };
    // (measured: the MMA family's rolling form is level with or ahead of one wavefront per segment up to where one block
    // per segment takes over, and far more even -- 6.7-7.0 against 6.5-7.1 TB/s on 512 MiB, 6.0-6.6 against 5.5-6.6 on
    // 128 MiB; the run-by-run forms are ahead only below 8000 bytes)
    const u64 runs_max = S.seg_runs_max ? (u64)S.seg_runs_max
                       : (effective_variant(S, dtype) == REDUX_VARIANT_MFMA && S.seg_runs_stream) ? 28671 : 7999;
    const bool runs_fit = S.seg_runs && seg_bytes > 1008 && seg_bytes <= runs_max;
    // Segments a little longer than the 32 KiB that a block reads at a time leave most of its second pass idle
    // (measured, 33000 and 36000 bytes: 6.4 and 6.5 TB/s by one block per segment, 6.7 as runs; from 40000 bytes on the
    // block is ahead, 6.8 against 6.5), so while there are enough of them to give every wavefront its own they go as runs too.
    const bool runs_long = S.seg_runs && seg_bytes > 32768 && seg_bytes <= (u64)S.seg_runs_long && nseg >= (u64)cus * 8;
    const bool ragged_fit = S.seg_ragged && seg_bytes <= 1008 && nseg <= ((u64)1 << 56);
    if (!ragged_fit && (dtype == REDUX_F16 || dtype == REDUX_I8) && S.rows_max_vec > 0 && seg_bytes % 16 == 0 &&
        x_addr % 16 == 0 && seg_bytes / 16 <= (u64)S.rows_max_vec) {
        p.kernel = REDUX_KERNEL_ROWS;
        p.nvec = (unsigned)(seg_bytes / 16);
        const unsigned steps = (p.nvec + 3) / 4;
        p.unroll = steps <= 1 ? 1 : steps <= 2 ? 2 : steps <= 4 ? 4 : 8;
        const u64 groups_per_iter = 8 / p.unroll;
        const u64 nsuper = ((nseg + 15) / 16 + groups_per_iter - 1) / groups_per_iter;
        u64 blocks = (nsuper + kWaves - 1) / kWaves;
        u64 gmax = (u64)cus * (u64)(S.seg_blocks_per_cu ? S.seg_blocks_per_cu : 2);   // measured best
        if (gmax > (u64)S.max_grid) gmax = (u64)S.max_grid;
        if (gmax < 1) gmax = 1;
        p.grid = (unsigned)(blocks < gmax ? blocks : gmax);
        return p;
    }
    // any other segment of up to 1008 bytes: the same contiguous stream, each group of 2^lg lanes reading the aligned
    // vectors that overlap its segment and clearing the bytes outside it
    if (ragged_fit) {
        // most vectors a segment can touch: its first byte sits at most 16 - es bytes into a vector (at exactly
        // x mod 16 if segments are whole vectors long; segments that divide a vector and start on their own size
        // never straddle one)
        const u64 max_off = seg_bytes % 16 == 0 ? (u64)(x_addr % 16)
                          : (16 % seg_bytes == 0 && x_addr % seg_bytes == 0) ? 16 - seg_bytes : (u64)(16 - es);
        const u64 cover = (max_off + seg_bytes + 15) / 16;
        p.kernel = REDUX_KERNEL_RAGGED;
        p.nvec = (unsigned)ragged_lanes(cover);
        p.unroll = kShortLoads;
        const u64 nslab = (nseg * p.nvec + kShortSlab - 1) / kShortSlab;
        // measured (offsets and masks are worked out once per lane, so a load costs what it costs in the aligned form):
        // one block per compute unit when most lanes of a group hold data (400 B: 7.0 TB/s, 750 B - 1 KB: 7.1), two when
        // about half of them idle (520 B, 33 of 64 lanes: 6.8 against 5.7) or the groups are small; the classic family,
        // whose lanes also convert and add, one block more
        const bool full = cover * 10 >= (u64)p.nvec * 7 && p.nvec >= 32;
        const long best_bpc = effective_variant(S, dtype) == REDUX_VARIANT_MFMA ? (full ? 1 : 2)
                                                                                : (cover * 10 >= (u64)p.nvec * 7 ? 2 : 3);
        u64 gmax = (u64)cus * (u64)(S.seg_blocks_per_cu ? S.seg_blocks_per_cu : best_bpc);
        if (gmax > (u64)S.max_grid) gmax = (u64)S.max_grid;
        if (gmax < 1) gmax = 1;
        p.grid = (unsigned)(nslab < gmax ? nslab : gmax);
        return p;
    }
    // segments of exactly 1, 2, 4 or 8 whole tiles, enough of them to fill the chip: the pipelined kernel
    if (S.seg_tiles && x_addr % 16 == 0 && seg_bytes % 1024 == 0 && seg_bytes <= 8192 &&
        ((seg_bytes / 1024) & (seg_bytes / 1024 - 1)) == 0 && nseg >= (u64)cus * kWaves) {
        p.kernel = REDUX_KERNEL_TILES;
        p.unroll = (int)(seg_bytes / 1024);
        u64 blocks = (nseg + kWaves - 1) / kWaves;
        const long best_bpc = p.unroll == 8 ? 1 : p.unroll == 4 ? 2 : p.unroll == 2 ? 3 : 8;   // measured on MI355X
        u64 gmax = (u64)cus * (u64)(S.seg_blocks_per_cu ? S.seg_blocks_per_cu : best_bpc);
        if (gmax > (u64)S.max_grid) gmax = (u64)S.max_grid;
        if (gmax < 1) gmax = 1;
        p.grid = (unsigned)(blocks < gmax ? blocks : gmax);
        return p;
    }
    // long segments (32 KiB and up): one block per segment, cut into pieces of at least 32 KiB while there are
    // fewer than two pieces per compute unit, as far as the workspace allows
    if (S.seg_block_bytes > 0 && seg_bytes >= (u64)S.seg_block_bytes && !runs_long) {
        const u64 want_blocks = (u64)cus * 2;
        u64 parts = 1;
        if (S.seg_parts > 0) parts = (u64)S.seg_parts;
        else {
            while (nseg * parts < want_blocks && nseg * parts * 2 <= (u64)kMaxGrid && seg_bytes / (parts * 2) >= 32768) parts *= 2;
            // (that is the number "seg_balance" = 0 keeps.)  Blocks take pieces in rounds, and a last round that is only partly
            // filled leaves the rest of the chip idle (measured: 1073 segments of 500000 bytes on 512 blocks, 2.1 rounds,
            // 6.1 TB/s against 6.9 for a whole number of rounds).  `used`: the share of the rounds' slots that hold a piece.
            const auto used = [&](u64 pr) {
                const u64 pieces = nseg * pr;
                const u64 piece_bytes = (seg_bytes + pr - 1) / pr;
                u64 g = (u64)cus * (u64)(S.seg_blocks_per_cu ? S.seg_blocks_per_cu : (piece_bytes >= ((u64)512 << 10) ? 1 : 2));
                if (g > (u64)S.max_grid) g = (u64)S.max_grid;
                if (g < 1) g = 1;
                if (g > pieces) g = pieces;
                return (double)pieces / (double)(g * ((pieces + g - 1) / g));
            };
            // All numbers of pieces that are allowed are looked at (halving while a piece stays above 64 KiB), and the one with
            // the lowest modelled time wins, fewer pieces within 1 %.  The model: whole rounds of pieces over the grid take
            // their full time, a last round that fills a fraction f of the grid the square root of f (fewer blocks leave each
            // more bandwidth) but at least half a round (what a block on its own can draw); pieces cost what adds them up,
            // 3 us for a second kernel and half a microsecond in the same one (where every piece has a block), against the
            // call's time at 6.5 TB/s.  Against the best of 1 .. 128 pieces measured on 60 shapes of 100 - 3000 segments
            // in 128 MiB - 1 GiB the choice is within 1 % on average and 7 % at worst (1 GiB: 700
            // segments whole 6.4 TB/s in 2.7 rounds, in 8 pieces each 6.9; 200 segments of 5 MB in 8 pieces 6.3, in 64 6.9;
            // 128 MiB: 200 segments whole 6.1, in 8 pieces 5.5).  ("seg_balance" 2 .. 99: the first number of pieces that uses
            // that percentage of its rounds' slots, as it used to be.)
            if (S.seg_balance == 1) {
                const double call_us = (double)nseg * (double)seg_bytes / 6.5e6;
                const auto score = [&](u64 pr) {
                    const u64 pieces = nseg * pr;
                    const u64 piece_bytes = (seg_bytes + pr - 1) / pr;
                    u64 g = (u64)cus * (u64)(S.seg_blocks_per_cu ? S.seg_blocks_per_cu : (piece_bytes >= ((u64)512 << 10) ? 1 : 2));
                    if (g > (u64)S.max_grid) g = (u64)S.max_grid;
                    if (g < 1) g = 1;
                    const double rounds = (double)pieces / (double)g;
                    const double whole = std::floor(rounds), f = rounds - whole;
                    const double last = f > 0.0 ? (f > 0.25 ? std::sqrt(f) : 0.5) : 0.0;
                    const double use = rounds / (whole + last);
                    const double extra = pr == 1 ? 0.0 : (pieces <= g && S.seg_finish != 0 ? 0.5 : 3.0);
                    return use * call_us / (call_us + extra);
                };
                // (pieces of 32 KiB are allowed as far as the first rule above goes, of 64 KiB beyond)
                u64 best = 1;
                for (u64 pr = 2; nseg * pr <= (u64)kMaxGrid && (pr <= parts || seg_bytes / pr >= 65536); pr *= 2)
                    if (score(pr) > score(best) * 1.01) best = pr;
                // ... and the numbers that make exactly one round of it (a handful of segments need not be a power of two)
                for (u64 per_cu = 1; per_cu <= 2; ++per_cu) {
                    u64 pr = (u64)cus * per_cu / nseg;
                    // (measured: 234, 238, 242, 246 or 250 blocks -- twice an odd number -- run 5 % behind 240, 243, 245, 247, 252, 253 or 255)
                    while (pr >= 2 && (nseg * pr) % 4 == 2) --pr;
                    if (pr >= 2 && nseg * pr <= (u64)kMaxGrid && seg_bytes / pr >= 65536 && score(pr) > score(best) * 1.01) best = pr;
                }
                parts = best;
            } else if (S.seg_balance > 1) {
                const double enough = (double)S.seg_balance / 100.0;
                while (used(parts) < enough && nseg * parts * 2 <= (u64)kMaxGrid && seg_bytes / (parts * 2) >= 65536) parts *= 2;
            }
        }
        if (parts > 1 && nseg <= (u64)kMaxGrid / parts) {
            p.parts = parts;
            p.part_len = ((seglen + parts - 1) / parts + 511) / 512 * 512;
        }
        p.kernel = REDUX_KERNEL_BLOCK;
        p.unroll = (int)S.unroll;
        if (p.unroll == 0) p.unroll = 8;
        // measured: two blocks per compute unit hide the per-piece fold for pieces below 512 KiB
        const long bpc = S.seg_blocks_per_cu ? S.seg_blocks_per_cu : (p.part_len * es >= ((u64)512 << 10) ? 1 : 2);
        const u64 blocks_needed = nseg * p.parts;
        u64 gmax = (u64)cus * (u64)bpc;
        if (gmax > (u64)S.max_grid) gmax = (u64)S.max_grid;
        if (gmax < 1) gmax = 1;
        p.grid = (unsigned)(blocks_needed < gmax ? blocks_needed : gmax);
        return p;
    }
    // A few long segments would leave most of the chip idle with one wavefront each: cut each into a power-of-two number
    // of pieces (whole 512-element tiles, at least 8 tiles each) until there are about 8 wavefronts per
    // compute unit, as far as the workspace allows.  Only where one block per segment is switched off, that is from
    // 32 KiB on: below, a call with so few segments is all launch, and the second launch that adds the piece totals costs more
    // than the pieces gain (measured, 4 - 1024 segments of 16 - 28 KB: 9.3 - 9.5 us cut in two or four, 6.4 - 7.9 us whole).
    const u64 want_waves = (u64)cus * 8;
    u64 parts = 1;
    if (S.seg_parts > 0) parts = (u64)S.seg_parts;
    else if (seg_bytes >= 32768)
        while (nseg * parts < want_waves && nseg * parts * 2 <= (u64)kMaxGrid && seglen / (parts * 2) >= 8 * 512) parts *= 2;
    p.kernel = REDUX_KERNEL_WAVE;
    if (parts > 1 && nseg <= (u64)kMaxGrid / parts) {
        p.kernel = REDUX_KERNEL_PIECES;
        p.parts = parts;
        p.part_len = ((seglen + parts - 1) / parts + 511) / 512 * 512;
    }
    // Whole segments of more than 1008 bytes up to 28 KiB (the run-by-run forms: less than 8000 bytes, from where on one
    // wavefront per segment is level or ahead of them), and those just above 32 KiB: a wavefront streams a run of up to
    // sixteen of them as one contiguous piece.
    if (p.kernel == REDUX_KERNEL_WAVE && (runs_fit || runs_long)) {
        p.kernel = REDUX_KERNEL_RUNS;
        const bool mfma = effective_variant(S, dtype) == REDUX_VARIANT_MFMA;
        // measured: the rolling form, which keeps its loads in flight across the end of a run, runs best with four loads
        // per lane and two blocks per compute unit (three for short segments, where the boundaries take more
        // instructions: below 1.5 KB in the MMA family, below 3 KB in the classic one); the run-by-run form of the MMA
        // family with four loads and three blocks (the fold and the store at the end of a run leave gaps that other
        // wavefronts fill), that of the classic family, whose lanes also convert and add, with eight loads and more
        // wavefronts the shorter the segments are
        const bool rolling = S.seg_runs_stream != 0;
        p.unroll = S.unroll == 0 ? (mfma || rolling ? 4 : 8) : (S.unroll <= 4 ? 4 : 8);
        const u64 step = 64 * (u64)p.unroll;                                    // vectors per iteration of a wavefront
        const long bpc = S.seg_blocks_per_cu ? S.seg_blocks_per_cu
                       : rolling ? (seg_bytes >= (mfma ? 1536u : 3000u) ? 2 : 3)
                       : mfma ? 3 : seg_bytes < 2560 ? 8 : 4;
        u64 gmax = (u64)cus * (u64)bpc;
        if (gmax > (u64)S.max_grid) gmax = (u64)S.max_grid;
        if (gmax < 1) gmax = 1;
        // Segments per run.  A run costs its iterations (whole ones: the lanes of the last one that lie behind the run's
        // end idle) plus a fixed amount for the fold, the store and the set-up of the next run, taken as one iteration
        // of four loads.  Every wavefront takes the same number of whole runs and then one shorter run, its share of
        // what is left (run_share), so the cost of a wavefront is known exactly and the length with the lowest one wins
        // (measured before the last run was shared out: 8200-byte segments in runs of 7 on 768 blocks, 2.08 rounds of
        // whole runs, 5.97 TB/s; in runs of 11, 1.3 rounds, 6.69).
        const auto run_cost = [&](u64 c) {
            const u64 slots = (15 + c * seg_bytes + 15) / 16;                  // worst alignment of the run's first byte
            return (double)(((slots + step - 1) / step) * step * 16 + 4096);
        };
        u64 len = 1;
        if (S.seg_run_len > 0) {
            len = (u64)S.seg_run_len;
        } else {
            double best = 0.0;
            for (u64 c = 1; c <= 16 && c <= nseg; ++c) {
                const u64 blocks = ((nseg + c - 1) / c + kWaves - 1) / kWaves;
                const u64 waves = (blocks < gmax ? blocks : gmax) * kWaves;
                const u64 full = nseg / (waves * c);
                const u64 tail = (nseg - full * waves * c + waves - 1) / waves;
                // Runs whose length is close to a multiple of 4 KiB, and more so of 32 KiB, make neighbouring wavefronts
                // walk the same memory channels in step (measured: 2052-byte segments in runs of 8, 16416 bytes, 6.29 TB/s,
                // in runs of 7 or 9 6.66 and 6.69; 3500-byte segments in runs of 14, 49000 bytes, 6.44, in runs of 13 or
                // 15 6.72 and 6.79; on 128 MiB, 4000-byte segments in runs of 16, 64000 bytes, 6.1, in runs of 15 6.8).
                const u64 over = (c * seg_bytes) % 4096, over32 = (c * seg_bytes) % 32768;
                const double in_step = (over32 <= 2560 || over32 >= 32768 - 2560) ? 1.10
                                     : (over <= 768 || over >= 4096 - 768) ? 1.05 : 1.0;
                const double cost = ((double)full * run_cost(c) + (tail ? run_cost(tail) : 0.0)) * in_step;
                if (c == 1 || cost <= best) { best = cost; len = c; }
            }
        }
        p.nvec = (unsigned)len;
        const u64 nruns = (nseg + len - 1) / len;
        const u64 blocks = (nruns + kWaves - 1) / kWaves;
        p.grid = (unsigned)(blocks < gmax ? blocks : gmax);
        return p;
    }
    // Measured on MI355X by piece size (aligned vectors a piece can overlap): up to 2 KiB two loads per lane take the
    // whole piece at once; up to 5 KiB one load per lane and as many wavefronts as fit hide the per-segment fold
    // best; longer pieces stream with two, then four loads in flight per lane.
    const u64 piece_bytes = p.part_len * es;
    const u64 cover = (piece_bytes + ((x_addr % 16 == 0 && seg_bytes % 16 == 0) ? 0 : 16 - es) + 15) / 16;
    p.unroll = (int)S.unroll;
    long best_bpc = 0;
    if (p.unroll == 0) {
        if (cover <= 64)       { p.unroll = 1; best_bpc = 16; }
        else if (cover <= 128) { p.unroll = 2; best_bpc = 8; }
        else if (cover <= 320) { p.unroll = 1; best_bpc = 16; }
        else if (cover <= 640) { p.unroll = 2; best_bpc = 4; }
        else                   { p.unroll = 4; best_bpc = 2; }
    } else {
        best_bpc = 8 / p.unroll;
    }
    const long bpc = S.seg_blocks_per_cu ? S.seg_blocks_per_cu : best_bpc;
    u64 blocks_needed = (nseg * p.parts + kWaves - 1) / kWaves;
    u64 gmax = (u64)cus * (u64)bpc;
    if (gmax > (u64)S.max_grid) gmax = (u64)S.max_grid;
    if (gmax < 1) gmax = 1;
    p.grid = (unsigned)(blocks_needed < gmax ? blocks_needed : gmax);
    return p;
}

SegPlan plan_segmented(const Settings &S, u64 nseg, u64 seglen, int dtype, size_t es, uintptr_t x_addr, int cus)
{
    SegPlan p = plan_segmented_shape(S, nseg, seglen, dtype, es, x_addr, cus);
    // one block per segment: the flat sum's four accumulator chains; one wavefront per segment: a single chain
    p.chain = chain_length(S, dtype, effective_variant(S, dtype) == REDUX_VARIANT_MFMA, p.unroll, p.kernel == REDUX_KERNEL_BLOCK ? 4 : 1);
    return p;
}

// Segments cut into pieces: does the same kernel add a segment's piece totals (the last block of the segment to arrive),
// or a second kernel?  Only the one-block-per-piece kernel can; its slots and tickets cover every shape it is given
// (pieces <= kMaxGrid, at least two per segment).  Measured, us per call back to back, second kernel / same kernel:
//   2 x 0.5 ... 8 MiB (16 - 256 pieces each)       9.2 / 6.3 (a launch less, and the call is all launch)
//   2 x 16 ... 64 MiB (256 pieces each)            9.2 / 8.9, 13.4 / 13.2, 23.2 / 23.0 with the arrivals counted in two
//       levels (one level: 8.4 / 10.1 ... 23.4 / 25.4, the 256 arrivals queue up at the segment's ticket)
//   16 x 0.5 ... 8 MiB                              9.2 / 6.3 - 7.1, 9.2 / 8.8, 13.4 / 13.2, 23.2 / 22.9
//   128 x 64 KiB ... 1 MiB (2 - 4 pieces each)      9.3 / 6.4 - 6.7, 9.4 / 8.9, 13.5 / 13.0, 23.3 / 22.6
//   int8: the same or better (one read-modify-write per piece, no piece totals to fetch): 9.7 / 8.0, 14.2 / 12.5, 24.0 / 22.5
//   more pieces than blocks (a block goes on to another piece, and would wait for its ticket first): 79.6 / 91.8,
//       256 MiB in 2 x 256 pieces on 256 blocks 41.5 / 42.5
// Arrivals counted in two levels: nine words per segment on a 256-byte line each fit the 64 KiB of per-segment words for
// up to 28 segments; worth it from 32 pieces per segment.
bool seg_two_levels(const SegPlan &p, u64 nseg)
{
    return p.kernel == REDUX_KERNEL_BLOCK && p.parts >= 32 && nseg * 9 <= (u64)(kMaxGrid / 2) * sizeof(u64) / 256;
}

bool seg_finish_in_kernel(const Settings &S, const SegPlan &p, u64 nseg)
{
    if (p.kernel != REDUX_KERNEL_BLOCK || p.parts <= 1 || S.seg_finish == 0) return false;
    if (S.seg_finish > 0) return true;
    return nseg * p.parts <= (u64)p.grid;
}

} // namespace

// =====================================================================================================
extern "C" {

// The flat sum: `ws` is where the block partials and the ticket live.
static int launch_sum(const Settings &S, int cus, const Workspace &ws, bool clear_ticket, const void *x, size_t n, size_t es,
                      int dtype, void *out, hipStream_t st)
{
    FlatArgs a;
    a.run = es == 4 ? make_run<4>(x, n) : es == 2 ? make_run<2>(x, n) : make_run<1>(x, n);
    a.partials = ws.partials;
    a.ticket = ws.ticket;
    a.slots = ws.slots;
    a.leaves = (unsigned *)ws.counted;
    a.out = out;
    a.layout = (int)S.layout;
    a.stagger = (unsigned)S.stagger;

    const FlatPlan plan = plan_flat(S, a.run.nvec, cus, dtype);
    const int unroll = plan.unroll;
    const unsigned grid = plan.grid;
    a.finish = plan.finish;
    a.max_chain = plan.chain;
    a.pause = plan.pause;

    const bool nt = S.nontemporal != 0;
    const bool mfma = effective_variant(S, dtype, true) == REDUX_VARIANT_MFMA;
    hipError_t e;
    if (a.finish == 3) {   // atomic additions start from zero
        if (dtype != REDUX_I8) hipLaunchKernelGGL(fill_zero_kernel<float>, dim3(1), dim3(64), 0, st, (float *)out, (u64)1);
        else                   hipLaunchKernelGGL(fill_zero_kernel<i64>, dim3(1), dim3(64), 0, st, (i64 *)out, (u64)1);
        e = hipGetLastError();
        if (e != hipSuccess) return hip_fail(e);
    } else if (clear_ticket && a.finish != 2) {
        // the ticket and the counted sum behind it; the slots of the blocks to come
        hipLaunchKernelGGL(empty_slots_kernel, dim3(1), dim3(256), 0, st, a.slots, a.finish == 6 || a.finish == 7 ? grid : 0u, a.ticket, 4u, a.leaves);
        e = hipGetLastError();
        if (e != hipSuccess) return hip_fail(e);
    }
    if (S.compensated && dtype == REDUX_F16 && mfma) launch_flat<F16MfmaCompensated>(unroll, nt, grid, st, a);
    else with_flat_family(dtype, mfma, [&](auto family) { launch_flat<decltype(family)>(unroll, nt, grid, st, a); });
    e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e);
    if (a.finish == 2) {
        if (dtype == REDUX_I8) hipLaunchKernelGGL(finish_kernel<I8Classic>, dim3(1), dim3(kBlock), 0, st, a.partials, grid, out);
        else if (mfma)         hipLaunchKernelGGL(finish_kernel<F16Mfma>, dim3(1), dim3(kBlock), 0, st, a.partials, grid, out);
        else                   hipLaunchKernelGGL(finish_kernel<F16Classic>, dim3(1), dim3(kBlock), 0, st, a.partials, grid, out);
        e = hipGetLastError();
        if (e != hipSuccess) return hip_fail(e);
    }
    return REDUX_OK;
}

static int launch_empty_sum(int dtype, void *out, hipStream_t st)
{
    if (dtype != REDUX_I8) hipLaunchKernelGGL(fill_zero_kernel<float>, dim3(1), dim3(64), 0, st, (float *)out, (u64)1);
    else                   hipLaunchKernelGGL(fill_zero_kernel<i64>, dim3(1), dim3(64), 0, st, (i64 *)out, (u64)1);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? REDUX_OK : hip_fail(e);
}

int redux_sum(const void *x, size_t n, int dtype, void *out, void *stream)
{
    std::call_once(g_env_once, read_env);
    size_t es = 0;
    int rc = check_common(x, n, dtype, out, 1, &es);
    if (rc != REDUX_OK) return rc;
    hipStream_t st = (hipStream_t)stream;
    if (n == 0) return launch_empty_sum(dtype, out, st);   // the empty sum

    // process-wide state is read under the lock; the launches run outside it, so host threads do not serialise
    Settings S;
    int cus = 0;
    Workspace ws;
    {
        std::lock_guard<std::mutex> lock(g_mu);
        S = g_set;
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return hip_fail(e);
        if ((rc = device_cus(dev, &cus)) != REDUX_OK) return rc;
        if ((rc = get_workspace(dev, st, &ws)) != REDUX_OK) return rc;
    }
    return launch_sum(S, cus, ws, false, x, n, es, dtype, out, st);
}

int redux_sum_static(const void *x, size_t n, int dtype, void *out, void *stream)
{
    std::call_once(g_env_once, read_env);
    size_t es = 0;
    int rc = check_common(x, n, dtype, out, 1, &es);
    if (rc != REDUX_OK) return rc;
    hipStream_t st = (hipStream_t)stream;
    if (n == 0) return launch_empty_sum(dtype, out, st);

    Settings S;
    int cus = 0;
    Workspace ws;
    {
        std::lock_guard<std::mutex> lock(g_mu);
        S = g_set;
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return hip_fail(e);
        if (dev < 0 || dev >= kStaticDevices) return REDUX_ERR_SCRATCH;
        if (g_static_cus[dev] == 0) {
            int c = 0;
            e = hipDeviceGetAttribute(&c, hipDeviceAttributeMultiprocessorCount, dev);
            if (e != hipSuccess) return hip_fail(e);
            g_static_cus[dev] = c > 0 ? c : 1;
        }
        cus = g_static_cus[dev];
        if (!g_scratch_ptr[dev]) {          // first call on this device, which is the current one
            void *ptr = nullptr;
            e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
            if (e != hipSuccess) return hip_fail(e);
            if (!ptr) return hip_fail(hipErrorInvalidSymbol);
            g_scratch_ptr[dev] = ptr;
        }
        ws.partials = (u64 *)g_scratch_ptr[dev];
        ws.ticket = (unsigned *)((char *)g_scratch_ptr[dev] + kScratchTicketOffset);
        ws.slots = ws.partials;             // marked empty by every call that uses them
        ws.counted = (u64 *)((char *)g_scratch_ptr[dev] + kScratchLeavesOffset);   // (only its use as second-level tickets)
    }
    // The launch writes one partial per block.  More blocks than the array has slots can only be asked for through
    // "blocks_per_cu" / "max_grid" on a device with many compute units; such a call is refused, never truncated.
    const Run run = es == 4 ? make_run<4>(x, n) : es == 2 ? make_run<2>(x, n) : make_run<1>(x, n);
    if (plan_flat(S, run.nvec, cus, dtype).grid > (unsigned)kScratchSlots) return REDUX_ERR_SCRATCH;
    // the array keeps what the last call left in it: a fill kernel ahead of the sum clears the ticket and, for the finish
    // that reads partials as they arrive, marks this call's slots empty (the other finishes only read what this call's
    // blocks have written)
    return launch_sum(S, cus, ws, true, x, n, es, dtype, out, st);
}

int redux_sum_segmented(const void *x, size_t nseg, size_t seglen, int dtype, void *out, void *stream)
{
    std::call_once(g_env_once, read_env);
    if (elem_size_of(dtype) == 0) return REDUX_ERR_DTYPE;
    if (seglen && nseg > ((size_t)1 << 62) / seglen) return REDUX_ERR_SIZE;
    if (nseg > ((size_t)1 << 59)) return REDUX_ERR_SIZE;
    size_t es = 0;
    int rc = check_common(x, nseg * seglen, dtype, out, nseg, &es);
    if (rc != REDUX_OK) return rc;
    if (nseg == 0) return REDUX_OK;

    hipStream_t st = (hipStream_t)stream;

    if (seglen == 0) {
        unsigned grid = (unsigned)((nseg + 255) / 256);
        if (dtype != REDUX_I8) hipLaunchKernelGGL(fill_zero_kernel<float>, dim3(grid), dim3(256), 0, st, (float *)out, (u64)nseg);
        else                   hipLaunchKernelGGL(fill_zero_kernel<i64>, dim3(grid), dim3(256), 0, st, (i64 *)out, (u64)nseg);
        hipError_t e = hipGetLastError();
        return e == hipSuccess ? REDUX_OK : hip_fail(e);
    }

    // process-wide state is read under the lock; the launches run outside it
    Settings S;
    int dev = 0, cus = 0;
    hipError_t e;
    {
        std::lock_guard<std::mutex> lock(g_mu);
        S = g_set;
        e = hipGetDevice(&dev);
        if (e != hipSuccess) return hip_fail(e);
        if ((rc = device_cus(dev, &cus)) != REDUX_OK) return rc;
    }

    const bool nt = S.nontemporal != 0;
    const bool mfma = effective_variant(S, dtype) == REDUX_VARIANT_MFMA;
    const SegPlan plan = plan_segmented(S, nseg, seglen, dtype, es, (uintptr_t)x, cus);
    const unsigned grid = plan.grid;

    // ---- short segments read as one contiguous stream: aligned powers of two, or ragged ----------------------
    if (plan.kernel == REDUX_KERNEL_SHORT || plan.kernel == REDUX_KERNEL_RAGGED) {
        const bool ragged = plan.kernel == REDUX_KERNEL_RAGGED;
        ShortArgs s;
        s.x = (const unsigned char *)x;
        s.nseg = nseg;
        s.lg = 0;
        while ((1u << s.lg) < plan.nvec) ++s.lg;
        s.nvec = (u64)nseg << s.lg;
        s.seg_bytes = (u64)seglen * es;
        s.out = out;
        s.layout = (int)S.layout;
        // measured: refilling registers one by one hides the second MMA and the stores of segments up to
        // 256 B (and the classic family's conversions); longer segments run fastest as a plain loop
        // (binary32 excepted: it needs four MMAs per load)
        // The ragged form: always refill.
        const int best_pipe = ragged ? 1 : (mfma && s.lg >= 5 && dtype != REDUX_F32 ? 0 : 1);
        s.pipe = S.seg_short_pipe >= 0 ? (int)S.seg_short_pipe : best_pipe;
        const bool wide = s.lg >= 5;       // 32 or 64 lanes per segment: eight loads share an accumulator
        with_short_family(dtype, [&](auto elem) {
            typedef decltype(elem) E;
#define REDUX_SHORT_NT(KERNEL, ...) do { if (nt) hipLaunchKernelGGL((KERNEL<E, __VA_ARGS__ true, RR>), dim3(grid), dim3(kBlock), 0, st, s); \
                                         else    hipLaunchKernelGGL((KERNEL<E, __VA_ARGS__ false, RR>), dim3(grid), dim3(kBlock), 0, st, s); } while (0)
#define REDUX_SHORT_ALL() do { if (!mfma) REDUX_SHORT_NT(sum_short_classic_kernel, ); \
                               else if (wide) REDUX_SHORT_NT(sum_short_mfma_kernel, 8, ); \
                               else REDUX_SHORT_NT(sum_short_mfma_kernel, 4, ); } while (0)
            if (ragged) { constexpr bool RR = true; REDUX_SHORT_ALL(); }
            else        { constexpr bool RR = false; REDUX_SHORT_ALL(); }
#undef REDUX_SHORT_ALL
#undef REDUX_SHORT_NT
        });
        e = hipGetLastError();
        return e == hipSuccess ? REDUX_OK : hip_fail(e);
    }

    // ---- medium segments: one wavefront streams a run of whole segments ----------------------------------------
    if (plan.kernel == REDUX_KERNEL_RUNS) {
        RunArgs r;
        r.x = (const unsigned char *)x;
        r.nseg = nseg;
        r.seg_bytes = (unsigned)(seglen * es);
        r.per_run = plan.nvec;
        r.out = out;
        r.layout = (int)S.layout;
        with_short_family(dtype, [&](auto elem) {
            typedef decltype(elem) E;
#define REDUX_RUNS(KERNEL, UU) do { if (nt) hipLaunchKernelGGL((KERNEL<E, UU, true>), dim3(grid), dim3(kBlock), 0, st, r); \
                                    else    hipLaunchKernelGGL((KERNEL<E, UU, false>), dim3(grid), dim3(kBlock), 0, st, r); } while (0)
            if (mfma && S.seg_runs_stream) { if (plan.unroll == 8) REDUX_RUNS(sum_segment_runs_mfma_stream_kernel, 8); else REDUX_RUNS(sum_segment_runs_mfma_stream_kernel, 4); }
            else if (mfma) { if (plan.unroll == 8) REDUX_RUNS(sum_segment_runs_mfma_kernel, 8); else REDUX_RUNS(sum_segment_runs_mfma_kernel, 4); }
            else if (S.seg_runs_stream) { if (plan.unroll == 8) REDUX_RUNS(sum_segment_runs_classic_stream_kernel, 8); else REDUX_RUNS(sum_segment_runs_classic_stream_kernel, 4); }
            else      { if (plan.unroll == 8) REDUX_RUNS(sum_segment_runs_classic_kernel, 8); else REDUX_RUNS(sum_segment_runs_classic_kernel, 4); }
#undef REDUX_RUNS
        });
        e = hipGetLastError();
        return e == hipSuccess ? REDUX_OK : hip_fail(e);
    }

    // ---- short segments: sixteen per wavefront, one per row of the A operand -------------------------
    if (plan.kernel == REDUX_KERNEL_ROWS) {
        RowArgs r;
        r.x = (const u32x4 *)x;
        r.nseg = nseg;
        r.nvec = plan.nvec;
        r.out = out;
        const int tc = plan.unroll;
#define REDUX_ROWS(R, TC) do { if (nt) hipLaunchKernelGGL((sum_rows_kernel<R, TC, true>), dim3(grid), dim3(kBlock), 0, st, r); \
                               else    hipLaunchKernelGGL((sum_rows_kernel<R, TC, false>), dim3(grid), dim3(kBlock), 0, st, r); } while (0)
#define REDUX_ROWS_TC(R) do { if (tc == 1) REDUX_ROWS(R, 1); else if (tc == 2) REDUX_ROWS(R, 2); \
                              else if (tc == 4) REDUX_ROWS(R, 4); else REDUX_ROWS(R, 8); } while (0)
        if (dtype == REDUX_F16) { if (mfma) REDUX_ROWS_TC(F16MfmaRows); else REDUX_ROWS_TC(F16ClassicRows); }
        else                    { if (mfma) REDUX_ROWS_TC(I8MfmaRows);  else REDUX_ROWS_TC(I8ClassicRows); }
#undef REDUX_ROWS_TC
#undef REDUX_ROWS
        e = hipGetLastError();
        return e == hipSuccess ? REDUX_OK : hip_fail(e);
    }

    // ---- general form: one wavefront per segment, or per piece of a long segment -------------------------
    SegArgs a;
    a.x = (const unsigned char *)x;
    a.nseg = nseg;
    a.seglen = seglen;
    a.out = out;
    a.max_chain = plan.chain;
    a.parts = plan.parts;
    a.part_len = plan.part_len;
    a.partials = nullptr;
    a.seg_finish = 0;
    a.seg_two_levels = 0;
    a.seg_word_stride = 1;
    a.slots = nullptr;
    a.tickets = nullptr;
    a.counted = nullptr;
    if (plan.parts > 1) {
        Workspace ws;
        std::lock_guard<std::mutex> lock(g_mu);
        if ((rc = get_workspace(dev, st, &ws)) != REDUX_OK) return rc;
        a.partials = ws.partials;
        a.seg_finish = seg_finish_in_kernel(S, plan, nseg) ? 1 : 0;
        a.seg_two_levels = seg_two_levels(plan, nseg) ? 1 : 0;
        a.seg_word_stride = nseg <= (u64)(kMaxGrid / 2) * sizeof(u64) / 256 ? 32u : 1u;      // a line per segment while they fit (256 segments)
        a.slots = ws.slots;
        a.tickets = (unsigned *)ws.counted;
        a.counted = ws.counted;
    }
    const int unroll = plan.unroll;

    if (plan.kernel == REDUX_KERNEL_TILES) {
        with_seg_family(dtype, mfma, [&](auto family) {
            typedef decltype(family) F;
            // measured on 8 KiB segments: issuing the next segment's loads ahead gains 1 % with the MMA family and loses
            // as much with the classic one
#define REDUX_TILES_P(UU, PP) do { if (nt) hipLaunchKernelGGL((sum_segments_tiles_kernel<F, UU, true, PP>), dim3(grid), dim3(kBlock), 0, st, a); \
                                   else    hipLaunchKernelGGL((sum_segments_tiles_kernel<F, UU, false, PP>), dim3(grid), dim3(kBlock), 0, st, a); } while (0)
#define REDUX_TILES(UU) do { if (mfma) REDUX_TILES_P(UU, 1); else REDUX_TILES_P(UU, 0); } while (0)
            if (unroll == 8) REDUX_TILES(8); else if (unroll == 4) REDUX_TILES(4); else if (unroll == 2) REDUX_TILES(2); else REDUX_TILES(1);
#undef REDUX_TILES
#undef REDUX_TILES_P
        });
        e = hipGetLastError();
        return e == hipSuccess ? REDUX_OK : hip_fail(e);
    }

    if (plan.kernel == REDUX_KERNEL_BLOCK) {
        with_flat_family(dtype, mfma, [&](auto family) {      // four accumulator chains, as in the flat sum
            typedef decltype(family) F;
#define REDUX_BLOCK(UU) do { if (nt) hipLaunchKernelGGL((sum_segments_block_kernel<F, UU, true>), dim3(grid), dim3(kBlock), 0, st, a); \
                             else    hipLaunchKernelGGL((sum_segments_block_kernel<F, UU, false>), dim3(grid), dim3(kBlock), 0, st, a); } while (0)
            if (unroll == 8) REDUX_BLOCK(8); else if (unroll == 4) REDUX_BLOCK(4); else if (unroll == 2) REDUX_BLOCK(2); else REDUX_BLOCK(1);
#undef REDUX_BLOCK
        });
    } else {
        with_seg_family(dtype, mfma, [&](auto family) { launch_seg<decltype(family)>(unroll, nt, grid, st, a); });
    }
    e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e);
    if (a.parts > 1 && !a.seg_finish) {
        const unsigned p = (unsigned)a.parts, g = (unsigned)nseg;
        if (dtype == REDUX_I8) hipLaunchKernelGGL(finish_segments_kernel<I8Classic>, dim3(g), dim3(kBlock), 0, st, a.partials, p, out);
        else if (mfma)         hipLaunchKernelGGL(finish_segments_kernel<F16Mfma>, dim3(g), dim3(kBlock), 0, st, a.partials, p, out);
        else                   hipLaunchKernelGGL(finish_segments_kernel<F16Classic>, dim3(g), dim3(kBlock), 0, st, a.partials, p, out);
        e = hipGetLastError();
        if (e != hipSuccess) return hip_fail(e);
    }
    return REDUX_OK;
}

int redux_sum_multipass(const void *x, size_t n, int dtype, void *out, int *levels, void *stream)
{
    std::call_once(g_env_once, read_env);
    if (dtype != REDUX_F16 && dtype != REDUX_I8) return REDUX_ERR_DTYPE;     // this form exists for the paper's binary16 (and int8)
    size_t es = 0;
    int rc = check_common(x, n, dtype, out, 1, &es);
    if (rc != REDUX_OK) return rc;
    if (levels) *levels = 0;

    hipStream_t st = (hipStream_t)stream;
    if (n == 0) return launch_empty_sum(dtype, out, st);

    Settings S;
    int dev = 0, cus = 0;
    hipError_t e;
    {
        std::lock_guard<std::mutex> lock(g_mu);
        S = g_set;
        e = hipGetDevice(&dev);
        if (e != hipSuccess) return hip_fail(e);
        if ((rc = device_cus(dev, &cus)) != REDUX_OK) return rc;
    }

    // group size m*m (m = 4, 16 or 32) for binary16; the int8 form has one shape (16 x 32, then 16 x 16)
    const int m = dtype == REDUX_F16 ? (int)S.lit_m : 16;
    const bool half = S.lit_half != 0;                  // binary16 throughout: the measuring form for binary16 and m = 16
    if (half && (dtype != REDUX_F16 || m != 16)) return REDUX_ERR_PARAM;
    const u64 group = (u64)m * m;
    const u64 first_group = dtype == REDUX_F16 ? group : (u64)kLitGroupI8;
    const u64 tile = m == 32 ? 1024 : 256;                                   // elements one wavefront step consumes
    const size_t ps = dtype == REDUX_F16 ? sizeof(float) : sizeof(i64);     // size of a partial sum
    const u64 n1 = ((u64)n + first_group - 1) / first_group;                 // partial sums after level 1
    const u64 n2 = (n1 + group - 1) / group;                                 // ... after level 2
    LevelBuffers lb;
    if (n1 > 1) {
        std::lock_guard<std::mutex> lock(g_mu);
        if ((rc = get_level_buffers(dev, st, (size_t)n1 * ps + 16, (size_t)n2 * ps + 16, &lb)) != REDUX_OK) return rc;
    }

    // measured best on MI355X (these kernels are bound by the matrix unit, not by HBM)
    const int U = S.lit_unroll ? (int)S.lit_unroll : (dtype == REDUX_I8 ? 4 : m == 4 ? 4 : m == 16 ? 16 : 8);
    const u64 bpc = S.lit_blocks_per_cu ? (u64)S.lit_blocks_per_cu : (dtype == REDUX_I8 ? 8 : m == 32 ? 2 : 4);
    const void *in = x;
    u64 count = n;
    int level = 0;
    while (true) {
        const u64 gsz = level == 0 ? first_group : group;
        const u64 ngroups = (count + gsz - 1) / gsz;
        const u64 ntiles = dtype == REDUX_F16 ? (count + tile - 1) / tile : ngroups;
        void *outp = ngroups == 1 ? out : lb.buf[level & 1];
        const u64 nbatch = (ntiles + U - 1) / U;
        u64 blocks = (nbatch + kWaves - 1) / kWaves;
        u64 gmax = (u64)cus * bpc;
        if (gmax > (u64)S.max_grid) gmax = (u64)S.max_grid;
        const unsigned grid = (unsigned)(blocks < gmax ? blocks : gmax);
        const bool first = level == 0;
        const bool fast = ((uintptr_t)in % (dtype == REDUX_F16 && m == 32 ? 16 : 8)) == 0;
#define REDUX_LIT_U(CALL) switch (U) { case 16: CALL(16); break; case 8: CALL(8); break; case 4: CALL(4); break; \
                                       case 2: CALL(2); break; default: CALL(1); break; }
        if (half) {
#define REDUX_LIT_HALF(UU) launch_literal_half<UU>(fast, ngroups == 1, in, count, outp, grid, st)
            REDUX_LIT_U(REDUX_LIT_HALF)
#undef REDUX_LIT_HALF
        } else if (dtype == REDUX_F16) {
#define REDUX_LIT_M4(UU) launch_literal_f16<4, UU>(first, fast, in, count, outp, grid, st)
#define REDUX_LIT_M16(UU) launch_literal_f16<16, UU>(first, fast, in, count, outp, grid, st)
#define REDUX_LIT_M32(UU) launch_literal_f16<32, UU>(first, fast, in, count, outp, grid, st)
            if (m == 4) REDUX_LIT_U(REDUX_LIT_M4)
            else if (m == 32) REDUX_LIT_U(REDUX_LIT_M32)
            else REDUX_LIT_U(REDUX_LIT_M16)
#undef REDUX_LIT_M4
#undef REDUX_LIT_M16
#undef REDUX_LIT_M32
        } else {
#define REDUX_LIT_I8(UU) launch_literal_i8<UU>(first, fast, in, count, outp, grid, st)
            REDUX_LIT_U(REDUX_LIT_I8)
#undef REDUX_LIT_I8
        }
#undef REDUX_LIT_U
        e = hipGetLastError();
        if (e != hipSuccess) return hip_fail(e);
        ++level;
        if (ngroups == 1) break;
        in = outp;
        count = ngroups;
    }
    if (levels) *levels = level;
    return REDUX_OK;
}

int redux_mma_group_probe(const void *x, size_t count, int dtype, void *D, void *Dprime, void *stream)
{
    if (dtype != REDUX_F16 && dtype != REDUX_I8) return REDUX_ERR_DTYPE;
    if (count > (dtype == REDUX_F16 ? 512u : 1024u)) return REDUX_ERR_SIZE;
    if ((!x && count) || !D || !Dprime) return REDUX_ERR_NULL;
    if ((uintptr_t)x % (dtype == REDUX_F16 ? 2 : 1) || (uintptr_t)D % 4 || (uintptr_t)Dprime % (dtype == REDUX_F16 ? 4 : 8))
        return REDUX_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    if (dtype == REDUX_F16)
        hipLaunchKernelGGL(group_probe_f16_kernel, dim3(1), dim3(64), 0, st, (const unsigned short *)x, (unsigned)count,
                           (float *)D, (float *)Dprime);
    else
        hipLaunchKernelGGL(group_probe_i8_kernel, dim3(1), dim3(64), 0, st, (const signed char *)x, (unsigned)count,
                           (int *)D, (double *)Dprime);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? REDUX_OK : hip_fail(e);
}

int redux_calibration_copy(void *dst, const void *src, size_t nbytes, void *stream)
{
    if ((!dst || !src) && nbytes) return REDUX_ERR_NULL;
    if ((uintptr_t)dst % 16 || (uintptr_t)src % 16 || nbytes % 16) return REDUX_ERR_ALIGN;
    if (nbytes == 0) return REDUX_OK;
    std::lock_guard<std::mutex> lock(g_mu);
    int dev = 0, cus = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e);
    int rc = device_cus(dev, &cus);
    if (rc != REDUX_OK) return rc;
    hipLaunchKernelGGL(copy_kernel, dim3((unsigned)cus * 4), dim3(kBlock), 0, (hipStream_t)stream,
                       (u32x4 *)dst, (const u32x4 *)src, (u64)(nbytes / 16));
    e = hipGetLastError();
    return e == hipSuccess ? REDUX_OK : hip_fail(e);
}

int redux_plan_sum(size_t n, int dtype, uintptr_t x_address, int compute_units, redux_plan *plan)
{
    if (!plan) return REDUX_ERR_NULL;
    const size_t es = elem_size_of(dtype);
    if (es == 0) return REDUX_ERR_DTYPE;
    if (n > ((size_t)1 << 62) / es) return REDUX_ERR_SIZE;
    if (compute_units < 1) return REDUX_ERR_PARAM;
    std::lock_guard<std::mutex> lock(g_mu);
    const void *x = (const void *)x_address;
    const Run run = es == 4 ? make_run<4>(x, n) : es == 2 ? make_run<2>(x, n) : make_run<1>(x, n);
    const FlatPlan p = plan_flat(g_set, run.nvec, compute_units, dtype);
    plan->kernel = REDUX_KERNEL_FLAT;
    plan->unroll = p.unroll;
    plan->grid = p.grid;
    plan->finish = p.finish;
    plan->parts = 1;
    plan->part_len = n;
    plan->head = (unsigned)run.nhead;
    plan->tail = (unsigned)run.ntail;
    plan->vectors = run.nvec;
    plan->chain = p.chain;
    return REDUX_OK;
}

int redux_plan_sum_segmented(size_t nseg, size_t seglen, int dtype, uintptr_t x_address, int compute_units, redux_plan *plan)
{
    if (!plan) return REDUX_ERR_NULL;
    const size_t es = elem_size_of(dtype);
    if (es == 0) return REDUX_ERR_DTYPE;
    if (seglen && nseg > ((size_t)1 << 62) / seglen / es) return REDUX_ERR_SIZE;
    if (nseg > ((size_t)1 << 59)) return REDUX_ERR_SIZE;
    if (compute_units < 1 || nseg == 0 || seglen == 0) return REDUX_ERR_PARAM;
    std::lock_guard<std::mutex> lock(g_mu);
    const SegPlan p = plan_segmented(g_set, nseg, seglen, dtype, es, x_address, compute_units);
    plan->kernel = p.kernel;
    plan->unroll = p.unroll;
    plan->grid = p.grid;
    plan->finish = p.parts > 1 ? (seg_finish_in_kernel(g_set, p, nseg) ? (dtype == REDUX_I8 ? 5 : 6) : 2) : 0;
    plan->parts = p.parts;
    plan->part_len = p.part_len;
    plan->head = 0;
    plan->tail = 0;
    plan->vectors = p.nvec;
    plan->chain = p.chain;
    return REDUX_OK;
}

int redux_plan_block_slabs(int layout, uint64_t nslab, uint64_t grid, uint64_t block, uint64_t *start, uint64_t *stride, uint64_t *count)
{
    if (!start || !stride || !count) return REDUX_ERR_NULL;
    if (layout < 0 || layout > 2 || grid < 1 || block >= grid) return REDUX_ERR_PARAM;
    u64 s = 0, st = 0, c = 0;
    slab_schedule(layout, nslab, grid, block, &s, &st, &c);
    *start = s;
    *stride = st;
    *count = c;
    return REDUX_OK;
}

int redux_plan_run_share(int layout, uint64_t nseg, unsigned per_run, uint64_t grid, uint64_t block, unsigned wave,
                         uint64_t *first, uint64_t *stride, uint64_t *rounds, uint64_t *tail_first, unsigned *tail_count)
{
    if (!first || !stride || !rounds || !tail_first || !tail_count) return REDUX_ERR_NULL;
    if (layout < 0 || layout > 2 || per_run < 1 || per_run > 16 || grid < 1 || grid > (uint64_t)kMaxGrid || block >= grid ||
        wave >= (unsigned)kWaves) return REDUX_ERR_PARAM;
    const RunShare r = run_share(layout, nseg, per_run, grid, block, wave);
    *first = r.first;
    *stride = r.stride;
    *rounds = r.full;
    *tail_first = r.tail_first;
    *tail_count = r.tail_count;
    return REDUX_OK;
}

int redux_set_variant(int variant)
{
    std::call_once(g_env_once, read_env);
    if (variant < REDUX_VARIANT_AUTO || variant > REDUX_VARIANT_CLASSIC) return REDUX_ERR_PARAM;
    std::lock_guard<std::mutex> lock(g_mu);
    g_set.variant = variant;
    return REDUX_OK;
}

int redux_get_variant(void)
{
    std::call_once(g_env_once, read_env);
    std::lock_guard<std::mutex> lock(g_mu);
    return g_set.variant;
}

int redux_resolved_variant(int dtype, int segmented)
{
    std::call_once(g_env_once, read_env);
    if (elem_size_of(dtype) == 0) return REDUX_ERR_DTYPE;
    std::lock_guard<std::mutex> lock(g_mu);
    return effective_variant(g_set, dtype, segmented == 0);
}

int redux_set_param(const char *name, long value)
{
    std::lock_guard<std::mutex> lock(g_mu);
    long lo = 0, hi = 0;
    long *slot = param_slot(name, &lo, &hi);
    if (!slot || value < lo || value > hi) return REDUX_ERR_PARAM;
    if ((slot == &g_set.unroll || slot == &g_set.lit_unroll) && (value & (value - 1)) != 0)
        return REDUX_ERR_PARAM;   // 0 or a power of two
    if (slot == &g_set.lit_m && value != 4 && value != 16 && value != 32) return REDUX_ERR_PARAM;
    *slot = value;
    return REDUX_OK;
}

long redux_get_param(const char *name)
{
    std::lock_guard<std::mutex> lock(g_mu);
    long lo = 0, hi = 0;
    long *slot = param_slot(name, &lo, &hi);
    return slot ? *slot : LONG_MIN;
}

const char *redux_strerror(int status)
{
    switch (status) {
    case REDUX_OK: return "success";
    case REDUX_ERR_NULL: return "null pointer for a non-empty input or for the output";
    case REDUX_ERR_DTYPE: return "unknown dtype";
    case REDUX_ERR_SIZE: return "size overflows or exceeds the supported range";
    case REDUX_ERR_ALIGN: return "pointer not aligned to its element size";
    case REDUX_ERR_HIP: return "a HIP call failed (see redux_last_hip_error)";
    case REDUX_ERR_NOMEM: return "workspace allocation failed";
    case REDUX_ERR_ALIAS: return "output lies inside the input range";
    case REDUX_ERR_PARAM: return "unknown parameter name or value out of range";
    case REDUX_ERR_SCRATCH: return "redux_sum_static: the call needs more block partials (or a higher device ordinal) than its static scratch array provides";
    default: return "unknown status";
    }
}

int redux_last_hip_error(void) { return t_last_hip; }

void redux_shutdown(void)
{
    std::lock_guard<std::mutex> lock(g_mu);
    for (auto &kv : g_ws) (void)hipFree(kv.second.partials);
    g_ws.clear();
    for (auto &kv : g_levels)
        for (int i = 0; i < 2; ++i)
            if (kv.second.buf[i]) (void)hipFree(kv.second.buf[i]);
    g_levels.clear();
    for (void *p : g_retired) (void)hipFree(p);
    g_retired.clear();
    g_cus.clear();
}

const char *redux_version(void) { return "libredux 0.1 (gfx950)"; }

} // extern "C"
