// redux_short.h -- segmented sum of short segments (up to 4 KiB each), read as one contiguous stream.
//
// Aligned form: a segment is 2^lg whole 16-byte vectors (lg = 0 .. 8) and the array starts on a 16-byte
// boundary, so every wavefront-wide load (64 vectors, 1 KiB) holds whole segments and the grid can read
// the array exactly like the flat sum does.  What changes is the constant operand of the two MMAs of
// Section IV-A: instead of all ones they are 0/1 *selection* matrices, so one MMA pair yields many
// independent sums instead of one.
//
//   first MMA   D <- A x B_t + D.  Lane l of a load holds vector l, which the matrix unit reads as
//               A[l % 16][k-group l / 16].  B_t has ones only where k-group g meets column c(t, g), so
//               D[i][c(t, g)] is the sum of the elements of vector 16 g + i of load t: up to four
//               loads (sixteen k-groups) share one accumulator and fill its sixteen columns with 256
//               per-vector sums.  For segments of 32 or 64 vectors two or four k-groups share a column; for
//               128 or 256 vectors (2 or 4 KiB) two or four whole loads of the wavefront do.
//   second MMA  D' <- S x D with S[m][i] = 1 where row i belongs to sub-segment m of its column
//               (i >> lg == m): D'[m][c] is the sum of segment m of column c.  For segments of sixteen
//               vectors or more S is all ones, the second MMA of the paper.
//
// The classic family adds each vector inside its lane and stops the lane butterfly of Section III
// after lg steps.
//
// Ragged form: any segment length up to 1008 bytes at any element alignment.  A group of 2^lg lanes still
// owns one segment, but lane j of the group loads the j-th 16-byte aligned vector that overlaps the segment
// and clears the bytes outside it (the zero padding of Section IV-A, applied per segment).  Everything after
// the load is the aligned form.
//
// A zero in a selection matrix still multiplies its data: an infinity or NaN in one segment would turn
// the other segments of its accumulator into NaN (0 x inf).  So whenever an accumulator yields a
// non-finite result -- which every non-finite input forces in its own segment -- the wavefront's part of
// that slab is read again after the streaming loop and summed with the lane butterfly, which never mixes
// segments.
#pragma once
#include "redux_kernels.h"

namespace redux {

constexpr int kShortLoads = 8;                                   // 16-byte loads per lane per slab
constexpr u64 kShortSlab = (u64)kBlock * kShortLoads;            // (virtual) vectors per slab: 32 KiB when aligned

struct ShortArgs {
    const unsigned char *x;  // first element; aligned form: on a 16-byte boundary
    u64 nseg;
    u64 nvec;           // nseg << lg: lane slots, one 16-byte vector each
    u64 seg_bytes;      // ragged form: bytes per segment
    unsigned lg;        // log2(lane slots per segment): 0 .. 6, aligned form of the MMA family also 7 and 8
    void *out;
    int layout;         // see slab_schedule
    int pipe;           // 0 = plain loop, 1 = refill each register as soon as it is consumed
};

// slot index, inside its slab, that load u of thread tid fills: every load of the block covers 256
// consecutive slots (4 KiB contiguous when aligned), every wavefront 64 of them
// (segments of more than 64 slots: every wavefront owns 512 consecutive slots, so that a segment stays in one wavefront)
__device__ __forceinline__ unsigned short_index(int u, unsigned tid, bool wide)
{
    return wide ? (tid >> 6) * (64u * kShortLoads) + (unsigned)u * 64u + (tid & 63u) : (unsigned)u * kBlock + tid;
}

// The vector of slot V (V < a.nvec).  Aligned form: vector V of the array.  Ragged form: slot V is lane
// j = V mod 2^lg of segment V >> lg; it reads the j-th aligned vector overlapping that segment and keeps the
// segment's bytes only.  An aligned vector that holds at least one byte of the array lies in the array's
// pages, so the bytes read beyond either end of the array are mapped; they are cleared like all others.
// Returns the vector as loaded and, in *m, which entry of the byte-mask table clears what is not the segment's:
// the AND is left to the consumer, so that the load can stay in flight.
template <bool NT, bool RAGGED>
__device__ __forceinline__ u32x4 short_fetch(const ShortArgs &a, u64 V, unsigned *m)
{
    if (!RAGGED) { *m = 0; return load16<NT>((const u32x4 *)a.x + V); }
    const u64 seg = V >> a.lg;
    const unsigned j = (unsigned)V & ((1u << a.lg) - 1u);
    // (pointer arithmetic on the kernel argument, not integer arithmetic on its value: the compiler then knows the
    // address is global memory and issues global, not flat, loads -- a flat load also counts as an LDS operation, and
    // every wait for the byte-mask table would wait for it)
    const unsigned char *first = a.x + seg * a.seg_bytes;            // the segment's first byte
    const unsigned off = (unsigned)(uintptr_t)first & 15u;
    const unsigned end = off + (unsigned)a.seg_bytes;                // segment end, in bytes from its first aligned vector
    const unsigned cover = (end + 15u) >> 4;                         // aligned vectors that overlap the segment (at least 1)
    // Lanes past the last overlapping vector read that vector again (the same cache line as their neighbour: no
    // extra traffic) and keep nothing of it, so that every lane issues its load and waits can be counted.
    const unsigned jj = j < cover ? j : cover - 1u;
    const u32x4 v = load16<NT>((const u32x4 *)(first - off) + jj);
    // bytes [lo, hi) of the vector belong to the segment
    const unsigned lo = j == 0 ? off : 0u;
    const unsigned hi = j >= cover ? 0u : (end - 16u * j >= 16u ? 16u : end - 16u * j);
    *m = lo * 17u + hi;
    return v;
}

// `count` (1, 2 or 4) consecutive results of one lane, as one store where alignment allows
template <class Out>
__device__ __forceinline__ void short_store(Out *p, const Out *v, unsigned count, u64 room)
{
    typedef Out Out4 __attribute__((ext_vector_type(4)));
    typedef Out Out2 __attribute__((ext_vector_type(2)));
    if (count == 4 && room >= 4 && ((uintptr_t)p & (4 * sizeof(Out) - 1)) == 0) {
        *(Out4 *)p = Out4{v[0], v[1], v[2], v[3]};
    } else if (count == 2 && room >= 2 && ((uintptr_t)p & (2 * sizeof(Out) - 1)) == 0) {
        *(Out2 *)p = Out2{v[0], v[1]};
    } else {
#pragma unroll
        for (unsigned r = 0; r < 4; ++r)
            if (r < count && r < room) p[r] = v[r];
    }
}

// first MMA with a 0/1 column selector as the constant operand: `sel` says whether this lane's slice of
// B is ones (its k-group feeds the column the lane holds) or zeros
template <int KIND>
__device__ __forceinline__ f32x4 mma1_select(u32x4 v, bool sel, f32x4 d)
{
    if (KIND == kF16) {
        const unsigned w = sel ? 0x3C003C00u : 0u;
        const u32x4 b = {w, w, w, w};
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, v), __builtin_bit_cast(f16x8, b), d, 0, 0, 0);
    } else if (KIND == kBF16) {
        const unsigned w = sel ? 0x3F803F80u : 0u;
        const u32x4 b = {w, w, w, w};
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, v), __builtin_bit_cast(bf16x8, b), d, 0, 0, 0);
    } else if (KIND == kF32) {
        const f32x4 f = __builtin_bit_cast(f32x4, v);
        const float b = sel ? 1.0f : 0.0f;
#pragma unroll
        for (int k = 0; k < 4; ++k) d = __builtin_amdgcn_mfma_f32_16x16x4f32(f[k], b, d, 0, 0, 0);
        return d;
    } else {
        const long lo = (long)(((u64)v[1] << 32) | v[0]), hi = (long)(((u64)v[3] << 32) | v[2]);
        if (KIND == kE4M3) {
            const long b = sel ? 0x3838383838383838L : 0L;
            d = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(lo, b, d, 0, 0, 0);
            return __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(hi, b, d, 0, 0, 0);
        } else {
            const long b = sel ? 0x3C3C3C3C3C3C3C3CL : 0L;
            d = __builtin_amdgcn_mfma_f32_16x16x32_bf8_bf8(lo, b, d, 0, 0, 0);
            return __builtin_amdgcn_mfma_f32_16x16x32_bf8_bf8(hi, b, d, 0, 0, 0);
        }
    }
}

// Element policies: how one vector enters the first MMA (or is added inside a lane), and how a
// per-segment result leaves.
template <int KIND>
struct ShortFloat {
    static constexpr bool kCanBeNonFinite = true;
    typedef float Out;
    typedef f32x4 Acc;
    typedef float Lane;
    static __device__ __forceinline__ Acc zero() { return f32x4{0.f, 0.f, 0.f, 0.f}; }
    static __device__ __forceinline__ Acc mma1(u32x4 v, bool sel, Acc d) { return mma1_select<KIND>(v, sel, d); }
    static __device__ __forceinline__ float fold_in(const Acc &d, int r) { return d[r]; }
    static __device__ __forceinline__ Out fold_out(float f) { return f; }
    static __device__ __forceinline__ Out fold_out_wide(float f) { return f; }
    static __device__ __forceinline__ Lane lane_sum(u32x4 v)
    {
        float s[4] = {0.f, 0.f, 0.f, 0.f};
        add_vector<KIND>(s, v);
        return (s[0] + s[1]) + (s[2] + s[3]);
    }
    static __device__ __forceinline__ Out lane_out(Lane v) { return v; }
};

// int8: a vector sums to at most 16 x 128 and a segment to at most 64 times that, so the binary32
// second MMA (and the int32 lane butterfly) are exact.
struct ShortI8 {
    static constexpr bool kCanBeNonFinite = false;
    typedef i64 Out;
    typedef i32x4 Acc;
    typedef int Lane;
    static __device__ __forceinline__ Acc zero() { return i32x4{0, 0, 0, 0}; }
    static __device__ __forceinline__ Acc mma1(u32x4 v, bool sel, Acc d)
    {
        const int w = sel ? 0x01010101 : 0;
        const i32x4 b = {w, w, w, w};
        return __builtin_amdgcn_mfma_i32_16x16x64_i8(__builtin_bit_cast(i32x4, v), b, d, 0, 0, 0);
    }
    static __device__ __forceinline__ float fold_in(const Acc &d, int r) { return (float)d[r]; }
    static __device__ __forceinline__ Out fold_out(float f) { return (i64)f; }
    static __device__ __forceinline__ Out fold_out_wide(i64 v) { return v; }
    static __device__ __forceinline__ Lane lane_sum(u32x4 v)
    {
        int s = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) s = __builtin_amdgcn_sdot4((int)v[k], 0x01010101, s, false);
        return s;
    }
    static __device__ __forceinline__ Out lane_out(Lane v) { return (i64)v; }
};

// One whole slab into registers.
// (CANWIDE: whether this kernel is ever launched for segments of more than 64 slots)
template <bool NT, bool RAGGED, bool CANWIDE>
__device__ __forceinline__ void short_load(u32x4 *dst, unsigned *m, const ShortArgs &a, u64 slab, unsigned tid)
{
#pragma unroll
    for (int u = 0; u < kShortLoads; ++u)
        dst[u] = short_fetch<NT, RAGGED>(a, slab * kShortSlab + short_index(u, tid, CANWIDE && a.lg >= 7), &m[u]);
}

// The slab that holds the end of the array; slots past the end read zeros.
template <bool NT, bool RAGGED, bool CANWIDE>
__device__ __forceinline__ void short_load_partial(u32x4 *dst, unsigned *m, const ShortArgs &a, u64 slab, unsigned tid)
{
#pragma unroll
    for (int u = 0; u < kShortLoads; ++u) {
        const u64 V = slab * kShortSlab + short_index(u, tid, CANWIDE && a.lg >= 7);
        u32x4 v = {0u, 0u, 0u, 0u};
        m[u] = 0;                                                    // (entry 0 keeps nothing)
        if (V < a.nvec) v = short_fetch<NT, RAGGED>(a, V, &m[u]);
        dst[u] = v;
    }
}

// `work(cur, m, slab, refill)` does everything for one slab held in `cur` (with mask entries m) and calls refill(u) as
// soon as it has consumed cur[u]: the register is then reloaded with the same block's next slab, so eight loads per
// lane stay in flight while the MMAs (or the butterfly) and the stores run.  The block's last slab is peeled off, so
// that no load in the loop is conditional and the wait in front of each use leaves exactly the seven newer loads
// outstanding.  The slab that holds the ragged end of the array is done by one block afterwards.
//
// work returns whether any of this wavefront's results of the slab must be computed again (the same answer in every
// lane); `redo(cur, m, slab)` does that.  It runs after the streaming loops, over the range of slabs that asked for it:
// anything heavier than a flag inside those loops -- above all a load under a branch -- costs them their pipelining.
template <bool NT, bool RAGGED, bool CANWIDE, class Work, class Redo>
__device__ __forceinline__ void short_stream(const ShortArgs &a, unsigned tid, Work &&work, Redo &&redo)
{
    const u64 nfull = a.nvec / kShortSlab;
    u64 s0, stride, count;
    slab_schedule(a.layout, nfull, gridDim.x, blockIdx.x, &s0, &stride, &count);
    u64 redo_first = ~0ull, redo_last = 0;                           // positions in this block's schedule
    if (count && a.pipe == 0) {
        for (u64 k = 0; k < count; ++k) {
            u32x4 cur[kShortLoads];
            unsigned m[kShortLoads];
            short_load<NT, RAGGED, CANWIDE>(cur, m, a, s0 + k * stride, tid);
            __builtin_amdgcn_sched_barrier(0);
            if (work(cur, m, s0 + k * stride, [](int) {})) {
                redo_first = redo_first < k ? redo_first : k;
                redo_last = k;
            }
        }
    } else if (count) {
        u32x4 cur[kShortLoads];
        unsigned m[kShortLoads];
        // Ragged form: what short_fetch derives from a slot -- where its vector lies relative to the slab and which bytes
        // of it belong to the segment -- is the same in every slab.  A slab holds 2048 >> lg whole segments, a multiple
        // of sixteen, so its first segment starts a multiple of 16 bytes behind the array's first byte, and slot
        // (u, tid) meets the same alignment in every slab.  So the byte offsets and mask entries are worked out once;
        // inside the loop a load is the slab's (wavefront-uniform) address plus a fixed 32-bit offset per lane.
        unsigned voff[kShortLoads];
        const unsigned xo = (unsigned)(uintptr_t)a.x & 15u;
        const unsigned char *xa = a.x - xo;                                   // (pointer arithmetic: stays a global address)
        const u64 slab_bytes = (u64)(kShortSlab >> a.lg) * a.seg_bytes;      // bytes of the segments of one slab
        if (RAGGED) {
#pragma unroll
            for (int u = 0; u < kShortLoads; ++u) {
                const unsigned idx = short_index(u, tid, false);
                const unsigned j = idx & ((1u << a.lg) - 1u);
                const unsigned rel = xo + (idx >> a.lg) * (unsigned)a.seg_bytes;  // first byte of the segment, from xa
                const unsigned off = rel & 15u;
                const unsigned end = off + (unsigned)a.seg_bytes;
                const unsigned cover = (end + 15u) >> 4;
                const unsigned jj = j < cover ? j : cover - 1u;
                voff[u] = rel - off + 16u * jj;
                const unsigned lo = j == 0 ? off : 0u;
                const unsigned hi = j >= cover ? 0u : (end - 16u * j >= 16u ? 16u : end - 16u * j);
                m[u] = lo * 17u + hi;
            }
        }
        // vector of slot (u, tid) of slab `sl`
        auto fetch = [&](u64 sl, int u) -> u32x4 {
            if (RAGGED) return load16<NT>((const u32x4 *)(xa + sl * slab_bytes + voff[u]));
            return short_fetch<NT, false>(a, sl * kShortSlab + short_index(u, tid, CANWIDE && a.lg >= 7), &m[u]);
        };
#pragma unroll
        for (int u = 0; u < kShortLoads; ++u) {      // issued strictly in the order they are consumed in: the waits count on it
            cur[u] = fetch(s0, u);
            __builtin_amdgcn_sched_barrier(0);
        }
        u64 slab = s0;
        for (u64 k = 1; k < count; ++k, slab += stride) {
            const u64 next = slab + stride;
            __builtin_amdgcn_sched_barrier(0);
            const bool again = work(cur, m, slab, [&](int u) {
                cur[u] = fetch(next, u);
                __builtin_amdgcn_sched_barrier(0);                   // keep the refill right behind the use
            });
            if (again) {
                redo_first = redo_first < k - 1 ? redo_first : k - 1;
                redo_last = k - 1;
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        if (work(cur, m, slab, [](int) {})) {
            redo_first = redo_first < count - 1 ? redo_first : count - 1;
            redo_last = count - 1;
        }
    }
    if (redo_first <= redo_last) {
        __builtin_amdgcn_s_waitcnt(0);                               // the first pass's stores have landed
        for (u64 k = redo_first; k <= redo_last; ++k) {
            u32x4 cur[kShortLoads];
            unsigned m[kShortLoads];
            short_load<NT, RAGGED, CANWIDE>(cur, m, a, s0 + k * stride, tid);
            redo(cur, m, s0 + k * stride);
        }
    }
    if (nfull * kShortSlab < a.nvec && blockIdx.x == (unsigned)(nfull % gridDim.x)) {
        u32x4 last[kShortLoads];
        unsigned m[kShortLoads];
        short_load_partial<NT, RAGGED, CANWIDE>(last, m, a, nfull, tid);
        if (work(last, m, nfull, [](int) {})) {
            __builtin_amdgcn_s_waitcnt(0);
            redo(last, m, nfull);
        }
    }
}

template <class T, int CTRL>
__device__ __forceinline__ T dpp_add(T v)
{
    return v + __builtin_bit_cast(T, dpp_i32<CTRL>(__builtin_bit_cast(int, v)));
}

// The lane butterfly of Section III over the 2^lg lanes of a segment (lg is the same for every lane):
// afterwards every lane of a segment holds the segment's sum.
template <class Lane>
__device__ __forceinline__ Lane short_butterfly(Lane s, unsigned lg)
{
    if (lg >= 1) s = dpp_add<Lane, kQuadXor1>(s);
    if (lg >= 2) s = dpp_add<Lane, kQuadXor2>(s);
    if (lg >= 3) s = dpp_add<Lane, kRowHalfMirror>(s);
    if (lg >= 4) s = dpp_add<Lane, kRowMirror>(s);
    if (lg >= 5) s = s + __builtin_bit_cast(Lane, __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, s), kSwizzleXor16));
    if (lg >= 6) s = __builtin_bit_cast(Lane, __builtin_amdgcn_readlane(__builtin_bit_cast(int, s), 0)) +
                     __builtin_bit_cast(Lane, __builtin_amdgcn_readlane(__builtin_bit_cast(int, s), 32));
    return s;
}

// one load of the classic family: the vector in v fills slot V (segments of up to 64 slots)
template <class E>
__device__ __forceinline__ void short_classic_one(const ShortArgs &a, u32x4 v, u64 V, unsigned lane)
{
    const typename E::Lane s = short_butterfly(E::lane_sum(v), a.lg);
    const u64 seg = V >> a.lg;
    if ((lane & ((1u << a.lg) - 1u)) == 0 && seg < a.nseg) ((typename E::Out *)a.out)[seg] = E::lane_out(s);
}

// Loads U0 .. U0 + COUNT - 1 of one slab through the classic family; get(u) hands over vector u and may start its
// refill.  Segments of 128, 256 or 512 slots span 2, 4 or 8 loads of the wavefront: their lane sums are added up
// before the butterfly.
template <class E, int U0, int COUNT, bool CANWIDE, class Get>
__device__ __forceinline__ void short_classic_range(const ShortArgs &a, u64 slab, unsigned tid, Get &&get)
{
    const unsigned lane = tid & 63u;
    if (!CANWIDE || a.lg <= 6) {
#pragma unroll
        for (int u = U0; u < U0 + COUNT; ++u) {
            const u32x4 v = get(u);
            short_classic_one<E>(a, v, slab * kShortSlab + short_index(u, tid, false), lane);
        }
    } else {
        const unsigned per_seg = 1u << (a.lg - 6);               // loads per segment
        typename E::Lane s = 0;
#pragma unroll
        for (int u = U0; u < U0 + COUNT; ++u) {
            s = s + E::lane_sum(get(u));
            if ((((unsigned)u + 1u) & (per_seg - 1u)) == 0) {
                const typename E::Lane total = short_butterfly(s, 6);
                const u64 seg = (slab * kShortSlab + short_index(u, tid, true)) >> a.lg;
                if (lane == 0 && seg < a.nseg) ((typename E::Out *)a.out)[seg] = E::lane_out(total);
                s = 0;
            }
        }
    }
}

// LPA = loads that share one accumulator: 4 for segments up to sixteen vectors (four columns per load),
// 8 for segments of 32 or 64 vectors (two columns or one column per load).
template <class E, int LPA, bool NT, bool RAGGED>
__global__ void __launch_bounds__(kBlock) sum_short_mfma_kernel(ShortArgs a)
{
    constexpr int U = kShortLoads;
    constexpr int NACC = U / LPA;
    const unsigned tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    __shared__ u32x4 masks[RAGGED ? kByteMasks : 1];
    if (RAGGED) fill_byte_masks(masks);
    const unsigned g = lane >> 4, n = lane & 15u;
    const unsigned lg = a.lg;
    const unsigned cpl = LPA == 4 ? 4u : (lg == 5 ? 2u : 1u);      // columns per load
    constexpr bool CANWIDE = LPA == 8 && !RAGGED;
    const bool wide = CANWIDE && lg >= 7;                          // a segment spans 2, 4 or 8 loads of the wavefront
    const unsigned sh = wide ? lg - 6u : 0u;
    const unsigned lgc = lg < 4 ? lg : 4u;
    const unsigned mask = (16u >> lgc) - 1u;                       // segments per column - 1

    // first MMA: k-group g of load t feeds column t * cpl + g * cpl / 4 (wide: all of load t feeds column t >> sh)
    bool sel[LPA];
#pragma unroll
    for (int t = 0; t < LPA; ++t) sel[t] = (n == (wide ? (unsigned)t >> sh : (unsigned)t * cpl + (g * cpl) / 4u));
    // second MMA, step r: the A operand of this lane is S[m = n][i = 4 g + r]
    float srow[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) srow[r] = (((4u * g + (unsigned)r) >> lgc) == (n & mask)) ? 1.0f : 0.0f;
    // after the second MMA this lane holds rows m = 4 g + r' of column n: the sums of segments m of
    // the 64 / cpl slots that start at slot col_off of load col_load
    const bool col_used = n < (wide ? 8u >> sh : (unsigned)LPA * cpl) && 4u * g <= mask;
    const unsigned col_load = wide ? n << sh : n / cpl;
    const unsigned col_off = (n % cpl) * (64u / cpl);
    const unsigned per_lane = mask >= 3u ? 4u : mask + 1u;        // results this lane writes per accumulator: 4, 2 or 1
    typename E::Out *out = (typename E::Out *)a.out;

    short_stream<NT, RAGGED, CANWIDE>(a, tid, [&](const u32x4 *cur, const unsigned *m, u64 slab, auto refill) {
        bool again = false;                                        // some accumulator holds a non-finite value
#pragma unroll
        for (int q = 0; q < NACC; ++q) {
            typename E::Acc d = E::zero();
#pragma unroll
            for (int t = 0; t < LPA; ++t) {
                const u32x4 v = RAGGED ? (cur[q * LPA + t] & masks[m[q * LPA + t]]) : cur[q * LPA + t];
                d = E::mma1(v, sel[t], d);
                refill(q * LPA + t);
            }
            f32x4 dp = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int r = 0; r < 4; ++r) dp = __builtin_amdgcn_mfma_f32_16x16x4f32(srow[r], E::fold_in(d, r), dp, 0, 0, 0);
            if (E::kCanBeNonFinite) {
                // finite - finite is 0; infinities and NaNs give NaN, which differs from itself
                const f32x4 z = dp - dp;
                again |= (z[0] != 0.f) | (z[1] != 0.f) | (z[2] != 0.f) | (z[3] != 0.f);
            }
            if (col_used) {
                const u64 vb = slab * kShortSlab + short_index(q * LPA + (int)col_load, wave * 64u, wide) + col_off;
                const u64 seg0 = (vb >> lg) + 4u * g;
                if (seg0 < a.nseg) {
                    const typename E::Out res[4] = {E::fold_out(dp[0]), E::fold_out(dp[1]), E::fold_out(dp[2]), E::fold_out(dp[3])};
                    short_store(out + seg0, res, per_lane, a.nseg - seg0);
                }
            }
        }
        return __builtin_amdgcn_ballot_w64(again) != 0;            // the same for the whole wavefront
    }, [&](const u32x4 *cur, const unsigned *m, u64 slab) {
        // the whole slab of this wavefront again, with the lane butterfly, which never mixes segments
        short_classic_range<E, 0, kShortLoads, CANWIDE>(a, slab, tid, [&](int u) { return RAGGED ? (cur[u] & masks[m[u]]) : cur[u]; });
    });
}

template <class E, bool NT, bool RAGGED>
__global__ void __launch_bounds__(kBlock) sum_short_classic_kernel(ShortArgs a)
{
    const unsigned tid = threadIdx.x;
    __shared__ u32x4 masks[RAGGED ? kByteMasks : 1];
    if (RAGGED) fill_byte_masks(masks);
    // (segments of more than 64 slots never come here: the host gives them to the MMA family only)
    short_stream<NT, RAGGED, false>(a, tid, [&](const u32x4 *cur, const unsigned *m, u64 slab, auto refill) {
        short_classic_range<E, 0, kShortLoads, false>(a, slab, tid, [&](int u) {
            const u32x4 v = RAGGED ? (cur[u] & masks[m[u]]) : cur[u];
            refill(u);
            return v;
        });
        return false;
    }, [](const u32x4 *, const unsigned *, u64) {});
}

} // namespace redux
