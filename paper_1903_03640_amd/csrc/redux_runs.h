// redux_runs.h -- segmented sum of medium segments (about 1 KiB to 256 KiB each, any length, any alignment).
//
// One wavefront takes a *run* of up to sixteen consecutive whole segments and streams the 16-byte aligned vectors
// that cover it, 64 x 8 at a time, exactly like the flat sum streams the array: every lane of every load holds
// data, whatever the segment length is.  Only the two ends of a run are ragged (a run starts and ends on a segment
// boundary, not on a vector boundary), so two neighbouring runs share at most one vector.
//
// MMA family.  Segment k of the run owns column k of the accumulator: the first MMA of Section IV-A,
// D <- A x B + D, is issued with B = "ones in column k, zeros elsewhere", so row sums of the data land in column k
// (D[i][k] += sum of the vector of lane 16 g + i over the four k-groups g).  A load that holds a segment boundary
// is issued twice, once with the bytes in front of the boundary (into column k) and once with the bytes behind it
// (into column k + 1); the bytes outside are cleared, which is the zero padding of Section IV-A.  Where the
// boundaries fall is the same for every lane of the wavefront, so it is worked out in scalar registers; a lane only
// clamps (boundary - 16 x lane) to 0..16 to find how many of its sixteen bytes lie in front.  At the end of the run
// the second MMA, D' <- 1 x D, adds the sixteen rows of every column at once and lanes 0 .. 15 store one result
// each.  Bytes in front of the run's first segment and behind its last one never enter an MMA.
//
// A zero in B still multiplies its data, so an infinity or NaN in one segment would turn the other columns into NaN:
// a run whose D' holds a non-finite value is computed again by the classic form below, which never mixes segments.
//
// Classic family.  Every lane adds up its vectors; at a boundary the lanes' sums of the finished segment go through
// the wavefront butterfly of Section III and lane 0 stores the result.
#pragma once
#include "redux_short.h"

namespace redux {

struct RunArgs {
    const unsigned char *x;  // first element, aligned to the element size only
    u64 nseg;
    unsigned seg_bytes;      // bytes per segment: 16 .. 2^18 (the run's byte positions are kept in 32 bits)
    unsigned per_run;        // segments per run: 1 .. 16
    void *out;
    int layout;              // 2: every accelerator die takes a contiguous eighth of the segments (see run_share)
};

// Which segments a wavefront takes.  The segments of a part (the whole array, or the eighth of it that belongs to one
// accelerator die: workgroup b runs on die b % 8) are dealt out in rounds: in round k wavefront j of the part's W
// takes the per_run segments from k x W x per_run + j x per_run on, so that at any time the part reads one contiguous
// moving window.  What is left after the last whole round is fewer than W x per_run segments: it is split into W
// nearly equal shares, one last, shorter run for every wavefront, so that all of them finish together whatever the
// number of segments is (dealing out whole runs to the end would leave most wavefronts idle for up to a round).
struct RunShare {
    u64 first;           // first segment of this wavefront's run of round 0
    u64 stride;          // segments from one round to the next
    u64 full;            // whole rounds
    u64 tail_first;      // the last, shorter run ...
    unsigned tail_count; // ... and its segments (0 .. per_run)
};

__host__ __device__ __forceinline__ RunShare run_share(int layout, u64 nseg, unsigned per_run, u64 G, u64 b, unsigned wave)
{
    const bool by_die = layout == 2 && G % (u64)kXcds == 0;      // (equal numbers of workgroups on every die)
    const u64 x = by_die ? b % kXcds : 0, l = by_die ? b / kXcds : b;
    const u64 lo = by_die ? (nseg >> 3) * x + (((nseg & 7u) * x) >> 3) : 0;              // floor(nseg x / 8)
    const u64 hi = by_die ? (nseg >> 3) * (x + 1) + (((nseg & 7u) * (x + 1)) >> 3) : nseg;
    const u64 W = (by_die ? G / kXcds : G) * kWaves;             // wavefronts of the part
    const u64 j = l * kWaves + wave;                             // this one among them
    RunShare r;
    r.stride = W * per_run;
    r.full = (hi - lo) / r.stride;
    const unsigned rest = (unsigned)((hi - lo) - r.full * r.stride);   // < W x per_run <= 2^20
    // floor(rest x j / W) in 32 bits: j <= W <= 2^16, so j x (rest mod W) < 2^32
    const unsigned w = (unsigned)W, q = rest / w, m = rest % w, jj = (unsigned)j;
    const unsigned t0 = jj * q + jj * m / w, t1 = (jj + 1u) * q + (jj + 1u) * m / w;
    r.first = lo + j * per_run;
    r.tail_first = lo + r.full * r.stride + t0;
    r.tail_count = (unsigned)(t1 - t0);                          // <= ceil(rest / W) <= per_run
    return r;
}

// U = 16-byte loads per lane per iteration (4 or 8); an iteration of a wavefront takes 64 x U vectors

// all-ones in the low b bytes of a vector, b = 0 .. 16, as a table in LDS
__device__ __forceinline__ void fill_low_masks(u32x4 *table /* 17 entries, shared */)
{
    if (threadIdx.x < 17u) table[threadIdx.x] = keep_bytes(u32x4{~0u, ~0u, ~0u, ~0u}, 0u, threadIdx.x);
    __syncthreads();
}

// Where a run lies: its first aligned vector, where its first segment starts in it, where its last one ends.
struct RunGeometry {
    const u32x4 *base;   // 16-byte aligned
    unsigned off;        // first byte of the run's first segment, from base (0 .. 15)
    unsigned total;      // first byte behind the run's last segment, from base
    unsigned nvec;       // aligned vectors that overlap the run
    unsigned count;      // segments in this run
    u64 first;           // index of the run's first segment
};

__device__ __forceinline__ RunGeometry run_geometry(const RunArgs &a, u64 first, unsigned count)
{
    RunGeometry g;
    g.first = first;
    g.count = count;
    // (pointer arithmetic on the kernel argument keeps the loads in the global address space)
    const unsigned char *start = a.x + g.first * a.seg_bytes;
    g.off = (unsigned)(uintptr_t)start & 15u;
    g.base = (const u32x4 *)(start - g.off);
    g.total = g.off + g.count * a.seg_bytes;
    g.nvec = (g.total + 15u) >> 4;
    return g;
}

// The 64 x U vectors of one iteration.  Lanes past the run's last vector read that vector again (one cache line
// for all of them); their bytes lie behind the run's end and are dropped like everything there.  An aligned
// vector that holds a byte of the array lies in the array's pages, so nothing unmapped is touched.
template <int U, bool NT>
__device__ __forceinline__ void run_load(u32x4 *cur, const RunGeometry &g, unsigned v0, unsigned lane)
{
    if (v0 + 64u * U <= g.nvec) {
#pragma unroll
        for (int u = 0; u < U; ++u) {              // issued in the order they are used in: the waits count on it
            cur[u] = load16<NT>(g.base + v0 + 64u * (unsigned)u + lane);
            __builtin_amdgcn_sched_barrier(0);
        }
    } else {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const unsigned idx = v0 + 64u * (unsigned)u + lane;
            cur[u] = load16<NT>(g.base + (idx < g.nvec ? idx : g.nvec - 1u));
        }
    }
    __builtin_amdgcn_sched_barrier(0);             // every load of the iteration in flight before the first use waits
}

// Walks the boundaries of a run.  `col` is the segment (0 .. count - 1) that the byte at `next` belongs to once
// the boundary at `next` has been passed; before the first boundary (col = ~0) and behind the last one
// (col = count) bytes belong to no segment of this run.
struct RunCursor {
    unsigned col, next;
    __device__ __forceinline__ void start(const RunGeometry &g) { col = ~0u; next = g.off; }
    __device__ __forceinline__ void pass(const RunGeometry &g, unsigned seg_bytes)
    {
        ++col;                                                        // ~0 -> 0 at the run's first byte
        next = col < g.count ? next + seg_bytes : ~0u;                // no boundary behind the run's end
    }
};

// How many of this lane's sixteen bytes of a load lie in front of the boundary `d` bytes into the load.
__device__ __forceinline__ unsigned bytes_in_front(unsigned d, int lane16)
{
    const int k = (int)d - lane16;
    return (unsigned)(k < 0 ? 0 : k > 16 ? 16 : k);
}

// ---- classic family: one run by the lane sums and the butterfly --------------------------------------------------
template <class E, int U, bool NT>
__device__ __forceinline__ void run_classic(const RunArgs &a, const RunGeometry &g, const u32x4 *low, unsigned lane)
{
    typedef typename E::Out Out;
    Out *out = (Out *)a.out + g.first;
    const int lane16 = 16 * (int)lane;
    typename E::Lane s = 0;                        // this lane's share of the current segment
    RunCursor c;
    c.start(g);
    for (unsigned v0 = 0; v0 < g.nvec; v0 += 64u * U) {
        u32x4 cur[U];
        run_load<U, NT>(cur, g, v0, lane);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const unsigned p = (v0 + 64u * (unsigned)u) * 16u;       // first byte of this load, from base
            if (p >= g.total) continue;                              // (the same for every lane)
            const u32x4 v = cur[u];
            if (c.next - p >= 1024u) {                               // no boundary in this load
                if (c.col < g.count) s = s + E::lane_sum(v);
            } else {
                u32x4 done = {0u, 0u, 0u, 0u};                       // bytes already handed to a segment
                do {
                    const u32x4 front = low[bytes_in_front(c.next - p, lane16)];
                    if (c.col < g.count) {                           // the segment in front of the boundary is complete
                        s = s + E::lane_sum(v & front & ~done);
                        const typename E::Lane t = short_butterfly(s, 6u);
                        if (lane == 0) out[c.col] = E::lane_out(t);
                        s = 0;
                    }
                    done = front;
                    c.pass(g, a.seg_bytes);
                } while (c.next - p < 1024u);
                if (c.col < g.count) s = s + E::lane_sum(v & ~done);
            }
        }
    }
    // A run that ends exactly where its last load ends never meets its last boundary inside a load.
    if (c.col < g.count) {
        const typename E::Lane t = short_butterfly(s, 6u);
        if (lane == 0) out[c.col] = E::lane_out(t);
    }
}

template <class E, int U, bool NT>
__global__ void __launch_bounds__(kBlock) sum_segment_runs_classic_kernel(RunArgs a)
{
    const unsigned lane = threadIdx.x & 63u;
    // (the wavefront's number read into a scalar register: everything about a run is then scalar, branches included)
    const unsigned wave = (unsigned)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    __shared__ u32x4 low[17];
    fill_low_masks(low);
    const RunShare sh = run_share(a.layout, a.nseg, a.per_run, gridDim.x, blockIdx.x, wave);
    for (u64 k = 0; k < sh.full; ++k) run_classic<E, U, NT>(a, run_geometry(a, sh.first + k * sh.stride, a.per_run), low, lane);
    if (sh.tail_count != 0u) run_classic<E, U, NT>(a, run_geometry(a, sh.tail_first, sh.tail_count), low, lane);
}

// ---- MMA family ------------------------------------------------------------------------------------------------------
// second MMA: D' <- 1 x D; every lane gets the total of column lane % 16.  *bad: some column is not finite.
__device__ __forceinline__ float run_fold(const f32x4 &d, bool *bad)
{
    f32x4 dp = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int r = 0; r < 4; ++r) dp = __builtin_amdgcn_mfma_f32_16x16x4f32(1.0f, d[r], dp, 0, 0, 0);
    const float z = dp[0] - dp[0];                 // finite - finite is 0; an infinity or NaN gives NaN
    *bad = z != 0.f;
    return dp[0];
}
// int32 row sums: no MFMA takes int32, so the second MMA runs exactly in binary64 (a column stays far below 2^53)
__device__ __forceinline__ i64 run_fold(const i32x4 &d, bool *bad)
{
    f64x4 dp = {0., 0., 0., 0.};
#pragma unroll
    for (int r = 0; r < 4; ++r) dp = __builtin_amdgcn_mfma_f64_16x16x4f64(1.0, (double)d[r], dp, 0, 0, 0);
    *bad = false;
    return (i64)dp[0];
}

template <class E, int U, bool NT>
__global__ void __launch_bounds__(kBlock) sum_segment_runs_mfma_kernel(RunArgs a)
{
    typedef typename E::Out Out;
    const unsigned lane = threadIdx.x & 63u, n = lane & 15u;
    const int lane16 = 16 * (int)lane;
    // (the wavefront's number read into a scalar register: everything about a run is then scalar, branches included)
    const unsigned wave = (unsigned)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    __shared__ u32x4 low[17];
    fill_low_masks(low);
    const RunShare sh = run_share(a.layout, a.nseg, a.per_run, gridDim.x, blockIdx.x, wave);

    for (u64 k = 0; k <= sh.full; ++k) {
        const bool last = k == sh.full;            // the shorter run behind the whole rounds
        if (last && sh.tail_count == 0u) break;
        const RunGeometry g = run_geometry(a, last ? sh.tail_first : sh.first + k * sh.stride, last ? sh.tail_count : a.per_run);
        typename E::Acc acc = E::zero();           // column k: the sixteen row sums of segment k of the run
        RunCursor c;
        c.start(g);
        for (unsigned v0 = 0; v0 < g.nvec; v0 += 64u * U) {
            u32x4 cur[U];
            run_load<U, NT>(cur, g, v0, lane);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const unsigned p = (v0 + 64u * (unsigned)u) * 16u;   // first byte of this load, from base
                if (p >= g.total) continue;                          // (the same for every lane)
                const u32x4 v = cur[u];
                if (c.next - p >= 1024u) {                           // no boundary in this load: one MMA, nothing cleared
                    if (c.col < g.count) acc = E::mma1(v, n == c.col, acc);
                } else {
                    u32x4 done = {0u, 0u, 0u, 0u};                   // bytes already handed to a segment
                    do {
                        const u32x4 front = low[bytes_in_front(c.next - p, lane16)];
                        if (c.col < g.count) acc = E::mma1(v & front & ~done, n == c.col, acc);
                        done = front;
                        c.pass(g, a.seg_bytes);
                    } while (c.next - p < 1024u);
                    if (c.col < g.count) acc = E::mma1(v & ~done, n == c.col, acc);
                }
            }
        }
        bool bad;
        const Out total = E::fold_out_wide(run_fold(acc, &bad));
        if (E::kCanBeNonFinite && __builtin_amdgcn_ballot_w64(bad) != 0) {
            run_classic<E, U, NT>(a, g, low, lane); // the same run again, segment by segment
        } else if (lane < g.count) {
            ((Out *)a.out)[g.first + lane] = total; // lanes 0 .. 15 hold columns 0 .. 15
        }
    }
}

// The same with the loads rolling: every register is loaded again -- with the vector that the wavefront's next
// iteration needs in it, which may belong to its next run -- as soon as it has been used, so U loads are in flight
// all the time, also while a run's second MMA and store are under way, and one block per compute unit is enough.
// The skeleton is that of the short-segment kernels: a loop whose every pass uses and reloads each register once, in
// the order the loads were issued in, and a last pass without loads.  Every reload is one load instruction whatever
// the position (lanes behind the run's last vector read that vector again), and the results are stored by a masked
// store that is issued in every pass (no lane takes part except at the end of a run), so that the number of memory
// operations between a load and its use is the same on every path and the waits can be exact.  A run with a
// non-finite D' is only noted (one bit for each of the wavefront's first 64 runs, one for all later ones together)
// and summed again by the classic form when the stream has ended, so that no load of the stream sits behind a branch.
// What the two families do with a run's data.  add: the bytes of v (already cleared outside the segment) belong to
// segment `col` of the run; done: segment `col` is complete; result: lane k's return value is the sum of segment k.
template <class E>
struct RunMma {
    typedef typename E::Acc State;
    static constexpr bool kCanMix = E::kCanBeNonFinite;   // a non-finite value reaches the other columns through 0 x inf
    static __device__ __forceinline__ void init(State &st) { st = E::zero(); }
    static __device__ __forceinline__ void add(State &st, u32x4 v, unsigned col, unsigned lane) { st = E::mma1(v, (lane & 15u) == col, st); }
    static __device__ __forceinline__ void done(State &, unsigned, unsigned) {}
    static __device__ __forceinline__ typename E::Out result(State &st, bool *bad)
    {
        const typename E::Out total = E::fold_out_wide(run_fold(st, bad));
        st = E::zero();
        return total;
    }
};
template <class E>
struct RunClassic {
    struct State { typename E::Lane s, res; };            // this lane's share of the open segment; lane k: sum of segment k
    static constexpr bool kCanMix = false;
    static __device__ __forceinline__ void init(State &st) { st.s = 0; st.res = 0; }
    static __device__ __forceinline__ void add(State &st, u32x4 v, unsigned, unsigned) { st.s = st.s + E::lane_sum(v); }
    static __device__ __forceinline__ void done(State &st, unsigned col, unsigned lane)
    {
        const typename E::Lane t = short_butterfly(st.s, 6u);         // the same total in every lane
        st.res = lane == col ? t : st.res;
        st.s = 0;
    }
    static __device__ __forceinline__ typename E::Out result(State &st, bool *bad)
    {
        *bad = false;
        const typename E::Out total = E::lane_out(st.res);
        st.res = 0;
        return total;
    }
};

template <class E, class P, int U, bool NT>
__device__ __forceinline__ void run_stream(const RunArgs &a)
{
    typedef typename E::Out Out;
    const unsigned lane = threadIdx.x & 63u;
    const int lane16 = 16 * (int)lane;
    const unsigned wave = (unsigned)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    __shared__ u32x4 low[17];
    fill_low_masks(low);
    const RunShare sh = run_share(a.layout, a.nseg, a.per_run, gridDim.x, blockIdx.x, wave);
    const u64 nruns = sh.full + (sh.tail_count != 0u ? 1u : 0u);      // this wavefront's runs
    if (nruns == 0) return;

    // where an iteration lies: run k of the wavefront, 64 U vectors from v0 on (scalar registers throughout)
    struct Iter { u64 k; unsigned v0; RunGeometry g; };
    const auto geometry = [&](u64 k) {
        const bool last = k == sh.full;
        return run_geometry(a, last ? sh.tail_first : sh.first + k * sh.stride, last ? sh.tail_count : a.per_run);
    };
    const auto advance = [&](Iter &it) {
        it.v0 += 64u * U;
        if (it.v0 >= it.g.nvec) {
            ++it.k;
            it.v0 = 0u;
            if (it.k < nruns) it.g = geometry(it.k);
        }
    };
    const auto fetch = [&](const Iter &it, int u) -> u32x4 {
        const unsigned idx = it.v0 + 64u * (unsigned)u + lane;
        return load16<NT>(it.g.base + (idx < it.g.nvec ? idx : it.g.nvec - 1u));
    };

    typename P::State st;
    P::init(st);
    RunCursor c;
    u64 redo = 0;                                  // bit k: run k of this wavefront must be summed again
    bool redo_later = false;                       // ... and every run from the 64th on
    // one iteration: its U loads into the run's sums, each register reloaded by `refill` right after its use;
    // at the end of a run the results; the store in every pass
    const auto work = [&](u32x4 *cur, const Iter &it, auto refill) {
        const RunGeometry &g = it.g;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const unsigned p = (it.v0 + 64u * (unsigned)u) * 16u;    // first byte of this load, from base
            const u32x4 v = cur[u];
            if (p < g.total) {                                       // (the same for every lane)
                if (c.next - p >= 1024u) {                           // no boundary in this load: nothing cleared
                    if (c.col < g.count) P::add(st, v, c.col, lane);
                } else {
                    u32x4 done = {0u, 0u, 0u, 0u};                   // bytes already handed to a segment
                    do {
                        const u32x4 front = low[bytes_in_front(c.next - p, lane16)];
                        if (c.col < g.count) {                       // the segment in front of the boundary is complete
                            P::add(st, v & front & ~done, c.col, lane);
                            P::done(st, c.col, lane);
                        }
                        done = front;
                        c.pass(g, a.seg_bytes);
                    } while (c.next - p < 1024u);
                    if (c.col < g.count) P::add(st, v & ~done, c.col, lane);
                }
            }
            refill(u);
        }
        const bool run_ends = it.v0 + 64u * U >= g.nvec;
        Out total = 0;
        unsigned stores = 0u;                                        // lanes that store: none, except at the end of a run
        if (run_ends) {
            // (a run that ends exactly where its last load ends never meets its last boundary inside a load)
            if (c.col < g.count) P::done(st, c.col, lane);
            bool bad;
            total = P::result(st, &bad);
            const bool any = P::kCanMix && __builtin_amdgcn_ballot_w64(bad) != 0;
            if (any) {
                if (it.k < 64) redo |= 1ull << it.k;
                else redo_later = true;
            }
            stores = any ? 0u : g.count;
        }
        if (lane < stores) ((Out *)a.out)[g.first + lane] = total;    // lanes 0 .. 15 hold the sums of segments 0 .. 15
    };

    Iter it;
    it.k = 0;
    it.v0 = 0u;
    it.g = geometry(0);
    c.start(it.g);
    u32x4 cur[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {                  // issued strictly in the order they are used in: the waits count on it
        cur[u] = fetch(it, u);
        __builtin_amdgcn_sched_barrier(0);
    }
    while (true) {
        Iter nx = it;
        advance(nx);
        if (nx.k >= nruns) break;
        __builtin_amdgcn_sched_barrier(0);
        work(cur, it, [&](int u) {
            cur[u] = fetch(nx, u);
            __builtin_amdgcn_sched_barrier(0);     // keep the reload right behind the use
        });
        if (nx.k != it.k) c.start(nx.g);
        it = nx;
    }
    __builtin_amdgcn_sched_barrier(0);
    work(cur, it, [](int) {});
    if (P::kCanMix && (redo != 0 || redo_later)) {
        __builtin_amdgcn_s_waitcnt(0);             // the first pass's stores have landed
        for (u64 k = 0; k < nruns; ++k)
            if (k < 64 ? ((redo >> k) & 1u) != 0 : redo_later) run_classic<E, U, NT>(a, geometry(k), low, lane);
    }
}

template <class E, int U, bool NT>
__global__ void __launch_bounds__(kBlock) sum_segment_runs_mfma_stream_kernel(RunArgs a) { run_stream<E, RunMma<E>, U, NT>(a); }
template <class E, int U, bool NT>
__global__ void __launch_bounds__(kBlock) sum_segment_runs_classic_stream_kernel(RunArgs a) { run_stream<E, RunClassic<E>, U, NT>(a); }

} // namespace redux
