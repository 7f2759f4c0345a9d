// redux_literal.h -- the reduction exactly as Sections IV-A and IV-B state it, level by level.
//
// Every level cuts its input into contiguous groups of m*m numbers, m = 16.  For each group, with
// C a zero matrix every time:
//     first MMA   D  = A x 1 + 0     (A = the group, B = all ones)
//     second MMA  D' = 1 x D + 0
// and the "thread in charge" writes D'[1,1] to the array of partial sums in global memory.  The
// partial sums are the input of the next level (a new kernel launch, since blocks cannot
// synchronise inside a kernel), until one value is left: ceil(log_{m*m} n) levels, the count
// behind T_tc(n) = 5 log_{m*m} n.  A last group that is not full is zero padded.
//
// Mapping to the CDNA4 matrix unit
//   binary16 level (input array):   A is 16 x 16 binary16, one v_mfma_f32_16x16x16_f16; lane l supplies
//                                   A[l%16][4*(l/16) .. +4) = the 8 bytes at group + 8*l.  D is binary32.
//   binary32 levels (partial sums): A is 16 x 16 binary32, four chained v_mfma_f32_16x16x4_f32 (one per
//                                   K-slice of four columns); lane l supplies the 16 bytes at group + 16*l.
//   second MMA, every level:        four chained v_mfma_f32_16x16x4_f32 with A = ones, B = the registers of D.
//   int8 level:                     the narrowest int8 tile is 16 x 32 (v_mfma_i32_16x16x32_i8), so the first
//                                   level's groups hold 512 numbers; D is int32.  Its second MMA and all
//                                   later levels (groups of 256 int64 partial sums) run in binary64
//                                   (v_mfma_f64_16x16x4_f64), which is exact below 2^53.
// Element -> (row, k) placement inside a group follows the lane order above (coalesced); any placement
// gives the same additions because B is all ones.
//
// Binary16 throughout (HALF, m = 16 only): Section I-B says that the multiply-accumulate itself works at half
// precision, and Section IV-B has every group result written back into X, a binary16 array; this is both taken literally.  The result
// of each of the two MMAs is rounded to binary16, the partial sums are stored as binary16 and every level reads
// binary16.  The matrix unit has no binary16 accumulator, so the rounding is applied to what the MFMA returns: a
// lower bound on the damage, since a true binary16 accumulate would also round inside the MMA.  It exists to be
// measured (it overflows to infinity as soon as a partial sum passes 65504), not to be used.
#pragma once
#include "redux_kernels.h"

namespace redux {

typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr unsigned kLitGroup = 256;      // m * m, m = 16
constexpr unsigned kLitGroupI8 = 512;    // first int8 level: 16 x 32

// second MMA on a binary32 D: returns D'[.,.] (the same value in every lane)
__device__ __forceinline__ float lit_mma2_f32(f32x4 d)
{
    f32x4 dp = {0.f, 0.f, 0.f, 0.f};     // C = 0
#pragma unroll
    for (int r = 0; r < 4; ++r) dp = __builtin_amdgcn_mfma_f32_16x16x4f32(1.0f, d[r], dp, 0, 0, 0);
    return dp[0];
}

__device__ __forceinline__ double lit_mma2_f64(f64x4 d)
{
    f64x4 dp = {0., 0., 0., 0.};
#pragma unroll
    for (int r = 0; r < 4; ++r) dp = __builtin_amdgcn_mfma_f64_16x16x4f64(1.0, d[r], dp, 0, 0, 0);
    return dp[0];
}

// ---- group shapes: m = 4, 16, 32 -----------------------------------------------------------------------------
// A "tile" is what one wavefront pushes through one first-MMA / second-MMA sequence:
//   m = 4    sixteen groups of 16 at once (the 4x4x4 MFMA works on 16 independent blocks; block b = lanes 4b..4b+3);
//            the sixteen results sit in lanes 0, 4, 8, ...
//   m = 16   one group of 256; the result sits in every lane
//   m = 32   one group of 1024 (four K-slices of 32x32x8 for binary16, sixteen of 32x32x2 for binary32)
// Both levels of a shape consume the lane's raw words in order: word w of lane l is byte
// (w / kChunkWords) * 64 * kChunkBytes + l * kChunkBytes + (w % kChunkWords) * 4 of the tile, so that every load
// instruction of the wavefront is contiguous.
template <int M> struct LitShape;

template <> struct LitShape<4> {
    static constexpr unsigned kGroup = 16, kTileElems = 256, kResults = 16;
    static __device__ __forceinline__ void mma_f16(const unsigned *raw, float *res)
    {
        const f16x4 ones = {1, 1, 1, 1};
        const f16x4 a = __builtin_bit_cast(f16x4, u32x2{raw[0], raw[1]});
        f32x4 d = __builtin_amdgcn_mfma_f32_4x4x4f16(a, ones, f32x4{0.f, 0.f, 0.f, 0.f}, 0, 0, 0);   // D_b = A_b x 1
        *res = mma2(d);
    }
    static __device__ __forceinline__ void mma_f32(const unsigned *raw, float *res)
    {
        f32x4 d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int k = 0; k < 4; ++k)                            // A_b[i][k] x 1, one K-slice at a time
            d = __builtin_amdgcn_mfma_f32_4x4x1f32(__builtin_bit_cast(float, raw[k]), 1.0f, d, 0, 0, 0);
        *res = mma2(d);
    }
    // lane 4b+j, register i of D holds D_b[i][j]; used as the B operand of a 4x4x1 step it is row i of D_b
    static __device__ __forceinline__ float mma2(f32x4 d)
    {
        f32x4 dp = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int k = 0; k < 4; ++k) dp = __builtin_amdgcn_mfma_f32_4x4x1f32(1.0f, d[k], dp, 0, 0, 0);
        return dp[0];
    }
};

// a binary32 value rounded to binary16 (to nearest even; above 65504 + 16 it becomes an infinity) and widened again
__device__ __forceinline__ float through_binary16(float v) { return (float)(_Float16)v; }

template <> struct LitShape<16> {
    static constexpr unsigned kGroup = 256, kTileElems = 256, kResults = 1;
    static __device__ __forceinline__ void mma_f16(const unsigned *raw, float *res)
    {
        const f16x4 ones = {1, 1, 1, 1};
        const f16x4 a = __builtin_bit_cast(f16x4, u32x2{raw[0], raw[1]});
        f32x4 d = __builtin_amdgcn_mfma_f32_16x16x16f16(a, ones, f32x4{0.f, 0.f, 0.f, 0.f}, 0, 0, 0);
        *res = lit_mma2_f32(d);
    }
    // the same with D and D' held in binary16
    static __device__ __forceinline__ void mma_f16_half(const unsigned *raw, float *res)
    {
        const f16x4 ones = {1, 1, 1, 1};
        const f16x4 a = __builtin_bit_cast(f16x4, u32x2{raw[0], raw[1]});
        f32x4 d = __builtin_amdgcn_mfma_f32_16x16x16f16(a, ones, f32x4{0.f, 0.f, 0.f, 0.f}, 0, 0, 0);
#pragma unroll
        for (int r = 0; r < 4; ++r) d[r] = through_binary16(d[r]);
        *res = through_binary16(lit_mma2_f32(d));
    }
    static __device__ __forceinline__ void mma_f32(const unsigned *raw, float *res)
    {
        f32x4 d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int k = 0; k < 4; ++k)
            d = __builtin_amdgcn_mfma_f32_16x16x4f32(__builtin_bit_cast(float, raw[k]), 1.0f, d, 0, 0, 0);
        *res = lit_mma2_f32(d);
    }
};

template <> struct LitShape<32> {
    static constexpr unsigned kGroup = 1024, kTileElems = 1024, kResults = 1;
    typedef float f32x16 __attribute__((ext_vector_type(16)));
    static __device__ __forceinline__ f32x16 zero16()
    {
        f32x16 z;
#pragma unroll
        for (int r = 0; r < 16; ++r) z[r] = 0.f;
        return z;
    }
    // lane l, register r of a 32x32 accumulator holds D[8*(r/4) + 4*(l/32) + r%4][l%32]; as the B operand of
    // a 32x32x2 step (B[l/32][l%32]) register r contributes two rows, and sixteen chained steps cover all 32.
    static __device__ __forceinline__ float mma2(f32x16 d)
    {
        f32x16 dp = zero16();
#pragma unroll
        for (int r = 0; r < 16; ++r) dp = __builtin_amdgcn_mfma_f32_32x32x2f32(1.0f, d[r], dp, 0, 0, 0);
        return dp[0];
    }
    static __device__ __forceinline__ void mma_f16(const unsigned *raw, float *res)
    {
        const f16x4 ones = {1, 1, 1, 1};
        f32x16 d = zero16();
#pragma unroll
        for (int t = 0; t < 4; ++t)                            // K = 32 as four slices of 8
            d = __builtin_amdgcn_mfma_f32_32x32x8f16(__builtin_bit_cast(f16x4, u32x2{raw[2 * t], raw[2 * t + 1]}), ones, d, 0, 0, 0);
        *res = mma2(d);
    }
    static __device__ __forceinline__ void mma_f32(const unsigned *raw, float *res)
    {
        f32x16 d = zero16();
#pragma unroll
        for (int k = 0; k < 16; ++k)                           // K = 32 as sixteen slices of 2
            d = __builtin_amdgcn_mfma_f32_32x32x2f32(__builtin_bit_cast(float, raw[k]), 1.0f, d, 0, 0, 0);
        *res = mma2(d);
    }
};

// ---- one level: binary16 input (F16IN) or binary32 partial sums -------------------------------------------------
// One wavefront reduces U tiles per iteration.  FAST: the input is aligned to the load width, so a lane's
// words come from 8- or 16-byte loads; otherwise (and for the ragged last tile) element loads with zero padding.
// HALF (m = 16, binary16 input): both MMA results rounded to binary16, partial sums stored as binary16.
template <int M, bool F16IN, int U, bool FAST, bool HALF = false>
__global__ void __launch_bounds__(kBlock) literal_level_kernel(const void *xin, u64 n, void *pout, int out_is_binary32)
{
    static_assert(!HALF || (M == 16 && F16IN), "the binary16 form exists for m = 16 only and reads binary16 at every level");
    // where group results go: the array of partial sums (binary32, or binary16 in the HALF form), or -- the last
    // level -- the caller's binary32 result
    auto put = [&](u64 g, float v) {
        if (!HALF || out_is_binary32) ((float *)pout)[g] = v;
        else ((_Float16 *)pout)[g] = (_Float16)v;       // (already a binary16 value: exact)
    };
    typedef LitShape<M> S;
    constexpr unsigned kElemBytes = F16IN ? 2 : 4;
    constexpr unsigned kWords = S::kTileElems * kElemBytes / 4 / 64;      // raw 32-bit words per lane per tile
    constexpr unsigned kChunkWords = kWords >= 4 ? 4 : kWords;            // words per load instruction (2 or 4)
    constexpr unsigned kChunkBytes = kChunkWords * 4;
    constexpr unsigned kChunks = kWords / kChunkWords;
    const unsigned lane = threadIdx.x & 63u;
    const u64 wave_global = (u64)blockIdx.x * kWaves + (threadIdx.x >> 6);
    const u64 nwaves = (u64)gridDim.x * kWaves;
    const u64 ngroups = (n + S::kGroup - 1) / S::kGroup;
    const u64 ntiles = (n + S::kTileElems - 1) / S::kTileElems;
    const u64 nfull = n / S::kTileElems;
    const u64 nbatch = (ntiles + U - 1) / U;
    const unsigned char *x = (const unsigned char *)xin;

    for (u64 b = wave_global; b < nbatch; b += nwaves) {
        const u64 t0 = b * U;
        unsigned raw[U][kWords];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const u64 t = t0 + u;
            const unsigned char *tile = x + t * S::kTileElems * kElemBytes;
            if (FAST && t < nfull) {
#pragma unroll
                for (unsigned c = 0; c < kChunks; ++c) {
                    const unsigned char *p = tile + (u64)c * 64 * kChunkBytes + lane * kChunkBytes;
                    if (kChunkWords == 4) {
                        u32x4 v = F16IN ? __builtin_nontemporal_load((const u32x4 *)p) : *(const u32x4 *)p;
#pragma unroll
                        for (int w = 0; w < 4; ++w) raw[u][4 * c + w] = v[w];
                    } else {
                        u32x2 v = F16IN ? __builtin_nontemporal_load((const u32x2 *)p) : *(const u32x2 *)p;
                        raw[u][2 * c] = v[0];
                        raw[u][2 * c + 1] = v[1];
                    }
                }
            } else {
#pragma unroll
                for (unsigned w = 0; w < kWords; ++w) {
                    unsigned word = 0;
                    if (t < ntiles) {
                        const u64 byte0 = (u64)(w / kChunkWords) * 64 * kChunkBytes + lane * kChunkBytes + (w % kChunkWords) * 4;
                        const u64 e0 = t * S::kTileElems + byte0 / kElemBytes;       // first element of this word
                        if (F16IN) {
                            const unsigned short *h = (const unsigned short *)xin;
                            const unsigned lo = e0 < n ? h[e0] : 0u, hi = e0 + 1 < n ? h[e0 + 1] : 0u;
                            word = lo | (hi << 16);
                        } else {
                            word = e0 < n ? ((const unsigned *)xin)[e0] : 0u;
                        }
                    }
                    raw[u][w] = word;
                }
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        float mine = 0.f;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float res;
            if constexpr (HALF) S::mma_f16_half(raw[u], &res);
            else if (F16IN) S::mma_f16(raw[u], &res);
            else S::mma_f32(raw[u], &res);
            if (S::kResults == 1) {
                if (lane == (unsigned)u) mine = res;           // lane u is in charge of tile t0 + u
            } else {                                           // m = 4: lane 4b is in charge of block b of the tile
                const u64 g = (t0 + u) * S::kResults + (lane >> 2);
                if ((lane & 3u) == 0 && g < ngroups) put(g, res);
            }
        }
        if (S::kResults == 1 && lane < (unsigned)U && t0 + lane < ngroups) put(t0 + lane, mine);
    }
}

// ---- level over the int8 input: groups of 512 (16 x 32) ---------------------------------------------------------
template <int U, bool FAST>
__global__ void __launch_bounds__(kBlock) literal_level_i8_kernel(const signed char *x, u64 n, i64 *partial)
{
    const unsigned lane = threadIdx.x & 63u;
    const u64 wave_global = (u64)blockIdx.x * kWaves + (threadIdx.x >> 6);
    const u64 nwaves = (u64)gridDim.x * kWaves;
    const u64 ngroups = (n + kLitGroupI8 - 1) / kLitGroupI8;
    const u64 nfull = n / kLitGroupI8;
    const u64 nbatch = (ngroups + U - 1) / U;
    const long ones = 0x0101010101010101L;

    for (u64 b = wave_global; b < nbatch; b += nwaves) {
        const u64 g0 = b * U;
        u64 raw[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const u64 g = g0 + u;
            u64 v = 0;
            if (FAST && g < nfull) {
                u32x2 w = __builtin_nontemporal_load((const u32x2 *)(x + g * kLitGroupI8) + lane);
                v = (u64)w[0] | ((u64)w[1] << 32);
            } else if (g < ngroups) {
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const u64 idx = g * kLitGroupI8 + 8 * lane + k;
                    const u64 byte = idx < n ? (u64)(unsigned char)x[idx] : 0;
                    v |= byte << (8 * k);
                }
            }
            raw[u] = v;
        }
        __builtin_amdgcn_sched_barrier(0);
        i64 mine = 0;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const i32x4 zero = {0, 0, 0, 0};
            i32x4 d = __builtin_amdgcn_mfma_i32_16x16x32_i8((long)raw[u], ones, zero, 0, 0, 0);
            const f64x4 dd = {(double)d[0], (double)d[1], (double)d[2], (double)d[3]};
            const i64 group_sum = (i64)lit_mma2_f64(dd);
            if (lane == (unsigned)u) mine = group_sum;
        }
        if (lane < (unsigned)U && g0 + lane < ngroups) partial[g0 + lane] = mine;
    }
}

// ---- level over int64 partial sums, in binary64 -------------------------------------------------------------------
template <int U>
__global__ void __launch_bounds__(kBlock) literal_level_i64_kernel(const i64 *x, u64 n, i64 *partial)
{
    const unsigned lane = threadIdx.x & 63u;
    const u64 wave_global = (u64)blockIdx.x * kWaves + (threadIdx.x >> 6);
    const u64 nwaves = (u64)gridDim.x * kWaves;
    const u64 ngroups = (n + kLitGroup - 1) / kLitGroup;
    const u64 nbatch = (ngroups + U - 1) / U;

    for (u64 b = wave_global; b < nbatch; b += nwaves) {
        const u64 g0 = b * U;
        f64x4 raw[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const u64 g = g0 + u;
            f64x4 v = {0., 0., 0., 0.};
            if (g < ngroups) {
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const u64 idx = g * kLitGroup + 4 * lane + k;
                    v[k] = idx < n ? (double)x[idx] : 0.0;       // |partial sum| < 2^53: exact
                }
            }
            raw[u] = v;
        }
        __builtin_amdgcn_sched_barrier(0);
        i64 mine = 0;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            f64x4 d = {0., 0., 0., 0.};
#pragma unroll
            for (int k = 0; k < 4; ++k) d = __builtin_amdgcn_mfma_f64_16x16x4f64(raw[u][k], 1.0, d, 0, 0, 0);
            const i64 group_sum = (i64)lit_mma2_f64(d);
            if (lane == (unsigned)u) mine = group_sum;
        }
        if (lane < (unsigned)U && g0 + lane < ngroups) partial[g0 + lane] = mine;
    }
}

} // namespace redux
