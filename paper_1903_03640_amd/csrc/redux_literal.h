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

// ---- level over the binary16 input -------------------------------------------------------------------------
// One wavefront reduces U groups per iteration and writes U consecutive partial sums.
// FAST: x is 8-byte aligned, so a lane's four elements are one 8-byte load; otherwise element loads.
template <int U, bool FAST>
__global__ void __launch_bounds__(kBlock) literal_level_f16_kernel(const unsigned short *x, u64 n, float *partial)
{
    const unsigned lane = threadIdx.x & 63u;
    const u64 wave_global = (u64)blockIdx.x * kWaves + (threadIdx.x >> 6);
    const u64 nwaves = (u64)gridDim.x * kWaves;
    const u64 ngroups = (n + kLitGroup - 1) / kLitGroup;
    const u64 nfull = n / kLitGroup;
    const u64 nbatch = (ngroups + U - 1) / U;
    const f16x4 ones = {1, 1, 1, 1};

    for (u64 b = wave_global; b < nbatch; b += nwaves) {
        const u64 g0 = b * U;
        u32x2 raw[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const u64 g = g0 + u;
            u32x2 v = {0u, 0u};
            if (FAST && g < nfull) {
                v = __builtin_nontemporal_load((const u32x2 *)(x + g * kLitGroup) + lane);
            } else if (g < ngroups) {                      // ragged last group or unaligned input: zero padded
                unsigned short e[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const u64 idx = g * kLitGroup + 4 * lane + k;
                    e[k] = idx < n ? x[idx] : (unsigned short)0;
                }
                v = u32x2{(unsigned)e[0] | ((unsigned)e[1] << 16), (unsigned)e[2] | ((unsigned)e[3] << 16)};
            }
            raw[u] = v;
        }
        __builtin_amdgcn_sched_barrier(0);
        float mine = 0.f;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const f32x4 zero = {0.f, 0.f, 0.f, 0.f};       // C = 0 for every group
            f32x4 d = __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(f16x4, raw[u]), ones, zero, 0, 0, 0);
            const float group_sum = lit_mma2_f32(d);
            if (lane == (unsigned)u) mine = group_sum;     // lane u is in charge of group g0 + u
        }
        if (lane < (unsigned)U && g0 + lane < ngroups) partial[g0 + lane] = mine;
    }
}

// ---- level over binary32 partial sums (16-byte aligned, library-owned) ----------------------------------------
template <int U>
__global__ void __launch_bounds__(kBlock) literal_level_f32_kernel(const float *x, u64 n, float *partial)
{
    const unsigned lane = threadIdx.x & 63u;
    const u64 wave_global = (u64)blockIdx.x * kWaves + (threadIdx.x >> 6);
    const u64 nwaves = (u64)gridDim.x * kWaves;
    const u64 ngroups = (n + kLitGroup - 1) / kLitGroup;
    const u64 nfull = n / kLitGroup;
    const u64 nbatch = (ngroups + U - 1) / U;

    for (u64 b = wave_global; b < nbatch; b += nwaves) {
        const u64 g0 = b * U;
        f32x4 raw[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const u64 g = g0 + u;
            f32x4 v = {0.f, 0.f, 0.f, 0.f};
            if (g < nfull) {
                v = *((const f32x4 *)(x + g * kLitGroup) + lane);
            } else if (g < ngroups) {
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const u64 idx = g * kLitGroup + 4 * lane + k;
                    v[k] = idx < n ? x[idx] : 0.f;
                }
            }
            raw[u] = v;
        }
        __builtin_amdgcn_sched_barrier(0);
        float mine = 0.f;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            f32x4 d = {0.f, 0.f, 0.f, 0.f};                // C = 0; the 16 x 16 x 16 product as four K-slices
#pragma unroll
            for (int k = 0; k < 4; ++k) d = __builtin_amdgcn_mfma_f32_16x16x4f32(raw[u][k], 1.0f, d, 0, 0, 0);
            const float group_sum = lit_mma2_f32(d);
            if (lane == (unsigned)u) mine = group_sum;
        }
        if (lane < (unsigned)U && g0 + lane < ngroups) partial[g0 + lane] = mine;
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
