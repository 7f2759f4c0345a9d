// redux_kernels.h -- gfx950 (CDNA4) device code of libredux.
//
// The reduction of Section IV-A of the paper, re-mapped to the CDNA4 matrix unit:
//
//   * a wavefront's coalesced 16-byte-per-lane load (1 KiB) IS the A operand of one
//     MFMA: 16 rows x 32 binary16 (v_mfma_f32_16x16x32_f16) or 16 rows x 64 int8
//     (v_mfma_i32_16x16x64_i8).  B is the all-ones constant.  This is the paper's
//     first MMA, D = A x 1 + C, except that C is not zero but the running D of the
//     previous tile ("chain"), so no per-group partial ever leaves the registers.
//     Which element lands in which (row, k) slot does not matter: B is all ones, so
//     every bijection gives the same set of additions.
//   * the paper's second MMA, D' = 1 x D, folds the 16 row sums: the accumulator
//     registers of D are fed back as the B operand of v_mfma_f32_16x16x4_f32 (binary64:
//     v_mfma_f64_16x16x4_f64) with an all-ones A.  Lane l, register r of a 16x16
//     accumulator holds D[4*(l/16)+r][l%16]; lane l of a 4x16 B operand holds
//     B[l/16][l%16]; so register r used as B contributes rows r, 4+r, 8+r, 12+r and four
//     chained MFMAs (r = 0..3) sum all 16 rows with no data movement between lanes.
//   * the next level of the paper's hierarchy (partials of all groups -> one value) is one
//     binary64 two-MMA group reduction over the per-block partials, run by the block that
//     arrives last (single pass over HBM instead of one kernel per level).
//
// The "classic" family is the tree reduction of Section III with Brent's coarsening: each lane
// accumulates serially, then a DPP / ds_swizzle butterfly combines the 64 lanes.
#pragma once
#include <type_traits>
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace redux {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef double f64x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef unsigned long long u64;
typedef long long i64;

constexpr int kBlock = 256;          // threads per block: 4 wavefronts of 64
constexpr int kWaves = kBlock / 64;
constexpr int kMaxGrid = 16384;      // capacity of the partials array

// ---------------------------------------------------------------------------------------------
// loads
// ---------------------------------------------------------------------------------------------
template <bool NT>
__device__ __forceinline__ u32x4 load16(const u32x4 *p)
{
    if (NT) return __builtin_nontemporal_load(p);
    return *p;
}

// ---------------------------------------------------------------------------------------------
// cross-lane helpers for the classic family (wave64)
// ---------------------------------------------------------------------------------------------
template <int CTRL>
__device__ __forceinline__ int dpp_i32(int v)
{
    return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, false);
}

constexpr int kQuadXor1 = 0xB1;       // quad_perm [1,0,3,2]
constexpr int kQuadXor2 = 0x4E;       // quad_perm [2,3,0,1]
constexpr int kRowHalfMirror = 0x141; // lane i <-> 7-i within each 8
constexpr int kRowMirror = 0x140;     // lane i <-> 15-i within each 16
constexpr int kSwizzleXor16 = 0x401F; // ds_swizzle bit mode: and 0x1f, or 0, xor 0x10

__device__ __forceinline__ float wave_sum_f32(float v)
{
    // butterfly inside each row of 16 lanes (DPP), then across rows (ds_swizzle, readlane).
    // Every step adds a lane's value and its partner's, so all lanes of a group hold the
    // same value afterwards and the result does not depend on which lane reads it.
    v += __builtin_bit_cast(float, dpp_i32<kQuadXor1>(__builtin_bit_cast(int, v)));
    v += __builtin_bit_cast(float, dpp_i32<kQuadXor2>(__builtin_bit_cast(int, v)));
    v += __builtin_bit_cast(float, dpp_i32<kRowHalfMirror>(__builtin_bit_cast(int, v)));
    v += __builtin_bit_cast(float, dpp_i32<kRowMirror>(__builtin_bit_cast(int, v)));
    v += __builtin_bit_cast(float, __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, v), kSwizzleXor16));
    float lo = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 0));
    float hi = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 32));
    return lo + hi;
}

template <int CTRL>
__device__ __forceinline__ i64 dpp_i64(i64 v)
{
    int lo = dpp_i32<CTRL>((int)(u64)v);
    int hi = dpp_i32<CTRL>((int)((u64)v >> 32));
    return (i64)(((u64)(unsigned)hi << 32) | (unsigned)lo);
}

__device__ __forceinline__ i64 wave_sum_i64(i64 v)
{
    v += dpp_i64<kQuadXor1>(v);
    v += dpp_i64<kQuadXor2>(v);
    v += dpp_i64<kRowHalfMirror>(v);
    v += dpp_i64<kRowMirror>(v);
    {
        int lo = __builtin_amdgcn_ds_swizzle((int)(u64)v, kSwizzleXor16);
        int hi = __builtin_amdgcn_ds_swizzle((int)((u64)v >> 32), kSwizzleXor16);
        v += (i64)(((u64)(unsigned)hi << 32) | (unsigned)lo);
    }
    i64 a = (i64)(((u64)(unsigned)__builtin_amdgcn_readlane((int)((u64)v >> 32), 0) << 32) |
                  (unsigned)__builtin_amdgcn_readlane((int)(u64)v, 0));
    i64 b = (i64)(((u64)(unsigned)__builtin_amdgcn_readlane((int)((u64)v >> 32), 32) << 32) |
                  (unsigned)__builtin_amdgcn_readlane((int)(u64)v, 32));
    return a + b;
}

__device__ __forceinline__ float uniform_f32(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, v)));
}

__device__ __forceinline__ double uniform_f64(double v)
{
    u64 b = __builtin_bit_cast(u64, v);
    unsigned lo = (unsigned)__builtin_amdgcn_readfirstlane((int)b);
    unsigned hi = (unsigned)__builtin_amdgcn_readfirstlane((int)(b >> 32));
    return __builtin_bit_cast(double, ((u64)hi << 32) | lo);
}

// ---------------------------------------------------------------------------------------------
// Kernel families.  Each one defines
//   Acc            per-lane accumulator state of the hot loop
//   Total          wide type that wave, block and grid totals are carried in
//   Out            type written to the caller's buffer
//   consume        take one 16-byte vector per lane (one 1-KiB tile per wavefront); u picks the accumulator
//   fold           reduce Acc to one wave-uniform Total and clear Acc
//   edge           build a vector holding a single element in slot 0 (zero padding elsewhere)
// ---------------------------------------------------------------------------------------------

// Floating-point element kinds.  Every kind accumulates in binary32 and differs only in how a
// 16-byte vector is handed to the matrix unit (or converted, in the classic family).
enum Kind { kF16 = 0, kBF16 = 1, kF32 = 2, kE4M3 = 3, kE5M2 = 4 };

template <int KIND> struct KindTraits;
template <> struct KindTraits<kF16>  { static constexpr int kElemSize = 2; };
template <> struct KindTraits<kBF16> { static constexpr int kElemSize = 2; };
template <> struct KindTraits<kF32>  { static constexpr int kElemSize = 4; };
template <> struct KindTraits<kE4M3> { static constexpr int kElemSize = 1; };
template <> struct KindTraits<kE5M2> { static constexpr int kElemSize = 1; };

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

// one element, zero padded to a vector (slot 0)
template <int ES>
__device__ __forceinline__ u32x4 edge_bits(const void *p)
{
    if (ES == 4) return u32x4{*(const unsigned *)p, 0u, 0u, 0u};
    if (ES == 2) return u32x4{(unsigned)*(const unsigned short *)p, 0u, 0u, 0u};
    return u32x4{(unsigned)*(const unsigned char *)p, 0u, 0u, 0u};
}

// first MMA of Section IV-A with the accumulator chained through C:  D <- A x 1 + D
template <int KIND>
__device__ __forceinline__ f32x4 mma1_chain(u32x4 v, f32x4 d)
{
    if (KIND == kF16) {
        const f16x8 ones = {1, 1, 1, 1, 1, 1, 1, 1};
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, v), ones, d, 0, 0, 0);
    } else if (KIND == kBF16) {
        const u32x4 ones = {0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};     // bfloat16 1.0 = 0x3F80
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, v), __builtin_bit_cast(bf16x8, ones), d, 0, 0, 0);
    } else if (KIND == kF32) {
        // A is 16 x 4 binary32 per MFMA: the lane's four values are four K-slices
        const f32x4 f = __builtin_bit_cast(f32x4, v);
#pragma unroll
        for (int k = 0; k < 4; ++k) d = __builtin_amdgcn_mfma_f32_16x16x4f32(f[k], 1.0f, d, 0, 0, 0);
        return d;
    } else {
        // 8-bit floating point: A is 16 x 32 per MFMA (8 bytes per lane), so a 16-byte vector is two MFMAs
        const long lo = (long)(((u64)v[1] << 32) | v[0]), hi = (long)(((u64)v[3] << 32) | v[2]);
        if (KIND == kE4M3) {
            const long ones = 0x3838383838383838L;                                    // E4M3 1.0 = 0x38
            d = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(lo, ones, d, 0, 0, 0);
            return __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(hi, ones, d, 0, 0, 0);
        } else {
            const long ones = 0x3C3C3C3C3C3C3C3CL;                                    // E5M2 1.0 = 0x3C
            d = __builtin_amdgcn_mfma_f32_16x16x32_bf8_bf8(lo, ones, d, 0, 0, 0);
            return __builtin_amdgcn_mfma_f32_16x16x32_bf8_bf8(hi, ones, d, 0, 0, 0);
        }
    }
}

// sum of the elements of one 16-byte vector, binary32 (classic family)
template <int KIND>
__device__ __forceinline__ void add_vector(float *s /* 4 running sums */, u32x4 v)
{
    if (KIND == kF16) {
        f16x8 h = __builtin_bit_cast(f16x8, v);
#pragma unroll
        for (int k = 0; k < 8; ++k) s[k & 3] += (float)h[k];
    } else if (KIND == kBF16) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {                         // a bfloat16 is the upper half of a binary32
            const unsigned w = v[k];
            s[k] += __builtin_bit_cast(float, w << 16);
            s[k] += __builtin_bit_cast(float, w & 0xFFFF0000u);
        }
    } else if (KIND == kF32) {
        const f32x4 f = __builtin_bit_cast(f32x4, v);
#pragma unroll
        for (int k = 0; k < 4; ++k) s[k] += f[k];
    } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            f32x2 a, b;
            if (KIND == kE4M3) { a = __builtin_amdgcn_cvt_pk_f32_fp8((int)v[k], false); b = __builtin_amdgcn_cvt_pk_f32_fp8((int)v[k], true); }
            else               { a = __builtin_amdgcn_cvt_pk_f32_bf8((int)v[k], false); b = __builtin_amdgcn_cvt_pk_f32_bf8((int)v[k], true); }
            s[k] += a[0] + a[1];
            s[k] += b[0] + b[1];
        }
    }
}

template <int KIND, int NACC>
struct FloatMfmaT {
    typedef double Total;
    typedef float Out;
    static constexpr int kElemSize = KindTraits<KIND>::kElemSize;
    static constexpr int kNumAcc = NACC;   // independent accumulator chains per wavefront
    static constexpr bool kMfmaFinish = true;
    struct Acc { f32x4 d[kNumAcc]; };

    static __device__ __forceinline__ void clear(Acc &c)
    {
#pragma unroll
        for (int i = 0; i < kNumAcc; ++i) c.d[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    static __device__ __forceinline__ void consume(Acc &c, int U, u32x4 v)
    {
        c.d[U % kNumAcc] = mma1_chain<KIND>(v, c.d[U % kNumAcc]);
    }
    // second MMA: D' <- 1 x D, chained over the four register slices of D.  The independent chains hold D_1 .. D_k with
    // D = D_1 + ... + D_k; the MMA is linear, so they are added entry by entry first and folded once (four dependent
    // MFMAs instead of 4 k at the end of every wavefront).
    static __device__ __forceinline__ Total fold(Acc &c)
    {
        f32x4 d = c.d[0];
#pragma unroll
        for (int i = 1; i < kNumAcc; ++i) d += c.d[i];
        f32x4 dp = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int r = 0; r < 4; ++r) dp = __builtin_amdgcn_mfma_f32_16x16x4f32(1.0f, d[r], dp, 0, 0, 0);
        clear(c);
        return (double)uniform_f32(dp[0]);
    }
    static __device__ __forceinline__ u32x4 edge(const void *p) { return edge_bits<kElemSize>(p); }
    static __device__ __forceinline__ Out to_out(Total t) { return (float)t; }
};

template <int NACC> using F16MfmaT = FloatMfmaT<kF16, NACC>;
typedef F16MfmaT<4> F16Mfma;      // flat sum: four chains, folded once per wavefront
typedef F16MfmaT<1> F16MfmaSeg;   // segmented sum: one chain, so the per-segment fold is four MFMAs

// Compensated chain (binary16 only; for the precision study, not a default).  The matrix unit does not expose the
// rounding error of its own accumulate, so the chain cannot be compensated inside the MMA.  What can be done: the first
// MMA runs with C = 0 as the paper writes it, D = A x 1 gives the tile's sixteen row sums, and those are added to
// the running sums on the vector ALU with Knuth's two-sum, whose second output is exactly what the addition lost;
// the lost parts are collected in a second accumulator and both are folded by the second MMA.
struct F16MfmaCompensated {
    typedef double Total;
    typedef float Out;
    static constexpr int kElemSize = 2;
    static constexpr bool kMfmaFinish = true;
    struct Acc { f32x4 sum, lost; };

    static __device__ __forceinline__ void clear(Acc &c)
    {
        c.sum = f32x4{0.f, 0.f, 0.f, 0.f};
        c.lost = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    static __device__ __forceinline__ void consume(Acc &c, int U, u32x4 v)
    {
        const f32x4 r = mma1_chain<kF16>(v, f32x4{0.f, 0.f, 0.f, 0.f});      // D = A x 1 + 0
        const f32x4 t = c.sum + r;
        const f32x4 bb = t - c.sum;
        c.lost += (c.sum - (t - bb)) + (r - bb);                             // two-sum: t + this term == sum + r exactly
        c.sum = t;
    }
    static __device__ __forceinline__ Total fold(Acc &c)
    {
        f32x4 dp = {0.f, 0.f, 0.f, 0.f}, dl = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            dp = __builtin_amdgcn_mfma_f32_16x16x4f32(1.0f, c.sum[r], dp, 0, 0, 0);
            dl = __builtin_amdgcn_mfma_f32_16x16x4f32(1.0f, c.lost[r], dl, 0, 0, 0);
        }
        clear(c);
        return (double)uniform_f32(dp[0]) + (double)uniform_f32(dl[0]);
    }
    static __device__ __forceinline__ u32x4 edge(const void *p) { return edge_bits<kElemSize>(p); }
    static __device__ __forceinline__ Out to_out(Total t) { return (float)t; }
};

template <int KIND>
struct FloatClassic {
    typedef double Total;
    typedef float Out;
    static constexpr int kElemSize = KindTraits<KIND>::kElemSize;
    static constexpr bool kMfmaFinish = false;
    struct Acc { float s[4]; };

    static __device__ __forceinline__ void clear(Acc &c) { c.s[0] = c.s[1] = c.s[2] = c.s[3] = 0.f; }
    static __device__ __forceinline__ void consume(Acc &c, int U, u32x4 v) { add_vector<KIND>(c.s, v); }
    static __device__ __forceinline__ Total fold(Acc &c)
    {
        float s = (c.s[0] + c.s[1]) + (c.s[2] + c.s[3]);
        clear(c);
        return (double)wave_sum_f32(s);
    }
    static __device__ __forceinline__ u32x4 edge(const void *p) { return edge_bits<kElemSize>(p); }
    static __device__ __forceinline__ Out to_out(Total t) { return (float)t; }
};
typedef FloatClassic<kF16> F16Classic;

template <int NACC>
struct I8MfmaT {
    typedef i64 Total;
    typedef i64 Out;
    static constexpr int kElemSize = 1;
    static constexpr int kNumAcc = NACC;
    static constexpr bool kMfmaFinish = false;
    struct Acc { i32x4 d[kNumAcc]; };

    static __device__ __forceinline__ void clear(Acc &c)
    {
#pragma unroll
        for (int i = 0; i < kNumAcc; ++i) c.d[i] = i32x4{0, 0, 0, 0};
    }
    static __device__ __forceinline__ void consume(Acc &c, int U, u32x4 v)
    {
        const i32x4 ones = {0x01010101, 0x01010101, 0x01010101, 0x01010101};
        c.d[U % kNumAcc] = __builtin_amdgcn_mfma_i32_16x16x64_i8(__builtin_bit_cast(i32x4, v), ones,
                                                                 c.d[U % kNumAcc], 0, 0, 0);
    }
    // There is no MFMA with int32 inputs.  Every accumulator entry is an int32 and a column of
    // sixteen of them sums to less than 2^35, so the second MMA runs exactly in binary64.
    static __device__ __forceinline__ Total fold(Acc &c)
    {
        f64x4 dp = {0., 0., 0., 0.};
#pragma unroll
        for (int i = 0; i < kNumAcc; ++i)
#pragma unroll
            for (int r = 0; r < 4; ++r)
                dp = __builtin_amdgcn_mfma_f64_16x16x4f64(1.0, (double)c.d[i][r], dp, 0, 0, 0);
        clear(c);
        return (i64)uniform_f64(dp[0]);
    }
    static __device__ __forceinline__ u32x4 edge(const void *p)
    {
        return u32x4{(unsigned)*(const unsigned char *)p, 0u, 0u, 0u};
    }
    static __device__ __forceinline__ Out to_out(Total t) { return t; }
};

typedef I8MfmaT<4> I8Mfma;
typedef I8MfmaT<1> I8MfmaSeg;

struct I8Classic {
    typedef i64 Total;
    typedef i64 Out;
    static constexpr int kElemSize = 1;
    static constexpr bool kMfmaFinish = false;
    struct Acc { int s[4]; };

    static __device__ __forceinline__ void clear(Acc &c) { c.s[0] = c.s[1] = c.s[2] = c.s[3] = 0; }
    static __device__ __forceinline__ void consume(Acc &c, int U, u32x4 v)
    {
#pragma unroll
        for (int k = 0; k < 4; ++k) c.s[k] = __builtin_amdgcn_sdot4((int)v[k], 0x01010101, c.s[k], false);
    }
    static __device__ __forceinline__ Total fold(Acc &c)
    {
        i64 s = ((i64)c.s[0] + (i64)c.s[1]) + ((i64)c.s[2] + (i64)c.s[3]);
        clear(c);
        return wave_sum_i64(s);
    }
    static __device__ __forceinline__ u32x4 edge(const void *p)
    {
        return u32x4{(unsigned)*(const unsigned char *)p, 0u, 0u, 0u};
    }
    static __device__ __forceinline__ Out to_out(Total t) { return t; }
};

// ---------------------------------------------------------------------------------------------
// geometry of one contiguous run of elements: unaligned head, 16-byte vectors, tail
// ---------------------------------------------------------------------------------------------
struct Run {
    const unsigned char *head; // first element
    const u32x4 *body;         // first 16-byte aligned vector
    const unsigned char *tail; // first element after the last whole vector
    u64 nvec;
    int nhead, ntail;          // element counts, each < 16 / elemsize
};

template <int ES>
__host__ __device__ __forceinline__ Run make_run(const void *x, u64 n)
{
    constexpr u64 kPerVec = 16 / ES;
    Run r;
    r.head = (const unsigned char *)x;
    u64 mis = (u64)(uintptr_t)x & 15u;
    u64 nh = mis ? (16 - mis) / ES : 0;
    if (nh > n) nh = n;
    r.nhead = (int)nh;
    r.body = (const u32x4 *)(r.head + nh * ES);
    r.nvec = (n - nh) / kPerVec;
    r.ntail = (int)(n - nh - r.nvec * kPerVec);
    r.tail = r.head + (nh + r.nvec * kPerVec) * ES;
    return r;
}

// head and tail elements, one per lane, each in slot 0 of an otherwise zero vector: a zero-padded tile
template <class F>
__device__ __forceinline__ u32x4 edge_vector(const Run &r, int lane)
{
    constexpr int kPerVec = 16 / F::kElemSize;
    u32x4 v = {0u, 0u, 0u, 0u};
    if (lane < r.nhead) v = F::edge(r.head + lane * F::kElemSize);
    else if (lane >= kPerVec && lane - kPerVec < r.ntail) v = F::edge(r.tail + (lane - kPerVec) * F::kElemSize);
    return v;
}

// ---------------------------------------------------------------------------------------------
// publishing block partials and electing the block that finishes
// ---------------------------------------------------------------------------------------------
template <class T>
__device__ __forceinline__ void store_partial(u64 *slot, T v)
{
    __hip_atomic_store(slot, __builtin_bit_cast(u64, v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <class T>
__device__ __forceinline__ T load_partial(const u64 *slot)
{
    return __builtin_bit_cast(T, __hip_atomic_load(slot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
}

// A slot that no block has written to since it was last read holds this pattern: a NaN that no sum can produce (a
// binary64 total comes from binary32 values, whose low 29 bits are zero, or is the default NaN), and which
// publish_to_slot replaces all the same.
constexpr u64 kEmptySlot = ~(u64)0;
constexpr unsigned kSlotSpins = 1u << 22;   // re-reads before a slot is given up (never reached: see fetch_partials)

template <class T>
__device__ __forceinline__ void publish_to_slot(u64 *slot, T v)
{
    u64 bits = __builtin_bit_cast(u64, v);
    if (bits == kEmptySlot) bits = 0x7ff8000000000000ull;
    (void)__hip_atomic_exchange(slot, bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // no value comes back: nothing waits
}
// The values that blocks have published to slots base + r x 256 + thread (r = 0 .. R-1; zeros past `count`), fetched in
// one go.  kSlots: the slots are then marked empty again for the next launch.  The caller holds the last ticket, so
// every exchange that fills a slot has been issued, ahead of its block's ticket, and completes without anybody's help;
// until it has, the slot still reads empty and is read again.
template <class T, bool kSlots, unsigned R>
__device__ __forceinline__ void fetch_partials(u64 *partials, unsigned base, unsigned count, T (&v)[R])
{
    u64 bits[R];
#pragma unroll
    for (unsigned r = 0; r < R; ++r) {
        const unsigned i = base + r * kBlock + threadIdx.x;
        bits[r] = i < count ? __hip_atomic_load(partials + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : (u64)0;
    }
#pragma unroll
    for (unsigned r = 0; r < R; ++r) {
        const unsigned i = base + r * kBlock + threadIdx.x;
        if (kSlots && i < count) {
            for (unsigned spins = 0; bits[r] == kEmptySlot && spins < kSlotSpins; ++spins)
                bits[r] = __hip_atomic_load(partials + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            (void)__hip_atomic_exchange(partials + i, kEmptySlot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        v[r] = __builtin_bit_cast(T, bits[r]);
    }
}

// Sum of the grid's partials in a fixed order, by all threads of the calling block.
// Returns the total in thread 0.  kSlots: the partials are slots (publish_to_slot), taken as they arrive.
template <class F, bool kSlots = false>
__device__ __forceinline__ typename F::Total sum_partials(u64 *partials, unsigned count,
                                                          typename F::Total *lds /* kBlock entries */)
{
    typedef typename F::Total Total;
    const unsigned tid = threadIdx.x;
    constexpr unsigned R = 8;                   // partials per thread and trip to where they live
    if (F::kMfmaFinish) {
        // The next level of the paper's hierarchy, in binary64, by one wavefront:
        // first MMA  D <- A x 1 + D with A = 64 partials (16 x 4), chained over all partials;
        // second MMA D' <- 1 x D.
        // Every thread of the block fetches partials, so 2048 of them cost one round trip to where they live; the first
        // wavefront takes them from shared memory, 256 at a time, in index order.
        Total total = 0;
        const bool first_wave = __builtin_amdgcn_readfirstlane(tid >> 6) == 0;   // scalar: matrix instructions ignore the lane mask
        f64x4 d = {0., 0., 0., 0.};
        for (unsigned base = 0; base < count; base += kBlock * R) {
            double a[R];
            fetch_partials<double, kSlots, R>(partials, base, count, a);
#pragma unroll
            for (unsigned r = 0; r < R; ++r) {
                const unsigned from = base + r * kBlock;
                if (from >= count) break;
                if (from) __syncthreads();          // the 256 before have been read
                lds[tid] = a[r];
                __syncthreads();
                if (first_wave) {
                    const unsigned left = count - from;
                    const unsigned chunks = left >= kBlock ? kBlock / 64 : (left + 63) / 64;
                    for (unsigned j = 0; j < chunks; ++j) d = __builtin_amdgcn_mfma_f64_16x16x4f64(lds[j * 64 + tid], 1.0, d, 0, 0, 0);
                }
            }
        }
        if (first_wave) {
            f64x4 dp = {0., 0., 0., 0.};
#pragma unroll
            for (int r = 0; r < 4; ++r) dp = __builtin_amdgcn_mfma_f64_16x16x4f64(1.0, d[r], dp, 0, 0, 0);
            total = (Total)dp[0];
        }
        return total;
    } else {
        Total t = 0;
        for (unsigned base = 0; base < count; base += kBlock * R) {
            Total a[R];
            fetch_partials<Total, kSlots, R>(partials, base, count, a);
#pragma unroll
            for (unsigned r = 0; r < R; ++r) t += a[r];
        }
        lds[tid] = t;
        __syncthreads();
        for (unsigned off = kBlock / 2; off > 0; off >>= 1) {
            if (tid < off) lds[tid] += lds[tid + off];
            __syncthreads();
        }
        return lds[0];
    }
}

// ---------------------------------------------------------------------------------------------
// flat sum: one pass over HBM, one partial per block, last block finishes
// ---------------------------------------------------------------------------------------------
struct FlatArgs {
    Run run;
    u64 *partials;      // kMaxGrid slots
    unsigned *ticket;   // zero before the launch; the finishing block resets it
    u64 *slots;         // finish 6, 7: one per block, all empty (kEmptySlot) before the launch; the finishing block empties them
    unsigned *leaves;   // finish 7, 8: eight tickets (8: counted sums), 256 bytes apart, zero before the launch and after it
    void *out;
    unsigned max_chain; // loop iterations between folds
    int layout;         // which slabs a block takes (see slab_schedule)
    int finish;         // 0/1/4: the last block to arrive sums the partials; 2: a second kernel does; 3: atomic additions;
                        // 5: atomic additions that count the blocks as well (integers only); 6: as 4, but nobody waits
                        // for its partial to arrive: the last block does, slot by slot (floating point only); 7, 8: as 6
                        // and 5, the arrivals counted in two levels (by accelerator die, then device-wide)
    unsigned stagger;   // start of wavefront w delayed by w x stagger x 64 cycles (long runs only)
    unsigned pause;     // every loop iteration ends with this many 64-cycle sleeps
};

constexpr int kXcds = 8;  // workgroup b is dispatched to accelerator die b % 8

// Which slabs (block-sized runs of U x 4 KiB) a block reads: slab k of the block is start + k*stride.
//   layout 0  interleaved: at any time the grid reads one contiguous moving window
//   layout 1  blocked: every block streams its own contiguous share of the array
//   layout 2  die-blocked: every accelerator die owns a contiguous eighth, interleaved among its blocks
__host__ __device__ __forceinline__ void slab_schedule(int layout, u64 nslab, u64 G, u64 b, u64 *start, u64 *stride, u64 *count)
{
    if (layout == 1) {
        const u64 q = nslab / G, r = nslab % G;
        *start = b * q + (b < r ? b : r);
        *stride = 1;
        *count = q + (b < r ? 1 : 0);
    } else if (layout == 2 && G >= (u64)kXcds) {
        const u64 x = b % kXcds, l = b / kXcds;
        const u64 gx = (G - x + kXcds - 1) / kXcds;              // blocks on this die
        const u64 lo = nslab * x / kXcds, hi = nslab * (x + 1) / kXcds;
        *start = lo + l;
        *stride = gx;
        *count = (hi - lo > l) ? (hi - lo - l + gx - 1) / gx : 0;
    } else {
        *start = b;
        *stride = G;
        *count = (nslab > b) ? (nslab - b + G - 1) / G : 0;
    }
}

template <class F, int U, bool NT>
__global__ void __launch_bounds__(kBlock) sum_flat_kernel(FlatArgs a)
{
    typedef typename F::Total Total;
    const unsigned tid = threadIdx.x, lane = tid & 63u;
    // The wavefront's number, read into a scalar register: a branch on it is then a real branch.  As a per-lane value
    // it would only mask lanes off, and a matrix instruction ignores that mask: a wavefront that was meant to skip an
    // MMA would execute it on whatever its registers hold.
    const unsigned wave = (unsigned)__builtin_amdgcn_readfirstlane((int)(tid >> 6));
    const u64 G = gridDim.x;
    constexpr u64 kSlab = (u64)kBlock * U;         // vectors per block iteration
    const u64 nslab = a.run.nvec / kSlab;

    typename F::Acc acc;
    F::clear(acc);
    Total wave_total = 0;
    unsigned chain = 0;

    u64 s0, stride, count;
    slab_schedule(a.layout, nslab, G, blockIdx.x, &s0, &stride, &count);
    // The four wavefronts of a block start a fraction of a loop period apart (wavefront w waits w x stagger x 64
    // cycles; the loop period is about 2700), so that they do not all issue their first loads in the same instant.
    // Measured: 1-2.5 us less per call at every size from 256 MiB to 4 GiB and for both families (a start-up effect,
    // it does not grow with the run), nothing or a slight loss at 128 MiB and below, so short runs skip it.  256 and
    // 512 cycles per wavefront are equally good; staggering blocks as well changed nothing; the segmented kernels
    // gain nothing from it.
    if (count >= 32)
        for (unsigned i = 0; i < wave * a.stagger; ++i) __builtin_amdgcn_s_sleep(1);
    // What does not fill a whole slab -- the vectors behind the last whole slab (one block's), the elements in front of
    // the first and behind the last aligned vector (block 0's) -- is loaded ahead of the stream and added behind it, so
    // that its latency is not paid on its own at the end of the block's work.  Every lane loads (those past the end
    // the array's last vector again), so no load sits under a per-lane branch; such a lane then adds zeros.
    const bool has_rest = blockIdx.x == (unsigned)(nslab % G) && nslab * kSlab < a.run.nvec;
    const bool has_edge = blockIdx.x == 0 && wave == 0 && (a.run.nhead | a.run.ntail);
    u32x4 rest[U];
    u32x4 edge = {0u, 0u, 0u, 0u};
    if (has_rest) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const u64 idx = nslab * kSlab + (u64)u * kBlock + tid;
            rest[u] = load16<NT>(a.run.body + (idx < a.run.nvec ? idx : a.run.nvec - 1));
        }
    }
    if (has_edge) edge = edge_vector<F>(a.run, (int)lane);

    // load u of a block covers 4 KiB contiguous: every wavefront reads whole 1-KiB tiles
    const u32x4 *p = a.run.body + s0 * kSlab + tid;
    const u64 step = stride * kSlab;

    for (u64 k = 0; k < count; ++k, p += step) {
        u32x4 cur[U];
#pragma unroll
        for (int u = 0; u < U; ++u) cur[u] = load16<NT>(p + u * kBlock);
        __builtin_amdgcn_sched_barrier(0);     // issue every load of the slab before the first MMA waits
#pragma unroll
        for (int u = 0; u < U; ++u) F::consume(acc, u, cur[u]);
        if (++chain >= a.max_chain) { wave_total += F::fold(acc); chain = 0; }
        for (unsigned i = 0; i < a.pause; ++i) __builtin_amdgcn_s_sleep(1);
    }

    if (has_rest) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const u64 idx = nslab * kSlab + (u64)u * kBlock + tid;
            const u32x4 zero = {0u, 0u, 0u, 0u};
            F::consume(acc, u, idx < a.run.nvec ? rest[u] : zero);
        }
    }
    if (has_edge) F::consume(acc, 0, edge);

    wave_total += F::fold(acc);

    __shared__ Total lds[kBlock];
    __shared__ unsigned is_last;
    if (lane == 0) lds[wave] = wave_total;
    __syncthreads();
    if (gridDim.x == 1 && a.finish != 2 && a.finish != 3) {
        // a single block has nobody to meet: its total is the result (what the next level would make of one partial, bit for bit)
        if (tid == 0) *(typename F::Out *)a.out = F::to_out((lds[0] + lds[1]) + (lds[2] + lds[3]));
        return;
    }
    if (a.finish == 2) {
        // partials are summed by finish_kernel, launched behind this kernel on the same stream
        if (tid == 0) a.partials[blockIdx.x] = __builtin_bit_cast(u64, (lds[0] + lds[1]) + (lds[2] + lds[3]));
        return;
    }
    if (a.finish == 3) {
        // the atomic-addition scheme of Section II: every block adds its total to the result (cleared by a fill kernel
        // launched ahead).  For floating point the order of arrival decides the rounding, so runs differ in the last bits.
        if (tid == 0)
            __hip_atomic_fetch_add((typename F::Out *)a.out, F::to_out((lds[0] + lds[1]) + (lds[2] + lds[3])), __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
        return;
    }
    if (a.finish == 5 || a.finish == 8) {
        // Integer totals only (the host sees to that).  Integer addition does not care about the order, so the blocks may
        // simply add their totals up with atomic additions, as Section II describes -- and the same addition can count
        // them: the word holds the running sum above bit 15 and the number of blocks that have added to it below (a grid
        // has at most 16384 blocks, and a block's total shifted left by 15 leaves the count alone, whatever its sign).
        // What the addition returns tells the block whether it was the last one, and then old + own is the whole sum:
        // one round trip instead of three (publish, ticket, read the partials), no partials, no second launch, and the
        // result cannot depend on who arrived when.  |sum| stays below 2^48 for up to 2^41 int8 elements.
        if constexpr (std::is_integral<Total>::value) {
            if (tid == 0) {
                const i64 block_total = (i64)((lds[0] + lds[1]) + (lds[2] + lds[3]));
                u64 *word = (u64 *)(a.ticket + 2);                       // the eight bytes behind the ticket, on its line
                u64 mine = ((u64)block_total << 15) + 1u;
                unsigned arrivals = gridDim.x;
                bool up = true;
                if (a.finish == 8) {
                    // in two levels (see finish 7 below for why): the blocks of a die add to the die's own word, and the
                    // one that completes its count adds the die's sum to the common word, which counts dies
                    const unsigned die = blockIdx.x % kXcds;
                    const unsigned on_die = (gridDim.x - die + kXcds - 1) / kXcds;
                    u64 *leaf = (u64 *)(a.leaves + die * 64u);
                    const u64 now = __hip_atomic_fetch_add(leaf, mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + mine;
                    up = (now & 0x7fffu) == on_die;
                    if (up) {
                        (void)__hip_atomic_exchange(leaf, (u64)0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        mine = (now & ~(u64)0x7fffu) + 1u;               // the die's sum, counted as one arrival
                        arrivals = gridDim.x < (unsigned)kXcds ? gridDim.x : (unsigned)kXcds;
                    }
                }
                if (up) {
                    const u64 now = __hip_atomic_fetch_add(word, mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + mine;
                    if ((now & 0x7fffu) == arrivals) {
                        *(typename F::Out *)a.out = (typename F::Out)((i64)now >> 15);
                        (void)__hip_atomic_exchange(word, (u64)0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
                }
            }
        }
        return;
    }
    if (a.finish == 6 || a.finish == 7) {
        // As finish 4 below, one round trip shorter: the block sends its partial off (an atomic exchange whose old value
        // nobody needs) and draws its ticket at once.  The last ticket then says that every partial is on its way, not
        // that it has arrived, so the slots start out empty and the finishing block reads each until it is not.
        if constexpr (!std::is_integral<Total>::value) {
            if (tid == 0) {
                publish_to_slot(a.slots + blockIdx.x, (lds[0] + lds[1]) + (lds[2] + lds[3]));
                unsigned last = 0u;
                if (a.finish == 7) {
                    // Tickets in two levels.  Read-modify-writes of one line of memory are served one after the other,
                    // about 8 ns each, so when all blocks arrive together the last waits for a queue of them.  Each die's
                    // blocks (block b runs on die b mod 8) draw from a ticket of their own, on a line of its own (eight
                    // tickets next to each other gain nothing), and the last of a die draws from the common one: eight
                    // short queues side by side and one of eight.
                    const unsigned die = blockIdx.x % kXcds;
                    const unsigned on_die = (gridDim.x - die + kXcds - 1) / kXcds;
                    unsigned *leaf = a.leaves + die * 64u;
                    const unsigned t = __hip_atomic_fetch_add(leaf, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    if (t == on_die - 1) {
                        (void)__hip_atomic_exchange(leaf, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        const unsigned dies = gridDim.x < (unsigned)kXcds ? gridDim.x : (unsigned)kXcds;
                        const unsigned r = __hip_atomic_fetch_add(a.ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        last = (r == dies - 1) ? 1u : 0u;
                    }
                } else {
                    const unsigned t = __hip_atomic_fetch_add(a.ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    last = (t == gridDim.x - 1) ? 1u : 0u;
                }
                is_last = last;
            }
            __syncthreads();
            if (is_last) {
                Total total = sum_partials<F, true>(a.slots, gridDim.x, lds);
                if (tid == 0) {
                    *(typename F::Out *)a.out = F::to_out(total);
                    (void)__hip_atomic_exchange(a.ticket, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
        }
        return;
    }
    if (tid == 0) {
        Total block_total = ((lds[0] + lds[1]) + (lds[2] + lds[3]));
        // The partial must be visible device-wide before the ticket moves.  The block that draws the
        // last ticket has read, through the chain of read-modify-writes, from every other block's
        // ticket; its acquire fence below then makes all partials visible to it.
        unsigned t;
        if (a.finish == 4) {
            // The partial is the only thing this block has to publish.  A device-scope release fence would write back
            // every dirty line of this die's L2 (several microseconds per block, which is what finish 0/1 pay), so the
            // partial travels in a read-modify-write instead: a device-scope atomic exchange is performed where the dies
            // of the device meet, exactly like the ticket's own addition, and it has been performed once its old value
            // has come back.  The ticket's increment is made to depend on that old value, so it cannot be issued earlier.
            const u64 old = __hip_atomic_exchange(a.partials + blockIdx.x, __builtin_bit_cast(u64, block_total),
                                                  __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            unsigned one = 1u;
            asm volatile("" : "+s"(one) : "v"((unsigned)old), "v"((unsigned)(old >> 32)));   // `one` exists only after `old` does
            t = __hip_atomic_fetch_add(a.ticket, one, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        } else {
            store_partial(a.partials + blockIdx.x, block_total);
            t = (a.finish == 0)
                ? __hip_atomic_fetch_add(a.ticket, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT)
                : __hip_atomic_fetch_add(a.ticket, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        }
        is_last = (t == gridDim.x - 1) ? 1u : 0u;
    }
    __syncthreads();
    if (is_last) {
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        Total total = sum_partials<F>(a.partials, gridDim.x, lds);
        if (tid == 0) {
            *(typename F::Out *)a.out = F::to_out(total);
            // (a read-modify-write like every other access to the ticket, so that the next launch's additions find it)
            (void)__hip_atomic_exchange(a.ticket, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

// Second kernel of the two-kernel finish: one block sums the partials in the same fixed order.
template <class F>
__global__ void __launch_bounds__(kBlock) finish_kernel(u64 *partials, unsigned count, void *out)
{
    typedef typename F::Total Total;
    __shared__ Total lds[kBlock];
    Total total = sum_partials<F>(partials, count, lds);
    if (threadIdx.x == 0) *(typename F::Out *)out = F::to_out(total);
}

// ---------------------------------------------------------------------------------------------
// segmented sum, general form: one wavefront per segment (or per part of a long segment)
// ---------------------------------------------------------------------------------------------
struct SegArgs {
    const unsigned char *x;
    u64 nseg, seglen;   // elements
    void *out;
    unsigned max_chain;
    // Long segments are cut into `parts` pieces of part_len elements so that a few segments still
    // fill the chip; piece totals go to `partials` and finish_segments_kernel adds them up.
    u64 parts, part_len;
    u64 *partials;
    // One block per piece, finish in the same kernel (seg_finish = 1): the block that is the last of its segment to arrive adds
    // the segment's piece totals.  Floating point: totals go to `slots` (one per piece, all empty before the launch and after
    // it) and arrivals are counted in tickets[segment]; int8: total and count share the 64-bit word counted[segment].
    // Tickets and counted words are zero before the launch and after it.
    int seg_finish;
    // 1 = arrivals counted in two levels (a few segments of many pieces): piece p of a segment meets the pieces with the same p mod 8 at
    // word 1 + p mod 8 of the segment's nine words, the last of each of the eight groups at word 0; every word on a 256-byte
    // line of its own (read-modify-writes of one line of memory are served one after the other)
    int seg_two_levels;
    unsigned seg_word_stride;   // one level: the words of two segments are this many 8-byte words apart (32 = a 256-byte line each, so
                                // that the arrivals of different segments do not queue up behind each other; 1 where there are too many)
    u64 *slots;
    unsigned *tickets;
    u64 *counted;
};

// all-ones in the low b bytes of a 128-bit word (b = 0 .. 16), as two 64-bit halves
__device__ __forceinline__ void bytes_below(unsigned b, u64 *lo, u64 *hi)
{
    *lo = b >= 8u ? ~0ull : (1ull << (8u * b)) - 1ull;
    *hi = b <= 8u ? 0ull : (b >= 16u ? ~0ull : (1ull << (8u * (b - 8u))) - 1ull);
}

// bytes [lo, hi) of a vector, zeros elsewhere (0 <= lo, hi <= 16; nothing is kept if hi <= lo)
__device__ __forceinline__ u32x4 keep_bytes(u32x4 v, unsigned lo, unsigned hi)
{
    u64 hl, hh, ll, lh;
    bytes_below(hi, &hl, &hh);
    bytes_below(lo, &ll, &lh);
    const u64 ml = hl & ~ll, mh = hh & ~lh;
    return u32x4{v[0] & (unsigned)ml, v[1] & (unsigned)(ml >> 32), v[2] & (unsigned)mh, v[3] & (unsigned)(mh >> 32)};
}

// keep_bytes for every (lo, hi) as a table in LDS: one 16-byte read and four ANDs per vector instead of a dozen
// 64-bit shifts and selects -- the kernels that clear bytes per load are bound by instruction issue, not by HBM.
constexpr int kByteMasks = 17 * 17;
__device__ __forceinline__ void fill_byte_masks(u32x4 *table /* kByteMasks entries, shared */)
{
    for (unsigned i = threadIdx.x; i < (unsigned)kByteMasks; i += kBlock)
        table[i] = keep_bytes(u32x4{~0u, ~0u, ~0u, ~0u}, i / 17u, i % 17u);
    __syncthreads();
}
__device__ __forceinline__ u32x4 keep_bytes(const u32x4 *table, u32x4 v, unsigned lo, unsigned hi)
{
    return v & table[lo * 17u + hi];
}

// The wavefront reads the 16-byte aligned vectors that overlap its segment (or piece), 64 x U at a time, and clears
// the bytes of the first and the last one that lie outside it: the zero padding of Section IV-A.  Lanes past the
// last vector read that vector again (one cache line for all of them) and keep nothing: a load under a branch would
// make the wait in front of the MMAs cover every load in flight.  An aligned vector that holds a byte of the array
// lies in the array's pages, so what is read beyond either end is mapped memory; it is cleared like the rest.
template <class F, int U, bool NT>
__global__ void __launch_bounds__(kBlock) sum_segmented_kernel(SegArgs a)
{
    typedef typename F::Total Total;
    const unsigned lane = threadIdx.x & 63u;
    const u64 wave_global = (u64)blockIdx.x * kWaves + (threadIdx.x >> 6);
    const u64 nwaves = (u64)gridDim.x * kWaves;
    constexpr u64 kChunk = 64ull * U;              // vectors per wave iteration
    const u64 npieces = a.nseg * a.parts;
    __shared__ u32x4 masks[kByteMasks];
    fill_byte_masks(masks);

    for (u64 piece = wave_global; piece < npieces; piece += nwaves) {
        // (a 64-bit division costs more than the rest of a short segment: only cut segments pay for it)
        const u64 seg = a.parts == 1 ? piece : piece / a.parts, part = a.parts == 1 ? 0 : piece % a.parts;
        const u64 first = part * a.part_len;
        const u64 len = first < a.seglen ? (a.seglen - first < a.part_len ? a.seglen - first : a.part_len) : 0;
        typename F::Acc acc;
        F::clear(acc);
        Total total = 0;
        if (len) {
            // (pointer arithmetic on the kernel argument keeps the loads in the global address space)
            const unsigned char *start = a.x + (seg * a.seglen + first) * F::kElemSize;
            const unsigned off = (unsigned)(uintptr_t)start & 15u;
            const u32x4 *base = (const u32x4 *)(start - off);
            const u64 end = off + len * F::kElemSize;          // end of the piece, in bytes from its first aligned vector
            const u64 cover = (end + 15) >> 4;                 // aligned vectors that overlap the piece
            unsigned chain = 0;
            for (u64 v0 = 0; v0 < cover; v0 += kChunk) {
                u32x4 cur[U];
                if (v0 != 0 && v0 + kChunk < cover) {          // neither end is in this chunk (the same for every lane)
#pragma unroll
                    for (int u = 0; u < U; ++u) cur[u] = load16<NT>(base + v0 + (u64)u * 64 + lane);
                    __builtin_amdgcn_sched_barrier(0);         // all loads of the chunk in flight before the first MMA waits
                } else {
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const u64 idx = v0 + (u64)u * 64 + lane;
                        cur[u] = load16<NT>(base + (idx < cover ? idx : cover - 1));
                    }
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const u64 idx = v0 + (u64)u * 64 + lane;
                        const unsigned lo = idx == 0 ? off : 0u;
                        const unsigned hi = idx >= cover ? 0u : (end - 16 * idx >= 16 ? 16u : (unsigned)(end - 16 * idx));
                        cur[u] = keep_bytes(masks, cur[u], lo, hi);
                    }
                }
#pragma unroll
                for (int u = 0; u < U; ++u) F::consume(acc, u, cur[u]);
                if (++chain >= a.max_chain) { total += F::fold(acc); chain = 0; }
            }
        }
        total += F::fold(acc);
        if (lane == 0) {
            if (a.parts == 1) ((typename F::Out *)a.out)[seg] = F::to_out(total);
            else a.partials[piece] = __builtin_bit_cast(u64, total);
        }
    }
}

// Segments that are exactly U whole tiles (1, 2, 4 or 8 KiB, 16-byte aligned): one wavefront per segment, the
// whole segment in flight at once, nothing but the MMAs, the fold and one store per segment.
// PIPE 0: plain loop.  PIPE 1: the next segment's loads are issued before the current one is worked on
// (the wait in front of the MMAs still covers both segments, because the loads ahead are conditional).
template <class F, int U, bool NT, int PIPE>
__global__ void __launch_bounds__(kBlock) sum_segments_tiles_kernel(SegArgs a)
{
    typedef typename F::Total Total;
    const unsigned lane = threadIdx.x & 63u;
    const u64 wave_global = (u64)blockIdx.x * kWaves + (threadIdx.x >> 6);
    const u64 nwaves = (u64)gridDim.x * kWaves;
    const u32x4 *base = (const u32x4 *)a.x + lane;
    typename F::Out *out = (typename F::Out *)a.out;
    if (PIPE == 0) {
        for (u64 seg = wave_global; seg < a.nseg; seg += nwaves) {
            u32x4 cur[U];
#pragma unroll
            for (int u = 0; u < U; ++u) cur[u] = load16<NT>(base + seg * (64ull * U) + (u64)u * 64);
            __builtin_amdgcn_sched_barrier(0);
            typename F::Acc acc;
            F::clear(acc);
#pragma unroll
            for (int u = 0; u < U; ++u) F::consume(acc, u, cur[u]);
            const Total total = F::fold(acc);
            if (lane == 0) out[seg] = F::to_out(total);
        }
    } else {
        u64 seg = wave_global;
        if (seg >= a.nseg) return;
        u32x4 cur[U];
#pragma unroll
        for (int u = 0; u < U; ++u) cur[u] = load16<NT>(base + seg * (64ull * U) + (u64)u * 64);
        while (true) {
            const u64 next = seg + nwaves;
            const bool more = next < a.nseg;                   // the same for every lane of the wavefront
            u32x4 nxt[U];
            if (more) {
#pragma unroll
                for (int u = 0; u < U; ++u) nxt[u] = load16<NT>(base + next * (64ull * U) + (u64)u * 64);
            }
            __builtin_amdgcn_sched_barrier(0);
            typename F::Acc acc;
            F::clear(acc);
#pragma unroll
            for (int u = 0; u < U; ++u) F::consume(acc, u, cur[u]);
            const Total total = F::fold(acc);
            if (lane == 0) out[seg] = F::to_out(total);
            if (!more) break;
            for (int u = 0; u < U; ++u) cur[u] = nxt[u];
            seg = next;
        }
    }
}

// Long segments: one block per segment (or per piece of one).  The block streams its piece exactly like the
// flat kernel streams the array -- slabs of U x 4 KiB, each load instruction of the block contiguous -- so a
// handful of long segments reads HBM as a few hundred wide streams instead of thousands of narrow ones.
template <class F, int U, bool NT>
__global__ void __launch_bounds__(kBlock) sum_segments_block_kernel(SegArgs a)
{
    typedef typename F::Total Total;
    const unsigned tid = threadIdx.x, lane = tid & 63u;
    // The wavefront's number, read into a scalar register: a branch on it is then a real branch.  As a per-lane value
    // it would only mask lanes off, and a matrix instruction ignores that mask: a wavefront that was meant to skip an
    // MMA would execute it on whatever its registers hold.
    const unsigned wave = (unsigned)__builtin_amdgcn_readfirstlane((int)(tid >> 6));
    constexpr u64 kSlab = (u64)kBlock * U;
    const u64 npieces = a.nseg * a.parts;
    __shared__ Total lds[kBlock];
    __shared__ unsigned is_last;

    for (u64 piece = blockIdx.x; piece < npieces; piece += gridDim.x) {
        const u64 seg = piece / a.parts, part = piece % a.parts;
        const u64 first = part * a.part_len;
        const u64 len = first < a.seglen ? (a.seglen - first < a.part_len ? a.seglen - first : a.part_len) : 0;
        const Run run = make_run<F::kElemSize>(a.x + (seg * a.seglen + first) * F::kElemSize, len);
        typename F::Acc acc;
        F::clear(acc);
        Total wave_total = 0;
        unsigned chain = 0;
        const u64 nslab = run.nvec / kSlab;
        const u32x4 *p = run.body + tid;
        // What does not fill a whole slab -- the vectors behind the last whole slab, and the elements in front of the
        // first and behind the last aligned vector -- is loaded ahead of the stream and added behind it, so that its
        // latency is not paid on its own at the end of every piece.  Every lane loads (those past the end the piece's
        // last vector again), so no load sits under a per-lane branch; what such a lane loaded is replaced by zeros.
        const bool has_edge = wave == 0 && (run.nhead | run.ntail);
        u32x4 edge = {0u, 0u, 0u, 0u};
        if (has_edge) edge = edge_vector<F>(run, (int)lane);
        const bool has_rest = nslab * kSlab < run.nvec;    // (the same for the whole block)
        u32x4 rest[U];
        if (has_rest) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const u64 idx = nslab * kSlab + (u64)u * kBlock + tid;
                rest[u] = load16<NT>(run.body + (idx < run.nvec ? idx : run.nvec - 1));
            }
        }
        for (u64 k = 0; k < nslab; ++k, p += kSlab) {
            u32x4 cur[U];
#pragma unroll
            for (int u = 0; u < U; ++u) cur[u] = load16<NT>(p + u * kBlock);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int u = 0; u < U; ++u) F::consume(acc, u, cur[u]);
            if (++chain >= a.max_chain) { wave_total += F::fold(acc); chain = 0; }
        }
        if (has_rest) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const u64 idx = nslab * kSlab + (u64)u * kBlock + tid;
                const u32x4 zero = {0u, 0u, 0u, 0u};
                F::consume(acc, u, idx < run.nvec ? rest[u] : zero);
            }
        }
        if (has_edge) F::consume(acc, 0, edge);
        wave_total += F::fold(acc);
        if (lane == 0) lds[wave] = wave_total;
        __syncthreads();
        if (tid == 0) {
            const Total total = (lds[0] + lds[1]) + (lds[2] + lds[3]);
            is_last = 0u;
            if (a.parts == 1) {
                ((typename F::Out *)a.out)[seg] = F::to_out(total);
            } else if (!a.seg_finish) {
                a.partials[piece] = __builtin_bit_cast(u64, total);      // finish_segments_kernel, launched behind this kernel, adds them
            } else if constexpr (std::is_integral<Total>::value) {
                // integer totals: one atomic addition per piece adds them up and counts them (sum above bit 15, count below;
                // at most 4096 pieces per segment); whoever completes the count holds the segment's sum
                u64 mine = ((u64)(i64)total << 15) + 1u;
                u64 *word = a.counted + seg * a.seg_word_stride;
                u64 arrivals = a.parts;
                bool up = true;
                if (a.seg_two_levels) {
                    const u64 group = part % 8u, in_group = (a.parts - group + 7u) / 8u;
                    u64 *leaf = a.counted + (seg * 9u + 1u + group) * 32u;
                    const u64 now = __hip_atomic_fetch_add(leaf, mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + mine;
                    up = (now & 0x7fffu) == in_group;
                    if (up) {
                        (void)__hip_atomic_exchange(leaf, (u64)0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        mine = (now & ~(u64)0x7fffu) + 1u;               // the group's sum, counted as one arrival
                    }
                    word = a.counted + seg * 9u * 32u;
                    arrivals = a.parts < 8u ? a.parts : 8u;
                }
                if (up) {
                    const u64 now = __hip_atomic_fetch_add(word, mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + mine;
                    if ((now & 0x7fffu) == arrivals) {
                        ((typename F::Out *)a.out)[seg] = (typename F::Out)((i64)now >> 15);
                        (void)__hip_atomic_exchange(word, (u64)0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
                }
            } else {
                // the piece total is sent off to its slot and the segment's ticket drawn at once; the last ticket says that all
                // of the segment's totals are on their way, and fetch_partials reads each slot until it has arrived
                publish_to_slot(a.slots + piece, total);
                unsigned last = 0u;
                if (a.seg_two_levels) {
                    const unsigned group = (unsigned)(part % 8u), in_group = ((unsigned)a.parts - group + 7u) / 8u;
                    unsigned *leaf = a.tickets + (seg * 9u + 1u + group) * 64u;
                    const unsigned t = __hip_atomic_fetch_add(leaf, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    if (t == in_group - 1u) {
                        (void)__hip_atomic_exchange(leaf, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        const unsigned r = __hip_atomic_fetch_add(a.tickets + seg * 9u * 64u, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        last = (r == ((unsigned)a.parts < 8u ? (unsigned)a.parts : 8u) - 1u) ? 1u : 0u;
                    }
                } else {
                    const unsigned t = __hip_atomic_fetch_add(a.tickets + seg * a.seg_word_stride * 2u, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    last = (t == (unsigned)a.parts - 1u) ? 1u : 0u;
                }
                is_last = last;
            }
        }
        __syncthreads();                                   // lds is reused: by the sum of the piece totals, or by the next piece
        if constexpr (!std::is_integral<Total>::value) {
            if (is_last) {                                 // (the same for the whole block)
                const Total total = sum_partials<F, true>(a.slots + seg * a.parts, (unsigned)a.parts, lds);
                if (tid == 0) {
                    ((typename F::Out *)a.out)[seg] = F::to_out(total);
                    (void)__hip_atomic_exchange(a.tickets + (a.seg_two_levels ? seg * 9u * 64u : seg * a.seg_word_stride * 2u), 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
                __syncthreads();
            }
        }
    }
}

// One block per segment adds that segment's piece totals in a fixed order.
template <class F>
__global__ void __launch_bounds__(kBlock) finish_segments_kernel(u64 *partials, unsigned parts, void *out)
{
    typedef typename F::Total Total;
    __shared__ Total lds[kBlock];
    Total total = sum_partials<F>(partials + (u64)blockIdx.x * parts, parts, lds);
    if (threadIdx.x == 0) ((typename F::Out *)out)[blockIdx.x] = F::to_out(total);
}

// ---------------------------------------------------------------------------------------------
// segmented sum, short segments: sixteen segments per wavefront, one per row of the A operand.
//
// The first MMA of Section IV-A already yields one independent sum per row of A (every column of
// D holds the m row sums), so short segments need no second MMA at all: row i of A takes the
// elements of segment s0 + i, 32 (binary16) or 64 (int8) per MFMA, and after the chain column 0 of
// the accumulator is the sixteen results.  Requires 16-byte aligned segments (host-checked).
//
// A lane holds A[lane % 16][(lane / 16) * w .. + w): row = lane & 15, quarter = lane >> 4.  The
// classic family uses the same loads with row = lane >> 2, quarter = lane & 3 and a DPP reduction
// over each quad.
// ---------------------------------------------------------------------------------------------
struct RowArgs {
    const u32x4 *x;     // 16-byte aligned
    u64 nseg;
    unsigned nvec;      // 16-byte vectors per segment (1 .. 64)
    void *out;
};

struct F16MfmaRows {
    typedef float Out;
    typedef f32x4 Acc;
    static __device__ __forceinline__ unsigned row(unsigned lane) { return lane & 15u; }
    static __device__ __forceinline__ unsigned quarter(unsigned lane) { return lane >> 4; }
    static __device__ __forceinline__ Acc zero() { return f32x4{0.f, 0.f, 0.f, 0.f}; }
    static __device__ __forceinline__ void consume(Acc &d, u32x4 v)
    {
        const f16x8 ones = {1, 1, 1, 1, 1, 1, 1, 1};
        d = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, v), ones, d, 0, 0, 0);
    }
    // lane l, register r holds D[4*(l/16)+r][l%16]; column 0 lives in lanes 0, 16, 32, 48
    static __device__ __forceinline__ void store(const Acc &d, Out *out, u64 seg0, u64 nseg, unsigned lane)
    {
        if ((lane & 15u) == 0) {
            const u64 s = seg0 + 4 * (lane >> 4);
            if (s + 4 <= nseg && ((uintptr_t)(out + s) & 15u) == 0) {
                *(f32x4 *)(out + s) = d;               // four results in one 16-byte store
            } else {
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (s + r < nseg) out[s + r] = d[r];
            }
        }
    }
};

struct I8MfmaRows {
    typedef i64 Out;
    typedef i32x4 Acc;
    static __device__ __forceinline__ unsigned row(unsigned lane) { return lane & 15u; }
    static __device__ __forceinline__ unsigned quarter(unsigned lane) { return lane >> 4; }
    static __device__ __forceinline__ Acc zero() { return i32x4{0, 0, 0, 0}; }
    static __device__ __forceinline__ void consume(Acc &d, u32x4 v)
    {
        const i32x4 ones = {0x01010101, 0x01010101, 0x01010101, 0x01010101};
        d = __builtin_amdgcn_mfma_i32_16x16x64_i8(__builtin_bit_cast(i32x4, v), ones, d, 0, 0, 0);
    }
    static __device__ __forceinline__ void store(const Acc &d, Out *out, u64 seg0, u64 nseg, unsigned lane)
    {
        if ((lane & 15u) == 0) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                u64 s = seg0 + 4 * (lane >> 4) + r;
                if (s < nseg) out[s] = (i64)d[r];
            }
        }
    }
};

struct F16ClassicRows {
    typedef float Out;
    typedef float Acc;
    static __device__ __forceinline__ unsigned row(unsigned lane) { return lane >> 2; }
    static __device__ __forceinline__ unsigned quarter(unsigned lane) { return lane & 3u; }
    static __device__ __forceinline__ Acc zero() { return 0.f; }
    static __device__ __forceinline__ void consume(Acc &s, u32x4 v)
    {
        f16x8 h = __builtin_bit_cast(f16x8, v);
        float a = ((float)h[0] + (float)h[1]) + ((float)h[2] + (float)h[3]);
        float b = ((float)h[4] + (float)h[5]) + ((float)h[6] + (float)h[7]);
        s += a + b;
    }
    static __device__ __forceinline__ void store(const Acc &s, Out *out, u64 seg0, u64 nseg, unsigned lane)
    {
        float v = s;
        v += __builtin_bit_cast(float, dpp_i32<kQuadXor1>(__builtin_bit_cast(int, v)));
        v += __builtin_bit_cast(float, dpp_i32<kQuadXor2>(__builtin_bit_cast(int, v)));
        u64 sg = seg0 + (lane >> 2);
        if ((lane & 3u) == 0 && sg < nseg) out[sg] = v;
    }
};

struct I8ClassicRows {
    typedef i64 Out;
    typedef int Acc;
    static __device__ __forceinline__ unsigned row(unsigned lane) { return lane >> 2; }
    static __device__ __forceinline__ unsigned quarter(unsigned lane) { return lane & 3u; }
    static __device__ __forceinline__ Acc zero() { return 0; }
    static __device__ __forceinline__ void consume(Acc &s, u32x4 v)
    {
#pragma unroll
        for (int k = 0; k < 4; ++k) s = __builtin_amdgcn_sdot4((int)v[k], 0x01010101, s, false);
    }
    static __device__ __forceinline__ void store(const Acc &s, Out *out, u64 seg0, u64 nseg, unsigned lane)
    {
        int v = s;                      // at most 64 vectors x 16 x 128 per lane: far inside int32
        v += dpp_i32<kQuadXor1>(v);
        v += dpp_i32<kQuadXor2>(v);
        u64 sg = seg0 + (lane >> 2);
        if ((lane & 3u) == 0 && sg < nseg) out[sg] = (i64)v;
    }
};

// TC = loads per row group per iteration (1, 2, 4 or 8); a wavefront keeps 8 loads in flight by
// working on GRP = 8 / TC groups of sixteen segments at a time.
template <class R, int TC, bool NT>
__global__ void __launch_bounds__(kBlock) sum_rows_kernel(RowArgs a)
{
    constexpr int GRP = 8 / TC;
    const unsigned lane = threadIdx.x & 63u;
    const unsigned row = R::row(lane), quarter = R::quarter(lane);
    const u64 wave_global = (u64)blockIdx.x * kWaves + (threadIdx.x >> 6);
    const u64 nwaves = (u64)gridDim.x * kWaves;
    const u64 ngroups = (a.nseg + 15) / 16;
    const u64 nsuper = (ngroups + GRP - 1) / GRP;

    for (u64 sg = wave_global; sg < nsuper; sg += nwaves) {
        typename R::Acc acc[GRP];
#pragma unroll
        for (int g = 0; g < GRP; ++g) acc[g] = R::zero();
        for (unsigned t0 = 0; t0 < a.nvec; t0 += 4 * TC) {       // one trip unless a segment has more than 4*TC vectors
            u32x4 cur[GRP][TC];
#pragma unroll
            for (int g = 0; g < GRP; ++g) {
                const u64 seg = (sg * GRP + g) * 16 + row;
#pragma unroll
                for (int t = 0; t < TC; ++t) {
                    const unsigned vi = t0 + 4 * t + quarter;
                    u32x4 v = {0u, 0u, 0u, 0u};
                    if (seg < a.nseg && vi < a.nvec) v = load16<NT>(a.x + seg * a.nvec + vi);
                    cur[g][t] = v;
                }
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int g = 0; g < GRP; ++g)
#pragma unroll
                for (int t = 0; t < TC; ++t) R::consume(acc[g], cur[g][t]);
        }
#pragma unroll
        for (int g = 0; g < GRP; ++g)
            R::store(acc[g], (typename R::Out *)a.out, (sg * GRP + g) * 16, a.nseg, lane);
    }
}

// ---------------------------------------------------------------------------------------------
// small helpers
// ---------------------------------------------------------------------------------------------
template <class T>
__global__ void fill_zero_kernel(T *out, u64 count)
{
    u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) out[i] = (T)0;
}

__global__ void fill_zero_words_kernel(unsigned *p, unsigned count)
{
    unsigned i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = 0u;
}

// `count` slots marked empty, the first `words` words at `zero` cleared, and (if given) the eight tickets of the second
// level, 256 bytes apart and eight bytes each, by one block
__global__ void empty_slots_kernel(u64 *slots, unsigned count, unsigned *zero, unsigned words, unsigned *leaves)
{
    for (unsigned i = threadIdx.x; i < count; i += blockDim.x) slots[i] = kEmptySlot;
    if (threadIdx.x < words) zero[threadIdx.x] = 0u;
    if (leaves && threadIdx.x < 16u) leaves[(threadIdx.x >> 1) * 64u + (threadIdx.x & 1u)] = 0u;
}

// Plain 16-byte-per-lane copy of `nvec` vectors: a kernel of exactly known traffic, used to
// calibrate hardware byte counters.
__global__ void __launch_bounds__(kBlock) copy_kernel(u32x4 *dst, const u32x4 *src, u64 nvec)
{
    for (u64 i = (u64)blockIdx.x * kBlock + threadIdx.x; i < nvec; i += (u64)gridDim.x * kBlock) dst[i] = src[i];
}

// One group through both MMAs of Section IV-A, results written out in matrix order.
// A is filled row by row: element e of the group sits at A[e / depth][e % depth].
// Lane l of the A operand holds A[l % 16][(l / 16) * w .. + w) with w = depth / 4 consecutive k.
__global__ void __launch_bounds__(64) group_probe_f16_kernel(const unsigned short *x, unsigned count,
                                                             float *D, float *Dp)
{
    const unsigned lane = threadIdx.x;
    const unsigned row = lane & 15u, kgrp = lane >> 4;
    f16x8 a;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        unsigned e = row * 32u + kgrp * 8u + k;
        unsigned short bits = e < count ? x[e] : (unsigned short)0;
        a[k] = __builtin_bit_cast(_Float16, bits);
    }
    const f16x8 ones = {1, 1, 1, 1, 1, 1, 1, 1};
    f32x4 d = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, ones, f32x4{0.f, 0.f, 0.f, 0.f}, 0, 0, 0);
    f32x4 dp = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        D[(4 * kgrp + r) * 16 + row] = d[r];       // accumulator register r of lane l is D[4*(l/16)+r][l%16]
        dp = __builtin_amdgcn_mfma_f32_16x16x4f32(1.0f, d[r], dp, 0, 0, 0);
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) Dp[(4 * kgrp + r) * 16 + row] = dp[r];
}

__global__ void __launch_bounds__(64) group_probe_i8_kernel(const signed char *x, unsigned count,
                                                            int *D, double *Dp)
{
    const unsigned lane = threadIdx.x;
    const unsigned row = lane & 15u, kgrp = lane >> 4;
    i32x4 a;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        unsigned word = 0;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            unsigned e = row * 64u + kgrp * 16u + w * 4 + b;
            unsigned byte = e < count ? (unsigned)(unsigned char)x[e] : 0u;
            word |= byte << (8 * b);
        }
        a[w] = (int)word;
    }
    const i32x4 ones = {0x01010101, 0x01010101, 0x01010101, 0x01010101};
    i32x4 d = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, ones, i32x4{0, 0, 0, 0}, 0, 0, 0);
    f64x4 dp = {0., 0., 0., 0.};
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        D[(4 * kgrp + r) * 16 + row] = d[r];
        dp = __builtin_amdgcn_mfma_f64_16x16x4f64(1.0, (double)d[r], dp, 0, 0, 0);
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) Dp[(4 * kgrp + r) * 16 + row] = dp[r];
}

} // namespace redux
