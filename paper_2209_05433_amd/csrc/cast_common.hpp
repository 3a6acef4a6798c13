// Pieces shared by the translation units of the amax / cast kernels (gfx950).
#pragma once

#include "common.hpp"
#include "fp8_decode.hpp"
#include "fp8_encode.hpp"

namespace fp8mm {
namespace {

constexpr int kThreads = 256;
constexpr int kAmaxBlocks = 256 * 4;      // read-only stream: 32 KB chunks dealt to this many workgroups measured best
// read+write stream: short contiguous runs of 16 384 elements per workgroup measured best at every
// size (6.04 10^8 bf16 elements: 290 us, against 320 us when the grid stopped growing at 16 384
// workgroups); the limit only keeps the grid dimension in range
constexpr int kCastBlocks = 1 << 20;
constexpr int kMultiMax = FP8_MULTI_MAX;  // tensors per launch of the multi-tensor forms
constexpr size_t kStreamingStoreBytes = (size_t)384 << 20;   // outputs from this size on are stored non-temporally

typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));

// ------------------------------------------------------------------------------------------
// amax.  Magnitude bits of IEEE numbers order like unsigned integers (Section 3.1 relies on
// the same property for FP8), NaN patterns sort above infinity, so an unsigned max of the
// sign-stripped bits is the NaN-propagating amax.  bfloat16 pairs are reduced as packed
// 16-bit integers.
// ------------------------------------------------------------------------------------------
template <int DT> struct Elem;
template <> struct Elem<FP8_F32>  { static constexpr int size = 4; static constexpr int per_vec = 4; };
template <> struct Elem<FP8_BF16> { static constexpr int size = 2; static constexpr int per_vec = 8; };

template <int DT>
__device__ __forceinline__ unsigned vec_mag_max(u32x4 v, unsigned run)
{
    if (DT == FP8_F32) {
        unsigned m0 = v.x & 0x7fffffffu, m1 = v.y & 0x7fffffffu;
        unsigned m2 = v.z & 0x7fffffffu, m3 = v.w & 0x7fffffffu;
        m0 = m0 > m1 ? m0 : m1;
        m2 = m2 > m3 ? m2 : m3;
        m0 = m0 > m2 ? m0 : m2;
        return run > m0 ? run : m0;
    } else {
        u16x2 r = __builtin_bit_cast(u16x2, run);
        r = __builtin_elementwise_max(r, __builtin_bit_cast(u16x2, v.x & 0x7fff7fffu));
        r = __builtin_elementwise_max(r, __builtin_bit_cast(u16x2, v.y & 0x7fff7fffu));
        r = __builtin_elementwise_max(r, __builtin_bit_cast(u16x2, v.z & 0x7fff7fffu));
        r = __builtin_elementwise_max(r, __builtin_bit_cast(u16x2, v.w & 0x7fff7fffu));
        return __builtin_bit_cast(unsigned, r);
    }
}

// Magnitude bits of one element, as the bits of an fp32 number.
template <int DT>
__device__ __forceinline__ unsigned scalar_mag(const void* x, size_t i)
{
    if (DT == FP8_F32) return ((const unsigned*)x)[i] & 0x7fffffffu;
    return ((unsigned)(((const unsigned short*)x)[i] & 0x7fffu)) << 16;
}

__device__ __forceinline__ unsigned block_max_u32(unsigned v)
{
    __shared__ unsigned part[kThreads / 64];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        unsigned o = __shfl_xor(v, off, 64);
        v = v > o ? v : o;
    }
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = v;
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
        for (int w = 1; w < kThreads / 64; ++w) v = v > part[w] ? v : part[w];
    }
    return v;   // valid in thread 0
}

__global__ void store_u32_kernel(unsigned* p, unsigned v) { *p = v; }

// ------------------------------------------------------------------------------------------
// scale = fmt_max / amax, one IEEE single division (Section 2; Table 1 "Max normal";
// Section 3.2: any real value).  Degenerate amax (0, NaN, inf) or a quotient that is not
// finite gives 1.
// ------------------------------------------------------------------------------------------
__host__ __device__ inline float scale_rule(float amax, int fmt)
{
    const float fmax = fmt == FP8_E4M3 ? 448.0f : 57344.0f;
    if (!(amax > 0.0f) || amax > 3.4028234663852886e38f) return 1.0f;
    const float s = fmax / amax;
    if (!(s <= 3.4028234663852886e38f)) return 1.0f;
    return s;
}

template <int DT>
__device__ __forceinline__ float load_scalar(const void* x, size_t i)
{
    if (DT == FP8_F32) return ((const float*)x)[i];
    return as_f32((unsigned)((const unsigned short*)x)[i] << 16);
}

// The 16 elements of one work item, scaled: from 2 (bf16) or 4 (fp32) 16-byte vectors.
template <int DT>
__device__ __forceinline__ void scale_item(const u32x4 (&v)[DT == FP8_BF16 ? 2 : 4], float s, float (&y)[16])
{
    if (DT == FP8_BF16) {
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                y[8 * j + 2 * d] = as_f32(v[j][d] << 16) * s;
                y[8 * j + 2 * d + 1] = as_f32(v[j][d] & 0xffff0000u) * s;
            }
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int d = 0; d < 4; ++d) y[4 * j + d] = as_f32(v[j][d]) * s;
    }
}

// How the vector kernels deal the work to lanes.  A lane that took 16 consecutive elements (32 or 64
// bytes of input) itself would make every load instruction of its wave touch 64 lines for a half
// or a quarter of their bytes.  Instead a lane takes single 16-byte vectors, kThreads vectors apart
// (every load instruction of a wave then reads 1 KB of consecutive bytes), rounds 16 elements from
// 2 (bf16) or 4 (fp32) such vectors at a time with the common routine, and stores the output bytes
// of each vector as one piece of 8 (bf16) or 4 (fp32) bytes, again consecutive across the wave.
// Measured on 2^28 elements against 16 consecutive elements per lane: bf16 6.4 -> 6.7 TB/s,
// fp32 4.25 -> 6.2 TB/s.
template <int DT> struct Piece;
template <> struct Piece<FP8_BF16> {
    typedef u32x2 type;
    static __device__ __forceinline__ type of(const u32x4& o, int k) { return (u32x2){o[2 * k], o[2 * k + 1]}; }
};
template <> struct Piece<FP8_F32> {
    typedef unsigned type;
    static __device__ __forceinline__ type of(const u32x4& o, int k) { return o[k]; }
};

// One group: the loaded vectors in[k] = xv[v + k * kThreads], k < VPI -> the pieces
// qp[v + k * kThreads]; only the first `count` pieces are stored.  AMAX: the running packed maximum of the
// vectors is kept in `run` (vectors beyond `count` must be zeros).
template <int DT, int FMT, int PATH, bool NTS, bool AMAX>
__device__ __forceinline__ void cast_group(const u32x4* in, typename Piece<DT>::type* __restrict__ qp,
                                           size_t v, int count, float s, unsigned& run)
{
    constexpr int VPI = DT == FP8_BF16 ? 2 : 4;
    u32x4 item[VPI];
#pragma unroll
    for (int k = 0; k < VPI; ++k) {
        item[k] = in[k];
        if (AMAX) run = vec_mag_max<DT>(item[k], run);
    }
    float y[16];
    scale_item<DT>(item, s, y);
    const u32x4 o = encode16<FMT, PATH>(y);
#pragma unroll
    for (int k = 0; k < VPI; ++k) {
        if (k < count) {
            typename Piece<DT>::type* dst = &qp[v + (size_t)k * kThreads];
            if (NTS) __builtin_nontemporal_store(Piece<DT>::of(o, k), dst); else *dst = Piece<DT>::of(o, k);
        }
    }
}

// A lane's walk over the vectors [vlo, vhi) of its workgroup: 8 vectors per step, all loads of a
// step issued before the first conversion; then the remainder, group by group.
template <int DT, int FMT, int PATH, bool NTS, bool AMAX>
__device__ __forceinline__ void cast_run(const u32x4* __restrict__ xv, typename Piece<DT>::type* __restrict__ qp,
                                         size_t vlo, size_t vhi, float s, unsigned& run)
{
    constexpr int VPI = DT == FP8_BF16 ? 2 : 4;
    size_t v = vlo + threadIdx.x;
    for (; v + 7 * kThreads < vhi; v += 8 * kThreads) {
        u32x4 in[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) in[k] = __builtin_nontemporal_load(&xv[v + (size_t)k * kThreads]);
#pragma unroll
        for (int g = 0; g < 8 / VPI; ++g)
            cast_group<DT, FMT, PATH, NTS, AMAX>(in + g * VPI, qp, v + (size_t)g * VPI * kThreads, VPI, s, run);
    }
    for (; v < vhi; v += VPI * kThreads) {
        const size_t left = (vhi - v + kThreads - 1) / kThreads;        // vectors of this lane still there
        const int count = left < (size_t)VPI ? (int)left : VPI;
        u32x4 in[VPI];
#pragma unroll
        for (int k = 0; k < VPI; ++k)
            in[k] = k < count ? __builtin_nontemporal_load(&xv[v + (size_t)k * kThreads]) : (u32x4){0u, 0u, 0u, 0u};
        cast_group<DT, FMT, PATH, NTS, AMAX>(in, qp, v, count, s, run);
    }
}

inline int grid_for(size_t work_items, int max_blocks)
{
    size_t b = (work_items + kThreads - 1) / kThreads;
    if (b < 1) b = 1;
    if (b > (size_t)max_blocks) b = max_blocks;
    return (int)b;
}

inline bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

}  // namespace
}  // namespace fp8mm
