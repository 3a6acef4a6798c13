// Pieces shared by the translation units of the amax / cast kernels (gfx950).
#pragma once

#include "common.hpp"
#include "fp8_decode.hpp"
#include "fp8_encode.hpp"

namespace fp8mm {
namespace {

constexpr int kThreads = 256;
constexpr int kAmaxBlocks = 256 * 4;      // read-only stream: 32 KB chunks dealt to this many workgroups measured best
constexpr int kCastBlocks = 256 * 64;     // read+write stream: many short contiguous chunks measured best

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
