// amax reduction, scale computation and the FP8 cast for gfx950 (MI355X).
//
// All three are HBM-streaming kernels: every lane moves 16-byte vectors, the arithmetic per
// element is a handful of VALU instructions.  The paper's scheme (arXiv 2209.05433,
// Section 2) is: find the largest magnitude of the tensor, pick scale = fmt_max / amax,
// multiply every element by the scale and round it to E4M3 / E5M2 (Table 1) with
// saturation.
#include "common.hpp"
#include "fp8_decode.hpp"
#include "fp8_encode.hpp"
#include "cast_common.hpp"

namespace fp8mm {
namespace {

// Vector path: x is 16-byte aligned.  nvec full vectors, then n - nvec*per_vec tail elements.
// Every workgroup takes whole chunks of 32 KB (8 vectors per lane, all loaded before the first
// compare), four workgroups per compute unit; one atomic per workgroup at the end (with one chunk
// per workgroup the thousands of atomics on one cell cost a quarter of the run time).
constexpr int kAmaxChunkVecs = kThreads * 8;

template <int DT>
__global__ __launch_bounds__(kThreads) void amax_vec_kernel(const void* __restrict__ x, size_t n,
                                                           unsigned* __restrict__ out_bits)
{
    constexpr int PV = Elem<DT>::per_vec;
    const u32x4* xv = (const u32x4*)x;
    const size_t nvec = n / PV;
    const size_t nchunk = nvec / kAmaxChunkVecs;
    unsigned run[4] = {0u, 0u, 0u, 0u};
    for (size_t c = blockIdx.x; c < nchunk; c += gridDim.x) {
        const u32x4* p = xv + c * kAmaxChunkVecs + threadIdx.x;
        u32x4 v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = __builtin_nontemporal_load(p + j * kThreads);
#pragma unroll
        for (int j = 0; j < 8; ++j) run[j & 3] = vec_mag_max<DT>(v[j], run[j & 3]);
    }
    // vectors after the last whole chunk, then the tail elements: workgroup 0
    if (blockIdx.x == 0) {
        for (size_t i = nchunk * kAmaxChunkVecs + threadIdx.x; i < nvec; i += kThreads)
            run[0] = vec_mag_max<DT>(__builtin_nontemporal_load(&xv[i]), run[0]);
    }
    unsigned r;
    if (DT == FP8_F32) {
        const unsigned a = run[0] > run[1] ? run[0] : run[1], b = run[2] > run[3] ? run[2] : run[3];
        r = a > b ? a : b;
    } else {
        u16x2 p = __builtin_elementwise_max(
            __builtin_elementwise_max(__builtin_bit_cast(u16x2, run[0]), __builtin_bit_cast(u16x2, run[1])),
            __builtin_elementwise_max(__builtin_bit_cast(u16x2, run[2]), __builtin_bit_cast(u16x2, run[3])));
        unsigned short m = p.x > p.y ? p.x : p.y;
        r = (unsigned)m << 16;
    }
    if (blockIdx.x == 0) {
        size_t t = nvec * PV + threadIdx.x;
        if (t < n) {
            unsigned m = scalar_mag<DT>(x, t);
            r = r > m ? r : m;
        }
    }
    r = block_max_u32(r);
    // most workgroups find the cell already large enough and skip the atomic
    if (threadIdx.x == 0 && r > __hip_atomic_load(out_bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(out_bits, r);
}

// Any alignment the element type allows: one element per lane per step.
template <int DT>
__global__ __launch_bounds__(kThreads) void amax_scalar_kernel(const void* __restrict__ x, size_t n,
                                                              unsigned* __restrict__ out_bits)
{
    const size_t stride = (size_t)gridDim.x * kThreads;
    unsigned r = 0;
    for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride) {
        unsigned m = scalar_mag<DT>(x, i);
        r = r > m ? r : m;
    }
    r = block_max_u32(r);
    if (threadIdx.x == 0) atomicMax(out_bits, r);
}

__global__ void scale_kernel(const float* __restrict__ amax, int fmt, float* __restrict__ out)
{
    *out = scale_rule(*amax, fmt);
}

// ------------------------------------------------------------------------------------------
// The cast.  y = fl32(x * scale) is one IEEE multiply; then y is rounded to the nearest
// FP8 value, ties to the even code (Table 1 encodings), finite overflow saturates to the
// largest finite value (Section 2), NaN -> NaN, inf -> NaN (E4M3) or inf (E5M2).
// ------------------------------------------------------------------------------------------

// Vector path: x and q are 16-byte aligned.  A work item is 16 consecutive elements:
// 2 (bf16) or 4 (fp32) non-temporal 16-byte loads and one ordinary 16-byte store per lane
// (measured: non-temporal stores cost about 15 % of the write bandwidth, non-temporal loads gain).
// Every workgroup owns one contiguous run of items and walks it U x 4 KB of output at a time;
// all loads of a step are issued before the first conversion.
template <int DT, int FMT, int PATH>
__global__ __launch_bounds__(kThreads) void quantize_vec_kernel(const void* __restrict__ x, size_t n,
                                                               float scale,
                                                               const float* __restrict__ scale_dev,
                                                               uint8_t* __restrict__ q)
{
    constexpr int V = DT == FP8_BF16 ? 2 : 4;       // 16-byte vectors per item
    constexpr int U = DT == FP8_BF16 ? 4 : 2;       // items per lane per step
    const float s = scale_dev ? *scale_dev : scale;
    const u32x4* xv = (const u32x4*)x;
    u32x4* qv = (u32x4*)q;
    const size_t nitem = n / 16;
    const size_t per = (nitem + gridDim.x - 1) / gridDim.x;
    const size_t lo = (size_t)blockIdx.x * per;
    const size_t hi = lo + per < nitem ? lo + per : nitem;
    size_t i = lo + threadIdx.x;
    for (; i + (U - 1) * kThreads < hi; i += U * kThreads) {
        u32x4 v[U][V];
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int j = 0; j < V; ++j) v[u][j] = __builtin_nontemporal_load(&xv[V * (i + u * kThreads) + j]);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float y[16];
            scale_item<DT>(v[u], s, y);
            qv[i + u * kThreads] = encode16<FMT, PATH>(y);
        }
    }
    for (; i < hi; i += kThreads) {
        u32x4 v[V];
#pragma unroll
        for (int j = 0; j < V; ++j) v[j] = __builtin_nontemporal_load(&xv[V * i + j]);
        float y[16];
        scale_item<DT>(v, s, y);
        qv[i] = encode16<FMT, PATH>(y);
    }
    if (blockIdx.x == 0) {                          // fewer than 16 tail elements
        const size_t t = nitem * 16 + threadIdx.x;
        if (t < n) q[t] = (uint8_t)encode_bits<FMT, PATH != kCastBitsStrict>(load_scalar<DT>(x, t) * s);
    }
}

// Any alignment: one element per lane per step, always the integer rounding.
template <int DT, int FMT, bool SAT>
__global__ __launch_bounds__(kThreads) void quantize_scalar_kernel(const void* __restrict__ x, size_t n,
                                                                  float scale,
                                                                  const float* __restrict__ scale_dev,
                                                                  uint8_t* __restrict__ q)
{
    const float s = scale_dev ? *scale_dev : scale;
    const size_t stride = (size_t)gridDim.x * kThreads;
    for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride)
        q[i] = (uint8_t)encode_bits<FMT, SAT>(load_scalar<DT>(x, i) * s);
}

}  // namespace

int launch_amax(const void* x, size_t n, int in_dtype, float* amax_out, hipStream_t stream)
{
    unsigned* out = (unsigned*)amax_out;
    hipLaunchKernelGGL(store_u32_kernel, dim3(1), dim3(1), 0, stream, out, 0u);
    if (n == 0) return check_launch("amax init");
    if (aligned16(x)) {
        const size_t per_vec = in_dtype == FP8_F32 ? 4 : 8;
        const size_t nchunk = n / per_vec / kAmaxChunkVecs;
        const int grid = (int)(nchunk < 1 ? 1 : nchunk > (size_t)kAmaxBlocks ? (size_t)kAmaxBlocks : nchunk);
        if (in_dtype == FP8_F32)
            hipLaunchKernelGGL(amax_vec_kernel<FP8_F32>, dim3(grid), dim3(kThreads), 0, stream, x, n, out);
        else
            hipLaunchKernelGGL(amax_vec_kernel<FP8_BF16>, dim3(grid), dim3(kThreads), 0, stream, x, n, out);
    } else {
        const int grid = grid_for(n, 2048);
        if (in_dtype == FP8_F32)
            hipLaunchKernelGGL(amax_scalar_kernel<FP8_F32>, dim3(grid), dim3(kThreads), 0, stream, x, n, out);
        else
            hipLaunchKernelGGL(amax_scalar_kernel<FP8_BF16>, dim3(grid), dim3(kThreads), 0, stream, x, n, out);
    }
    return check_launch("amax");
}

float scale_from_amax_host(float amax, int fmt) { return scale_rule(amax, fmt); }

int launch_scale_from_amax(const float* amax, int fmt, float* scale_out, hipStream_t stream)
{
    hipLaunchKernelGGL(scale_kernel, dim3(1), dim3(1), 0, stream, amax, fmt, scale_out);
    return check_launch("scale_from_amax");
}

namespace {
template <int DT, int FMT>
void launch_quantize_typed(const void* x, size_t n, float scale, const float* scale_dev,
                           uint8_t* q, bool saturate, hipStream_t stream)
{
    if (aligned16(x) && aligned16(q)) {
        const int grid = grid_for((n / 16 + 3) / 4, kCastBlocks);
        if (!saturate)
            hipLaunchKernelGGL((quantize_vec_kernel<DT, FMT, kCastBitsStrict>), dim3(grid), dim3(kThreads), 0,
                               stream, x, n, scale, scale_dev, q);
        else if (cast_path() == kCastCvt)
            hipLaunchKernelGGL((quantize_vec_kernel<DT, FMT, kCastCvt>), dim3(grid), dim3(kThreads), 0,
                               stream, x, n, scale, scale_dev, q);
        else
            hipLaunchKernelGGL((quantize_vec_kernel<DT, FMT, kCastBits>), dim3(grid), dim3(kThreads), 0,
                               stream, x, n, scale, scale_dev, q);
    } else if (saturate) {
        hipLaunchKernelGGL((quantize_scalar_kernel<DT, FMT, true>), dim3(grid_for(n, 2048)), dim3(kThreads), 0,
                           stream, x, n, scale, scale_dev, q);
    } else {
        hipLaunchKernelGGL((quantize_scalar_kernel<DT, FMT, false>), dim3(grid_for(n, 2048)), dim3(kThreads), 0,
                           stream, x, n, scale, scale_dev, q);
    }
}

// ------------------------------------------------------------------------------------------
// dequantize: out[i] = fl_out(decode(q[i]) / scale), one IEEE single division per element
// (Section 2: values are unscaled by the inverse of the scaling factor after conversion from
// FP8), then rounding to bf16 if asked.  16 bytes in, 32 or 64 bytes out per lane.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ unsigned to_bf16_bits(float f)
{
    const unsigned u = as_u32(f);
    const unsigned r = (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
    return (u & 0x7fffffffu) > 0x7f800000u ? ((u >> 16) | 0x40u) : r;
}

template <int FMT, int OUT>
__global__ __launch_bounds__(kThreads) void dequantize_kernel(const uint8_t* __restrict__ q, size_t n, float scale,
                                                             const float* __restrict__ scale_dev,
                                                             void* __restrict__ out, bool vec)
{
    const float s = scale_dev ? *scale_dev : scale;
    const size_t stride = (size_t)gridDim.x * kThreads;
    const size_t nitem = vec ? n / 16 : 0;
    for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < nitem; i += stride) {
        const u32x4 v = __builtin_nontemporal_load(&((const u32x4*)q)[i]);
        float y[16];
#pragma unroll
        for (int d = 0; d < 4; ++d)
#pragma unroll
            for (int b = 0; b < 4; ++b) y[4 * d + b] = decode_fp8<FMT>((v[d] >> (8 * b)) & 0xffu) / s;
        if (OUT == FP8_F32) {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                ((u32x4*)out)[4 * i + j] = (u32x4){as_u32(y[4 * j]), as_u32(y[4 * j + 1]), as_u32(y[4 * j + 2]), as_u32(y[4 * j + 3])};
        } else {
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                u32x4 o;
#pragma unroll
                for (int d = 0; d < 4; ++d) o[d] = to_bf16_bits(y[8 * j + 2 * d]) | (to_bf16_bits(y[8 * j + 2 * d + 1]) << 16);
                ((u32x4*)out)[2 * i + j] = o;
            }
        }
    }
    for (size_t t = nitem * 16 + (size_t)blockIdx.x * kThreads + threadIdx.x; t < n; t += stride) {
        const float y = decode_fp8<FMT>(q[t]) / s;
        if (OUT == FP8_F32) ((float*)out)[t] = y;
        else ((unsigned short*)out)[t] = (unsigned short)to_bf16_bits(y);
    }
}
}  // namespace

int launch_quantize(const void* x, size_t n, int in_dtype, int fmt, float scale,
                    const float* scale_dev, bool saturate, uint8_t* q_out, hipStream_t stream)
{
    if (n == 0) return FP8_OK;
    if (in_dtype == FP8_F32) {
        if (fmt == FP8_E4M3) launch_quantize_typed<FP8_F32, FP8_E4M3>(x, n, scale, scale_dev, q_out, saturate, stream);
        else                 launch_quantize_typed<FP8_F32, FP8_E5M2>(x, n, scale, scale_dev, q_out, saturate, stream);
    } else {
        if (fmt == FP8_E4M3) launch_quantize_typed<FP8_BF16, FP8_E4M3>(x, n, scale, scale_dev, q_out, saturate, stream);
        else                 launch_quantize_typed<FP8_BF16, FP8_E5M2>(x, n, scale, scale_dev, q_out, saturate, stream);
    }
    return check_launch("quantize");
}

int launch_dequantize(const uint8_t* q, size_t n, int fmt, float scale, const float* scale_dev,
                      int out_dtype, void* out, hipStream_t stream)
{
    if (n == 0) return FP8_OK;
    const bool vec = aligned16(q) && aligned16(out);
    const int grid = grid_for(vec ? n / 16 + 1 : n, 256 * 16);
    if (fmt == FP8_E4M3) {
        if (out_dtype == FP8_F32) hipLaunchKernelGGL((dequantize_kernel<FP8_E4M3, FP8_F32>), dim3(grid), dim3(kThreads), 0, stream, q, n, scale, scale_dev, out, vec);
        else hipLaunchKernelGGL((dequantize_kernel<FP8_E4M3, FP8_BF16>), dim3(grid), dim3(kThreads), 0, stream, q, n, scale, scale_dev, out, vec);
    } else {
        if (out_dtype == FP8_F32) hipLaunchKernelGGL((dequantize_kernel<FP8_E5M2, FP8_F32>), dim3(grid), dim3(kThreads), 0, stream, q, n, scale, scale_dev, out, vec);
        else hipLaunchKernelGGL((dequantize_kernel<FP8_E5M2, FP8_BF16>), dim3(grid), dim3(kThreads), 0, stream, q, n, scale, scale_dev, out, vec);
    }
    return check_launch("dequantize");
}

}  // namespace fp8mm
