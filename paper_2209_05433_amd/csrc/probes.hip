// Measurement probes for gfx950 (MI355X), built into a library of their own (libfp8probes.so): they
// are not part of the product path.  bench.py runs them beside the kernels they put into
// perspective:
//   fp8probe_mfma    a register-only loop of the matrix-core instruction a GEMM mode issues, on
//                    operand bytes taken from real FP8 tensors: what the chip sustains on that
//                    instruction when nothing else (LDS, global loads, barriers) is going on
//   fp8probe_stream  plain streaming kernels (read, write, copy, two reads per write): what the
//                    memory system sustains for the access mix of the amax / cast kernels
// No torch types, plain pointers, status codes as in fp8mm.h (0 = ok, 1 = bad argument, 3 = HIP error).
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef _Float16 v2h __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;           // 4 waves, one per SIMD, as in the tiled GEMM

__device__ __forceinline__ v8h widen8_e4m3(int lo, int hi)
{
    const v2h p0 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8((unsigned)lo, 1.0f, false);
    const v2h p1 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8((unsigned)lo, 1.0f, true);
    const v2h p2 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8((unsigned)hi, 1.0f, false);
    const v2h p3 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8((unsigned)hi, 1.0f, true);
    return (v8h){p0.x, p0.y, p1.x, p1.y, p2.x, p2.y, p3.x, p3.y};
}

// KIND 0: v_mfma_f32_32x32x64_f8f6f4 on E4M3 bytes; KIND 1: the bytes widened to fp16 once, then
// v_mfma_f32_32x32x16_f16.  A wave holds 4 + 4 operand blocks of 32 bytes per lane and 4 x 4
// accumulator blocks (256 registers) and runs `iters` rounds of the 16 block products of one K step
// of 64: 2 * 32 * 32 * 64 * 16 flop per wave and round in either kind.
template <int KIND>
__global__ __launch_bounds__(kThreads, 1) void mfma_loop_kernel(const uint8_t* __restrict__ a_bytes,
                                                              const uint8_t* __restrict__ b_bytes, size_t span,
                                                              int iters, float* __restrict__ out)
{
    const size_t lane = (size_t)blockIdx.x * kThreads + threadIdx.x;
    v8i a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const size_t off = ((lane * 4 + i) * 32) % span;                    // span is a multiple of 32
        a[i] = *(const v8i*)(a_bytes + off);
        b[i] = *(const v8i*)(b_bytes + off);
    }
    v16f acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
    if (KIND == 0) {
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(b[i], a[j], acc[i][j], 0, 0, 0, 0, 0, 0);
        }
    } else {
        v8h ah[4][4], bh[4][4];                                              // [block][K sub-step of 16]
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                ah[i][s] = widen8_e4m3(a[i][2 * s], a[i][2 * s + 1]);
                bh[i][s] = widen8_e4m3(b[i][2 * s], b[i][2 * s + 1]);
            }
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(bh[i][s], ah[j][s], acc[i][j], 0, 0, 0);
        }
    }
    float sum = 0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) sum += acc[i][j][r];
    out[lane] = sum;
}

// MODE 0: read n16 vectors (their XOR goes to dst[workgroup], so that the loads stay);
// MODE 1: write n16 vectors; MODE 2: copy n16 vectors; MODE 3: read 2 n16 vectors, write n16 (the
// mix of the bf16 -> FP8 cast).  Loads and stores are non-temporal 16-byte vectors, a lane's
// consecutive accesses lie kThreads vectors apart, every workgroup owns one contiguous run.
template <int MODE>
__global__ __launch_bounds__(kThreads) void stream_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t n16)
{
    constexpr int U = 8;
    const size_t per = (n16 + gridDim.x - 1) / gridDim.x;
    const size_t lo = (size_t)blockIdx.x * per < n16 ? (size_t)blockIdx.x * per : n16, hi = lo + per < n16 ? lo + per : n16;
    // (MODE 3: the workgroup reads the 2 (hi - lo) vectors from 2 lo on, as two runs of hi - lo)
    u32x4 keep = {0u, 0u, 0u, 0u};
    size_t v = lo + threadIdx.x;
    for (; v + (U - 1) * kThreads < hi; v += U * kThreads) {
        u32x4 x[U], y[U];
#pragma unroll
        for (int k = 0; k < U; ++k) {
            if (MODE == 0 || MODE == 2) x[k] = __builtin_nontemporal_load(&src[v + (size_t)k * kThreads]);
            if (MODE == 3) {
                x[k] = __builtin_nontemporal_load(&src[2 * lo + (v - lo) + (size_t)k * kThreads]);
                y[k] = __builtin_nontemporal_load(&src[2 * lo + (hi - lo) + (v - lo) + (size_t)k * kThreads]);
            }
            if (MODE == 1) x[k] = (u32x4){(unsigned)v, (unsigned)k, 3u, 4u};
        }
#pragma unroll
        for (int k = 0; k < U; ++k) {
            if (MODE == 0) keep ^= x[k];
            if (MODE == 3) x[k] ^= y[k];
            if (MODE != 0) __builtin_nontemporal_store(x[k], &dst[v + (size_t)k * kThreads]);
        }
    }
    for (; v < hi; v += kThreads) {
        u32x4 x = {1u, 2u, 3u, 4u};
        if (MODE == 0 || MODE == 2) x = __builtin_nontemporal_load(&src[v]);
        if (MODE == 3) x = __builtin_nontemporal_load(&src[2 * lo + (v - lo)]) ^ __builtin_nontemporal_load(&src[2 * lo + (hi - lo) + (v - lo)]);
        if (MODE == 0) keep ^= x; else __builtin_nontemporal_store(x, &dst[v]);
    }
    if (MODE == 0) {
        // one vector per workgroup: every lane's value enters through a wave reduction
        unsigned r = keep.x ^ keep.y ^ keep.z ^ keep.w;
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) r ^= (unsigned)__shfl_xor((int)r, d, 64);
        if ((threadIdx.x & 63) == 0) atomicXor(&((unsigned*)dst)[blockIdx.x * 4], r);
    }
}

int status_of_launch()
{
    return hipGetLastError() == hipSuccess ? 0 : 3;
}

}  // namespace

extern "C" {

// kind 0: FP8 instruction, kind 1: fp16 instruction on widened bytes.  a_bytes, b_bytes: device, `span`
// bytes each (a multiple of 32, at least 32) of E4M3 codes; out: device, workgroups * 256 floats.
// Runs workgroups x 4 waves x iters rounds of 16 block products; flop = workgroups * 4 * iters * 2097152.
int fp8probe_mfma(int kind, const uint8_t* a_bytes, const uint8_t* b_bytes, size_t span, int workgroups, int iters,
                  float* out, void* stream)
{
    if ((kind != 0 && kind != 1) || !a_bytes || !b_bytes || !out || span < 32 || span % 32 || workgroups <= 0 || iters < 0 ||
        ((uintptr_t)a_bytes | (uintptr_t)b_bytes) % 32)
        return 1;
    if (kind == 0)
        hipLaunchKernelGGL(mfma_loop_kernel<0>, dim3(workgroups), dim3(kThreads), 0, (hipStream_t)stream, a_bytes, b_bytes, span, iters, out);
    else
        hipLaunchKernelGGL(mfma_loop_kernel<1>, dim3(workgroups), dim3(kThreads), 0, (hipStream_t)stream, a_bytes, b_bytes, span, iters, out);
    return status_of_launch();
}

// mode 0 read, 1 write, 2 copy, 3 two reads per write.  src: device, n16 vectors of 16 bytes (2 n16 for
// mode 3; unused for mode 1); dst: device, n16 vectors (mode 0: at least 16 bytes per workgroup, zeroed by
// the caller).  Bytes moved: n16 * 16 * (1, 1, 2, 3).
int fp8probe_stream(int mode, const void* src, void* dst, size_t n16, int workgroups, void* stream)
{
    if (mode < 0 || mode > 3 || !dst || (mode != 1 && !src) || workgroups <= 0 || ((uintptr_t)src | (uintptr_t)dst) % 16) return 1;
    const dim3 grid(workgroups), block(kThreads);
    hipStream_t s = (hipStream_t)stream;
    switch (mode) {
        case 0: hipLaunchKernelGGL(stream_kernel<0>, grid, block, 0, s, (const u32x4*)src, (u32x4*)dst, n16); break;
        case 1: hipLaunchKernelGGL(stream_kernel<1>, grid, block, 0, s, (const u32x4*)src, (u32x4*)dst, n16); break;
        case 2: hipLaunchKernelGGL(stream_kernel<2>, grid, block, 0, s, (const u32x4*)src, (u32x4*)dst, n16); break;
        default: hipLaunchKernelGGL(stream_kernel<3>, grid, block, 0, s, (const u32x4*)src, (u32x4*)dst, n16); break;
    }
    return status_of_launch();
}

}  // extern "C"
