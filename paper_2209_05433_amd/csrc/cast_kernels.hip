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

// Last step of the amax kernels in their one-launch form (fp8_amax_scale): no cell has to be
// cleared beforehand and the scale comes out of the same launch.  Every workgroup leaves its
// maximum in the workspace and takes a ticket; the workgroup that draws the last ticket reduces the
// gridDim.x partial maxima, writes amax and scale = fmt_max / amax.  Tickets are drawn in two levels
// (groups of kTicketGroup workgroups, then one ticket per group): a thousand workgroups that finish
// together and draw from one counter queue up at that counter for longer than small tensors take
// to read.  Every counter is put back to 0 by the workgroup that drew its last ticket.
// Workspace words: [0] top counter; [32 (1 + g)] counter of group g (one 128-byte line each);
// [kTicketPartials + b] partial maximum of workgroup b.
// Ordering: the partial maximum is stored with an agent-scope atomic store (written through to where
// every other workgroup sees it) and has been acknowledged (vmcnt) before the ticket is drawn; the
// reader draws the last ticket before it loads, again with agent-scope atomic loads.  No other
// data is exchanged, so no cache-wide write-back or invalidate is needed.
// r: the workgroup's maximum, valid in thread 0.
constexpr unsigned kTicketGroup = 32;
constexpr unsigned kTicketPartials = 32 * (1 + kAmaxBlocks / kTicketGroup);

__device__ __forceinline__ unsigned draw_ticket(unsigned* counter)
{
    return __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// bid, grid: the workgroup's number and the number of workgroups that work on this tensor.
__device__ __forceinline__ void amax_finish_ticket(unsigned r, unsigned* __restrict__ ws, int fmt,
                                                   float* __restrict__ amax_out, float* __restrict__ scale_out,
                                                   unsigned bid, unsigned grid)
{
    __shared__ bool last;
    if (threadIdx.x == 0) {
        __hip_atomic_store(&ws[kTicketPartials + bid], r, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __atomic_signal_fence(__ATOMIC_SEQ_CST);            // (the compiler keeps the three steps in this order)
        __builtin_amdgcn_s_waitcnt(0x0070);                 // vmcnt(0) (and lgkmcnt(0)): the store has been acknowledged
        __atomic_signal_fence(__ATOMIC_SEQ_CST);
        const unsigned g = bid / kTicketGroup, groups = (grid + kTicketGroup - 1) / kTicketGroup;
        const unsigned members = min(kTicketGroup, grid - g * kTicketGroup);
        bool l = false;
        if (draw_ticket(&ws[32 * (1 + g)]) == members - 1) {
            __hip_atomic_store(&ws[32 * (1 + g)], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            l = draw_ticket(&ws[0]) == groups - 1;
        }
        last = l;
    }
    __syncthreads();
    if (!last) return;
    unsigned m = 0;
    for (unsigned i = threadIdx.x; i < grid; i += kThreads) {
        const unsigned p = __hip_atomic_load(&ws[kTicketPartials + i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        m = m > p ? m : p;
    }
    m = block_max_u32(m);
    if (threadIdx.x == 0) {
        const float a = as_f32(m);
        *amax_out = a;
        if (scale_out) *scale_out = scale_rule(a, fmt);
        __hip_atomic_store(&ws[0], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// The work of workgroup `bid` of `grid` on one tensor.
template <int DT, bool TICKET>
__device__ __forceinline__ void amax_vec_body(const void* __restrict__ x, size_t n, unsigned* __restrict__ out_bits,
                                              unsigned* __restrict__ ws, int fmt, float* __restrict__ scale_out,
                                              unsigned bid, unsigned grid)
{
    constexpr int PV = Elem<DT>::per_vec;
    const u32x4* xv = (const u32x4*)x;
    const size_t nvec = n / PV;
    const size_t nchunk = nvec / kAmaxChunkVecs;
    unsigned run[4] = {0u, 0u, 0u, 0u};
    for (size_t c = bid; c < nchunk; c += grid) {
        const u32x4* p = xv + c * kAmaxChunkVecs + threadIdx.x;
        u32x4 v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = __builtin_nontemporal_load(p + j * kThreads);
#pragma unroll
        for (int j = 0; j < 8; ++j) run[j & 3] = vec_mag_max<DT>(v[j], run[j & 3]);
    }
    // vectors after the last whole chunk, then the tail elements: workgroup 0
    if (bid == 0) {
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
    if (bid == 0) {
        size_t t = nvec * PV + threadIdx.x;
        if (t < n) {
            unsigned m = scalar_mag<DT>(x, t);
            r = r > m ? r : m;
        }
    }
    r = block_max_u32(r);
    if (TICKET) {
        __syncthreads();                                    // block_max_u32's LDS cells are used again below
        amax_finish_ticket(r, ws, fmt, (float*)out_bits, scale_out, bid, grid);
        return;
    }
    // most workgroups find the cell already large enough and skip the atomic
    if (threadIdx.x == 0 && r > __hip_atomic_load(out_bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(out_bits, r);
}

template <int DT, bool TICKET>
__global__ __launch_bounds__(kThreads) void amax_vec_kernel(const void* __restrict__ x, size_t n,
                                                           unsigned* __restrict__ out_bits, unsigned* __restrict__ ws,
                                                           int fmt, float* __restrict__ scale_out)
{
    amax_vec_body<DT, TICKET>(x, n, out_bits, ws, fmt, scale_out, blockIdx.x, gridDim.x);
}

// Up to kMultiMax tensors in one launch (fp8_amax_scale_multi): the grid is the concatenation of the
// grids the single-tensor launches would use; tensor t has the workgroups first[t] .. first[t + 1] - 1,
// its own 4096 words of workspace, and cells t of amax_out / scale_out.
struct MultiTensors {
    const void* x[kMultiMax];
    uint8_t* q[kMultiMax];
    size_t n[kMultiMax];
    int fmt[kMultiMax];
    unsigned first[kMultiMax + 1];
    int count;
};

__device__ __forceinline__ int multi_find(const MultiTensors& m, unsigned b)
{
    int t = 0;
#pragma unroll
    for (int i = 1; i < kMultiMax; ++i)
        if (i < m.count && b >= m.first[i]) t = i;
    return t;
}

template <int DT>
__global__ __launch_bounds__(kThreads) void amax_multi_kernel(MultiTensors m, float* __restrict__ amax_out,
                                                             float* __restrict__ scale_out, unsigned* __restrict__ ws)
{
    const int t = multi_find(m, blockIdx.x);
    amax_vec_body<DT, true>(m.x[t], m.n[t], (unsigned*)(amax_out + t), ws + (size_t)t * (FP8_AMAX_WORKSPACE_BYTES / 4), m.fmt[t],
                            scale_out ? scale_out + t : nullptr, blockIdx.x - m.first[t], m.first[t + 1] - m.first[t]);
}

// Any alignment the element type allows: one element per lane per step.
template <int DT, bool TICKET>
__global__ __launch_bounds__(kThreads) void amax_scalar_kernel(const void* __restrict__ x, size_t n,
                                                              unsigned* __restrict__ out_bits, unsigned* __restrict__ ws,
                                                              int fmt, float* __restrict__ scale_out)
{
    const size_t stride = (size_t)gridDim.x * kThreads;
    unsigned r = 0;
    for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride) {
        unsigned m = scalar_mag<DT>(x, i);
        r = r > m ? r : m;
    }
    r = block_max_u32(r);
    if (TICKET) {
        __syncthreads();
        amax_finish_ticket(r, ws, fmt, (float*)out_bits, scale_out, blockIdx.x, gridDim.x);
        return;
    }
    if (threadIdx.x == 0) atomicMax(out_bits, r);
}

// n == 0 in the one-launch form: amax 0, scale by the degenerate rule.
__global__ void amax_empty_kernel(int fmt, float* __restrict__ amax_out, float* __restrict__ scale_out)
{
    *amax_out = 0.0f;
    if (scale_out) *scale_out = scale_rule(0.0f, fmt);
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

// Vector path: x and q are 16-byte aligned.  Every workgroup owns one contiguous run of the
// tensor (see cast_run / cast_group for how its lanes share the work).  Stores are ordinary up to
// kStreamingStoreBytes of output, where they win 5 % because part of the output stays in the
// 256 MB memory-side cache, and non-temporal beyond (5-8 % better there).
template <int DT, int FMT, int PATH, bool NTS>
__device__ __forceinline__ void quantize_vec_body(const void* __restrict__ x, size_t n, float s, uint8_t* __restrict__ q,
                                                  unsigned bid, unsigned grid)
{
    constexpr int VPI = DT == FP8_BF16 ? 2 : 4;     // 16-byte vectors per 16 elements
    const size_t nitem = n / 16;
    const size_t per = (nitem + grid - 1) / grid;
    const size_t lo = (size_t)bid * per;
    const size_t hi = lo + per < nitem ? lo + per : nitem;
    unsigned unused = 0;
    if (lo < hi)
        cast_run<DT, FMT, PATH, NTS, false>((const u32x4*)x, (typename Piece<DT>::type*)q, VPI * lo, VPI * hi, s, unused);
    if (bid == 0) {                                 // fewer than 16 tail elements
        const size_t t = nitem * 16 + threadIdx.x;
        if (t < n) q[t] = (uint8_t)encode_bits<FMT, PATH != kCastBitsStrict>(load_scalar<DT>(x, t) * s);
    }
}

template <int DT, int FMT, int PATH, bool NTS>
__global__ __launch_bounds__(kThreads) void quantize_vec_kernel(const void* __restrict__ x, size_t n,
                                                               float scale,
                                                               const float* __restrict__ scale_dev,
                                                               uint8_t* __restrict__ q)
{
    quantize_vec_body<DT, FMT, PATH, NTS>(x, n, scale_dev ? *scale_dev : scale, q, blockIdx.x, gridDim.x);
}

// Up to kMultiMax tensors in one launch (fp8_quantize_multi), grid as for amax_multi_kernel; tensor t is
// cast with scale_dev[t] to format fmt[t].
template <int DT, int PATH>
__global__ __launch_bounds__(kThreads) void quantize_multi_kernel(MultiTensors m, const float* __restrict__ scale_dev)
{
    const int t = multi_find(m, blockIdx.x);
    const unsigned bid = blockIdx.x - m.first[t], grid = m.first[t + 1] - m.first[t];
    if (m.fmt[t] == FP8_E4M3) quantize_vec_body<DT, FP8_E4M3, PATH, false>(m.x[t], m.n[t], scale_dev[t], m.q[t], bid, grid);
    else quantize_vec_body<DT, FP8_E5M2, PATH, false>(m.x[t], m.n[t], scale_dev[t], m.q[t], bid, grid);
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

namespace {
// ws == nullptr: amax_out was cleared by the caller, workgroups raise it with atomics.
// ws != nullptr: the one-launch form (see amax_finish_ticket); grids stay within kAmaxWorkgroupsMax.
template <bool TICKET>
void launch_amax_kernels(const void* x, size_t n, int in_dtype, unsigned* out, unsigned* ws, int fmt, float* scale_out,
                         hipStream_t stream)
{
    if (aligned16(x)) {
        const size_t per_vec = in_dtype == FP8_F32 ? 4 : 8;
        const size_t nchunk = n / per_vec / kAmaxChunkVecs;
        const int grid = (int)(nchunk < 1 ? 1 : nchunk > (size_t)kAmaxBlocks ? (size_t)kAmaxBlocks : nchunk);
        if (in_dtype == FP8_F32)
            hipLaunchKernelGGL((amax_vec_kernel<FP8_F32, TICKET>), dim3(grid), dim3(kThreads), 0, stream, x, n, out, ws, fmt, scale_out);
        else
            hipLaunchKernelGGL((amax_vec_kernel<FP8_BF16, TICKET>), dim3(grid), dim3(kThreads), 0, stream, x, n, out, ws, fmt, scale_out);
    } else {
        const int grid = grid_for(n, kAmaxBlocks);
        if (in_dtype == FP8_F32)
            hipLaunchKernelGGL((amax_scalar_kernel<FP8_F32, TICKET>), dim3(grid), dim3(kThreads), 0, stream, x, n, out, ws, fmt, scale_out);
        else
            hipLaunchKernelGGL((amax_scalar_kernel<FP8_BF16, TICKET>), dim3(grid), dim3(kThreads), 0, stream, x, n, out, ws, fmt, scale_out);
    }
}
}  // namespace

int launch_amax(const void* x, size_t n, int in_dtype, float* amax_out, hipStream_t stream)
{
    unsigned* out = (unsigned*)amax_out;
    hipLaunchKernelGGL(store_u32_kernel, dim3(1), dim3(1), 0, stream, out, 0u);
    if (n == 0) return check_launch("amax init");
    launch_amax_kernels<false>(x, n, in_dtype, out, nullptr, 0, nullptr, stream);
    return check_launch("amax");
}

int launch_amax_scale(const void* x, size_t n, int in_dtype, int fmt, float* amax_out, float* scale_out, void* workspace,
                      hipStream_t stream)
{
    static_assert((kTicketPartials + kAmaxBlocks) * sizeof(unsigned) <= FP8_AMAX_WORKSPACE_BYTES, "counters + one partial per workgroup");
    if (n == 0) hipLaunchKernelGGL(amax_empty_kernel, dim3(1), dim3(1), 0, stream, fmt, amax_out, scale_out);
    else launch_amax_kernels<true>(x, n, in_dtype, (unsigned*)amax_out, (unsigned*)workspace, fmt, scale_out, stream);
    return check_launch("amax_scale");
}

// One launch where every tensor takes the vector path (non-empty, 16-byte aligned); tensor by tensor
// otherwise.  Results are those of the single-tensor launches either way.
int launch_amax_scale_multi(int count, const void* const* x, const size_t* n, int in_dtype, const int* fmt, float* amax_out,
                            float* scale_out, void* workspace, hipStream_t stream)
{
    bool one = count > 1;
    for (int i = 0; i < count; ++i) one = one && n[i] > 0 && aligned16(x[i]);
    if (!one) {
        for (int i = 0; i < count; ++i)
            if (int e = launch_amax_scale(x[i], n[i], in_dtype, fmt[i], amax_out + i, scale_out ? scale_out + i : nullptr,
                                          (char*)workspace + (size_t)i * FP8_AMAX_WORKSPACE_BYTES, stream))
                return e;
        return FP8_OK;
    }
    MultiTensors m{};
    m.count = count;
    unsigned total = 0;
    const size_t per_vec = in_dtype == FP8_F32 ? 4 : 8;
    for (int i = 0; i < count; ++i) {
        const size_t nchunk = n[i] / per_vec / kAmaxChunkVecs;
        m.x[i] = x[i]; m.n[i] = n[i]; m.fmt[i] = fmt[i]; m.first[i] = total;
        total += (unsigned)(nchunk < 1 ? 1 : nchunk > (size_t)kAmaxBlocks ? (size_t)kAmaxBlocks : nchunk);
    }
    for (int i = count; i <= kMultiMax; ++i) m.first[i] = total;
    if (in_dtype == FP8_F32)
        hipLaunchKernelGGL(amax_multi_kernel<FP8_F32>, dim3(total), dim3(kThreads), 0, stream, m, amax_out, scale_out, (unsigned*)workspace);
    else
        hipLaunchKernelGGL(amax_multi_kernel<FP8_BF16>, dim3(total), dim3(kThreads), 0, stream, m, amax_out, scale_out, (unsigned*)workspace);
    return check_launch("amax_scale_multi");
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
        const size_t per_lane = knob(FP8_KNOB_CAST_RUN) ? (size_t)knob(FP8_KNOB_CAST_RUN) : 4;    // items of 16 elements per lane
        const int grid = grid_for((n / 16 + per_lane - 1) / per_lane, kCastBlocks);
        // An output that does not fit the memory-side cache (256 MB) is written past it.
        const bool nts = n >= kStreamingStoreBytes;
#define FP8MM_LAUNCH_QV(PATH)                                                                                      \
    do {                                                                                                           \
        if (nts) hipLaunchKernelGGL((quantize_vec_kernel<DT, FMT, PATH, true>), dim3(grid), dim3(kThreads), 0,     \
                                    stream, x, n, scale, scale_dev, q);                                            \
        else hipLaunchKernelGGL((quantize_vec_kernel<DT, FMT, PATH, false>), dim3(grid), dim3(kThreads), 0,        \
                                stream, x, n, scale, scale_dev, q);                                                \
    } while (0)
        if (!saturate) FP8MM_LAUNCH_QV(kCastBitsStrict);
        else if (cast_path() == kCastCvt) FP8MM_LAUNCH_QV(kCastCvt);
        else FP8MM_LAUNCH_QV(kCastBits);
#undef FP8MM_LAUNCH_QV
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
    // The result depends on the byte alone: every workgroup first tabulates the 256 results (one
    // decode, one IEEE division and, for bf16, one rounding per thread) in LDS, then streams.  With
    // the arithmetic done per element the kernel was bound by the vector ALU at 3.2 TB/s.
    // A lane takes the 8 (bf16 out) or 4 (fp32 out) bytes that make one 16-byte output vector, so that
    // the load and the store instruction of a wave both cover consecutive bytes.
    constexpr int EPV = OUT == FP8_F32 ? 4 : 8;
    constexpr int U = 4;                            // vectors per lane in flight
    static_assert(kThreads == 256, "one table entry per thread");
    __shared__ unsigned table[256];                 // fp32 bits, or bf16 bits in the low half
    {
        const float y = decode_fp8<FMT>(threadIdx.x) / (scale_dev ? *scale_dev : scale);
        table[threadIdx.x] = OUT == FP8_F32 ? as_u32(y) : to_bf16_bits(y);
    }
    __syncthreads();
    const size_t stride = (size_t)gridDim.x * kThreads;
    const size_t nvec = vec ? n / EPV : 0;
    auto load_piece = [&](size_t i) {
        if (OUT == FP8_F32) return (u32x2){__builtin_nontemporal_load(&((const unsigned*)q)[i]), 0u};
        return __builtin_nontemporal_load(&((const u32x2*)q)[i]);
    };
    auto emit = [&](size_t i, u32x2 p) {
        unsigned r[EPV];
#pragma unroll
        for (int e = 0; e < EPV; ++e) r[e] = table[(p[e >> 2] >> (8 * (e & 3))) & 0xffu];
        u32x4 o;
        if constexpr (OUT == FP8_F32) {
            o = (u32x4){r[0], r[1], r[2], r[3]};
        } else {
#pragma unroll
            for (int d = 0; d < 4; ++d) o[d] = r[2 * d] | (r[2 * d + 1] << 16);
        }
        ((u32x4*)out)[i] = o;
    };
    // every workgroup owns one contiguous run of the vectors
    const size_t per = (nvec + gridDim.x - 1) / gridDim.x;
    const size_t lo = (size_t)blockIdx.x * per;
    const size_t hi = lo + per < nvec ? lo + per : nvec;
    size_t i = lo + threadIdx.x;
    for (; i + (U - 1) * kThreads < hi; i += U * kThreads) {
        u32x2 p[U];
#pragma unroll
        for (int u = 0; u < U; ++u) p[u] = load_piece(i + u * kThreads);
#pragma unroll
        for (int u = 0; u < U; ++u) emit(i + u * kThreads, p[u]);
    }
    for (; i < hi; i += kThreads) emit(i, load_piece(i));
    for (size_t t = nvec * EPV + (size_t)blockIdx.x * kThreads + threadIdx.x; t < n; t += stride) {
        if (OUT == FP8_F32) ((unsigned*)out)[t] = table[q[t]];
        else ((unsigned short*)out)[t] = (unsigned short)table[q[t]];
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
    const int grid = grid_for(vec ? n / 16 + 1 : n, 256 * 256);     // many short runs measured best (write-heavy stream)
    if (fmt == FP8_E4M3) {
        if (out_dtype == FP8_F32) hipLaunchKernelGGL((dequantize_kernel<FP8_E4M3, FP8_F32>), dim3(grid), dim3(kThreads), 0, stream, q, n, scale, scale_dev, out, vec);
        else hipLaunchKernelGGL((dequantize_kernel<FP8_E4M3, FP8_BF16>), dim3(grid), dim3(kThreads), 0, stream, q, n, scale, scale_dev, out, vec);
    } else {
        if (out_dtype == FP8_F32) hipLaunchKernelGGL((dequantize_kernel<FP8_E5M2, FP8_F32>), dim3(grid), dim3(kThreads), 0, stream, q, n, scale, scale_dev, out, vec);
        else hipLaunchKernelGGL((dequantize_kernel<FP8_E5M2, FP8_BF16>), dim3(grid), dim3(kThreads), 0, stream, q, n, scale, scale_dev, out, vec);
    }
    return check_launch("dequantize");
}

int launch_quantize_multi(int count, const void* const* x, const size_t* n, int in_dtype, const int* fmt,
                          const float* scale_dev, uint8_t* const* q_out, hipStream_t stream)
{
    // one launch where every tensor takes the vector path with ordinary stores; else tensor by tensor
    bool one = count > 1;
    for (int i = 0; i < count; ++i) one = one && n[i] > 0 && n[i] < kStreamingStoreBytes && aligned16(x[i]) && aligned16(q_out[i]);
    if (!one) {
        for (int i = 0; i < count; ++i)
            if (int e = launch_quantize(x[i], n[i], in_dtype, fmt[i], 0.0f, scale_dev + i, true, q_out[i], stream)) return e;
        return FP8_OK;
    }
    MultiTensors m{};
    m.count = count;
    unsigned total = 0;
    const size_t per_lane = knob(FP8_KNOB_CAST_RUN) ? (size_t)knob(FP8_KNOB_CAST_RUN) : 4;
    for (int i = 0; i < count; ++i) {
        m.x[i] = x[i]; m.q[i] = q_out[i]; m.n[i] = n[i]; m.fmt[i] = fmt[i]; m.first[i] = total;
        total += (unsigned)grid_for((n[i] / 16 + per_lane - 1) / per_lane, kCastBlocks);
    }
    for (int i = count; i <= kMultiMax; ++i) m.first[i] = total;
    const bool cvt = cast_path() == kCastCvt;
    if (in_dtype == FP8_F32) {
        if (cvt) hipLaunchKernelGGL((quantize_multi_kernel<FP8_F32, kCastCvt>), dim3(total), dim3(kThreads), 0, stream, m, scale_dev);
        else hipLaunchKernelGGL((quantize_multi_kernel<FP8_F32, kCastBits>), dim3(total), dim3(kThreads), 0, stream, m, scale_dev);
    } else {
        if (cvt) hipLaunchKernelGGL((quantize_multi_kernel<FP8_BF16, kCastCvt>), dim3(total), dim3(kThreads), 0, stream, m, scale_dev);
        else hipLaunchKernelGGL((quantize_multi_kernel<FP8_BF16, kCastBits>), dim3(total), dim3(kThreads), 0, stream, m, scale_dev);
    }
    return check_launch("quantize_multi");
}

}  // namespace fp8mm
