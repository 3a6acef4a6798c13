// Split-K form of the FP8 GEMM for gfx950 (MI355X): problems with few output tiles and a long K
// (the weight gradient dW = dY^T X of a layer, K = tokens) leave most compute units idle when every
// tile is one workgroup.  Here K is cut into slices; every (tile, slice) is one workgroup of the
// tiled kernel, which writes its fp32 sums, without the scales, into slice s of a workspace; a
// second kernel adds the slices in slice order (the same order in every run: results are
// deterministic), takes the scaling factors out once per output (arXiv 2209.05433, Section 2:
// unscaling is applied once per dot product) and converts to the output type.
#include "gemm_common.hpp"

#include <mutex>

namespace fp8mm {
namespace {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v2f __attribute__((ext_vector_type(2)));
typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int kReduceThreads = 256;

// out = cast((ws[0] + ws[1] + ... + ws[splits-1]) * r), r = fl32(1 / (sA sB)), element by element.
// VEC: mn is a multiple of 4 and ws / C are aligned for 16-byte loads and whole-vector stores.
template <int OUT, bool VEC>
__global__ __launch_bounds__(kReduceThreads) void splitk_reduce_kernel(
    const float* __restrict__ ws, size_t mn, int splits, float sA, float sB,
    const float* __restrict__ sA_dev, const float* __restrict__ sB_dev, void* __restrict__ C)
{
    const float r = (float)(1.0 / ((double)scale_value(sA_dev, sA) * (double)scale_value(sB_dev, sB)));
    const size_t stride = (size_t)gridDim.x * kReduceThreads;
    const size_t first = (size_t)blockIdx.x * kReduceThreads + threadIdx.x;
    if (VEC) {
        const size_t nvec = mn / 4;
        for (size_t v = first; v < nvec; v += stride) {
            v4f acc = *(const v4f*)(ws + 4 * v);
            for (int s = 1; s < splits; ++s) {
                const v4f p = *(const v4f*)(ws + (size_t)s * mn + 4 * v);
                acc.x += p.x; acc.y += p.y; acc.z += p.z; acc.w += p.w;
            }
            acc.x *= r; acc.y *= r; acc.z *= r; acc.w *= r;
            if (OUT == OUT_F32) {
                *(v4f*)((float*)C + 4 * v) = acc;
            } else {
                u32x2 o;
                o.x = __builtin_bit_cast(unsigned, __builtin_convertvector((v2f){acc.x, acc.y}, v2bf));
                o.y = __builtin_bit_cast(unsigned, __builtin_convertvector((v2f){acc.z, acc.w}, v2bf));
                *(u32x2*)((unsigned short*)C + 4 * v) = o;
            }
        }
    } else {
        for (size_t i = first; i < mn; i += stride) {
            float acc = ws[i];
            for (int s = 1; s < splits; ++s) acc += ws[(size_t)s * mn + i];
            acc *= r;
            if (OUT == OUT_F32) {
                ((float*)C)[i] = acc;
            } else {
                const v2bf b = __builtin_convertvector((v2f){acc, 0.0f}, v2bf);
                ((unsigned short*)C)[i] = (unsigned short)(__builtin_bit_cast(unsigned, b) & 0xffffu);
            }
        }
    }
}

inline bool aligned_to(const void* p, uintptr_t a) { return ((uintptr_t)p & (a - 1)) == 0; }

}  // namespace

// How a split-K call cuts a problem that the tiled kernel takes.  One round of workgroups (256
// compute units) is the target; a slice is never shorter than 4 stage pairs (512 of K), whose
// prologue and epilogue a shorter slice would not pay for.  requested > 0 forces the count.
SplitPlan plan_splitk(const GemmArgs& g, int requested)
{
    SplitPlan sp{1, 0, 256};
    GemmArgs probe = g;
    const int kernel = plan_gemm(probe).kernel;
    if (kernel != GEMM_TILED_256 && kernel != GEMM_TILED_128 && kernel != GEMM_TILED_MIXED) return sp;
    const int forced_tile = knob(FP8_KNOB_TILE_N);
    sp.tile_n = forced_tile ? forced_tile : 256;             // the slices fill the chip: the wide tile is the faster one
    const int64_t tiles = ((g.M + TILE_M - 1) / TILE_M) * ((g.N + sp.tile_n - 1) / sp.tile_n);
    const int64_t pairs = (g.K + 2 * TILE_K - 1) / (2 * TILE_K);
    int64_t want = requested > 0 ? requested : (tiles >= 256 ? 1 : 256 / tiles);
    if (requested <= 0 && want > pairs / 4) want = pairs / 4;
    if (want > kMaxSplitK) want = kMaxSplitK;
    if (want > pairs) want = pairs;
    if (want < 1) want = 1;
    const int64_t per = (pairs + want - 1) / want;
    sp.pairs_per_split = (int)per;
    sp.splits = (int)((pairs + per - 1) / per);             // every slice holds at least one pair
    return sp;
}

size_t splitk_workspace_bytes(const GemmArgs& g, const SplitPlan& sp)
{
    return sp.splits > 1 ? (size_t)sp.splits * (size_t)g.M * (size_t)g.N * sizeof(float) : 0;
}

// g: the problem with its real output and scales (fp32 / bf16 out, per-tensor scales); ws: workspace
// of at least splitk_workspace_bytes(g, sp) bytes, 4-byte aligned.
int launch_gemm_splitk(const GemmArgs& g, const SplitPlan& sp, void* ws)
{
    if (g.M == 0 || g.N == 0 || g.K == 0 || sp.splits <= 1) return launch_gemm(g);
    GemmArgs part = g;
    part.C = ws;
    part.ep = EpilogueArgs{};
    part.ep.sA = 1.0f; part.ep.sB = 1.0f;                   // the slices carry plain sums
    part.ep.out_kind = OUT_F32;
    part.ep.ragged_n = (g.N % 4 != 0 || !aligned_to(ws, 16)) ? 1 : 0;
    part.tile_n = sp.tile_n;
    part.persist = false;
    part.splits = sp.splits;
    part.pairs_per_split = sp.pairs_per_split;
    if (int e = launch_tiled(part)) return e;

    const size_t mn = (size_t)g.M * (size_t)g.N;
    const bool bf16 = g.ep.out_kind == OUT_BF16;
    const bool vec = mn % 4 == 0 && aligned_to(ws, 16) && aligned_to(g.C, bf16 ? 8 : 16);
    size_t blocks = ((vec ? mn / 4 : mn) + kReduceThreads - 1) / kReduceThreads;
    if (blocks > 65536) blocks = 65536;
    const dim3 grid((unsigned)blocks), block(kReduceThreads);
#define FP8MM_LAUNCH_REDUCE(OUT, VEC)                                                                     \
    hipLaunchKernelGGL((splitk_reduce_kernel<OUT, VEC>), grid, block, 0, g.stream, (const float*)ws, mn,  \
                       sp.splits, g.ep.sA, g.ep.sB, g.ep.sA_dev, g.ep.sB_dev, g.C)
    if (bf16) { if (vec) FP8MM_LAUNCH_REDUCE(OUT_BF16, true); else FP8MM_LAUNCH_REDUCE(OUT_BF16, false); }
    else      { if (vec) FP8MM_LAUNCH_REDUCE(OUT_F32, true);  else FP8MM_LAUNCH_REDUCE(OUT_F32, false); }
#undef FP8MM_LAUNCH_REDUCE
    return check_launch("gemm (split-K reduction)");
}

// ---- the form that allocates nothing ---------------------------------------------------------
// The slices' sums go to a file-scope device array instead of a caller-supplied workspace.  Every
// device the library runs on holds its own copy of the array, at its own address, until the process
// ends.  In host code the array's name is only a handle: its device address comes from
// hipGetSymbolAddress, asked once per device with that device current, and is what kernels get.
namespace {

constexpr size_t kScratchBytes = FP8_SPLITK_STATIC_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices];          // device address of `scratch` on each device, 0 = not asked yet

int scratch_of_current_device(const char* who, void** out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(FP8_ERR_DEVICE, "%s: hipGetDevice: %s", who, hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return fail(FP8_ERR_UNSUPPORTED, "%s: device index %d is beyond %d", who, dev, kMaxDevices - 1);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return fail(FP8_ERR_DEVICE, "%s: hipGetSymbolAddress(scratch) on device %d: %s", who, dev, hipGetErrorString(e));
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return FP8_OK;
}

}  // namespace
}  // namespace fp8mm

using namespace fp8mm;

extern "C" {

size_t fp8_gemm_splitk_workspace_size(int64_t M, int64_t N, int64_t K, int transA, int transB, int splits)
{
    clear_error();
    if (M <= 0 || N <= 0 || K <= 0 || splits < 0 || splits > kMaxSplitK) return 0;
    GemmArgs g{};
    g.M = M; g.N = N; g.K = K; g.transA = transA != 0; g.transB = transB != 0;     // null pointers count as aligned
    const SplitPlan sp = plan_splitk(g, splits ? splits : knob(FP8_KNOB_SPLIT_K));
    return splitk_workspace_bytes(g, sp);
}

int fp8_gemm_splitk(const uint8_t* A, int fmtA, int transA, const uint8_t* B, int fmtB, int transB,
                    void* C, int64_t M, int64_t N, int64_t K, int out_dtype,
                    float sA, float sB, const float* sA_dev, const float* sB_dev, int flags,
                    int splits, void* workspace, size_t workspace_bytes, void* stream)
{
    const char* who = "fp8_gemm_splitk";
    GemmArgs g{};
    if (int e = fill_gemm_args(who, g, A, fmtA, transA, B, fmtB, transB, C, M, N, K, out_dtype, sA, sB, sA_dev, sB_dev,
                               flags, stream))
        return e;
    if (splits < 0 || splits > kMaxSplitK) return fail(FP8_ERR_INVALID_ARG, "%s: splits = %d is not in 0..%d", who, splits, kMaxSplitK);
    if ((uintptr_t)workspace % 4) return fail(FP8_ERR_INVALID_ARG, "%s: workspace is not 4-byte aligned", who);
    if (M == 0 || N == 0 || K == 0) return launch_gemm(g);
    const SplitPlan sp = plan_splitk(g, splits ? splits : knob(FP8_KNOB_SPLIT_K));
    const size_t need = splitk_workspace_bytes(g, sp);
    if (need > 0 && (!workspace || workspace_bytes < need))
        return fail(FP8_ERR_INVALID_ARG, "%s: %d slices of %lld x %lld fp32 sums need a workspace of %zu bytes, %zu given",
                    who, sp.splits, (long long)M, (long long)N, need, workspace ? workspace_bytes : (size_t)0);
    return launch_gemm_splitk(g, sp, workspace);
}

int fp8_gemm_splitk_static(const uint8_t* A, int fmtA, int transA, const uint8_t* B, int fmtB, int transB,
                           void* C, int64_t M, int64_t N, int64_t K, int out_dtype,
                           float sA, float sB, const float* sA_dev, const float* sB_dev, int flags,
                           int splits, void* stream)
{
    const char* who = "fp8_gemm_splitk_static";
    GemmArgs g{};
    if (int e = fill_gemm_args(who, g, A, fmtA, transA, B, fmtB, transB, C, M, N, K, out_dtype, sA, sB, sA_dev, sB_dev,
                               flags, stream))
        return e;
    if (splits < 0 || splits > kMaxSplitK) return fail(FP8_ERR_INVALID_ARG, "%s: splits = %d is not in 0..%d", who, splits, kMaxSplitK);
    if (M == 0 || N == 0 || K == 0) return launch_gemm(g);
    const int requested = splits ? splits : knob(FP8_KNOB_SPLIT_K);
    SplitPlan sp = plan_splitk(g, requested);
    size_t need = splitk_workspace_bytes(g, sp);
    if (need > kScratchBytes) {
        const size_t fit = kScratchBytes / ((size_t)M * (size_t)N * sizeof(float));     // slices the array holds
        if (requested > 0 || fit < 2)
            return fail(FP8_ERR_UNSUPPORTED, "%s: %d slices of %lld x %lld fp32 sums need %zu bytes, the static scratch array holds %zu",
                        who, sp.splits, (long long)M, (long long)N, need, kScratchBytes);
        sp = plan_splitk(g, (int)fit);                       // the library's own choice is cut down to what fits
        need = splitk_workspace_bytes(g, sp);
    }
    void* ws = nullptr;
    if (need > 0)
        if (int e = scratch_of_current_device(who, &ws)) return e;
    return launch_gemm_splitk(g, sp, ws);
}

}  // extern "C"
