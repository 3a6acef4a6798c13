// GEMM dispatcher and the generic kernel for gfx950 (MI355X).
//
// Shapes and pointers that meet the tiled kernel's conditions (K a multiple of 16, 16-byte aligned
// operands whose rows start on 16-byte boundaries) go to one of its instances; everything else to the
// matrix-core kernel for any shape (gemm_mfma_any.hip).  The generic kernel below (plain FMAs: any
// shape, any alignment, every storage order, the same epilogue) remains as the independent
// cross-check the tests force through a knob, and for outputs with more tiles than a grid holds
// (arXiv 2209.05433, Section 2: FP8 operands, fp32 accumulation, scales taken out once per output).
#include "gemm_common.hpp"

#include <algorithm>

namespace fp8mm {
namespace {

// fp32 -> bf16 bits, round to nearest even; NaN stays NaN.
__device__ __forceinline__ unsigned bf16_bits(float f)
{
    const unsigned u = as_u32(f);
    const unsigned r = (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
    return (u & 0x7fffffffu) > 0x7f800000u ? ((u >> 16) | 0x40u) : r;
}

// ------------------------------------------------------------------------------------------
// Generic kernel: 64 x 64 tile per 256-thread workgroup, 4 x 4 outputs per thread, operands
// decoded to fp32 (exactly) on their way into LDS, fp32 FMAs (each product of two FP8 values
// is exact in fp32, so this is fp32 accumulation of exact products as well).
// ------------------------------------------------------------------------------------------
constexpr int GT = 64, GK = 16;

template <int FMT_A, int FMT_B>
__global__ __launch_bounds__(256) void gemm_generic_kernel(
    const uint8_t* __restrict__ A, const uint8_t* __restrict__ B, void* __restrict__ C,
    int64_t M, int64_t N, int64_t K, EpilogueArgs ep, bool transA, bool transB)
{
    __shared__ float As[GK][GT + 1];
    __shared__ float Bs[GK][GT + 1];
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    // tiles are numbered row by row in the x dimension of the grid (the y dimension stops at 65 535)
    const int64_t tiles_n = (N + GT - 1) / GT;
    const int64_t m0 = (int64_t)(blockIdx.x / tiles_n) * GT, n0 = (int64_t)(blockIdx.x % tiles_n) * GT;
    float acc[4][4] = {};
    for (int64_t k0 = 0; k0 < K; k0 += GK) {
        for (int e = tid; e < GT * GK; e += 256) {
            const int r = e / GK, kk = e % GK;              // A: consecutive lanes along K
            const int64_t gm = m0 + r, gk = k0 + kk;
            As[kk][r] = (gm < M && gk < K) ? decode_fp8<FMT_A>(A[transA ? gk * M + gm : gm * K + gk]) : 0.0f;
            const int kb = e / GT, c = e % GT;              // B: consecutive lanes along N
            const int64_t gn = n0 + c, gkb = k0 + kb;
            Bs[kb][c] = (gn < N && gkb < K) ? decode_fp8<FMT_B>(B[transB ? gn * K + gkb : gkb * N + gn]) : 0.0f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < GK; ++kk) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
    const float sD = (ep.out_kind >= OUT_E4M3) ? scale_value(ep.sD_dev, 1.0f) : 1.0f;
    unsigned amax_bits = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t gm = m0 + ty * 4 + i, gn = n0 + tx * 4 + j;
            if (gm < M && gn < N) {
                const double a = ep.a_per_row ? (double)ep.sA_dev[gm] : (double)scale_value(ep.sA_dev, ep.sA);
                const double b = ep.b_per_col ? (double)ep.sB_dev[gn] : (double)scale_value(ep.sB_dev, ep.sB);
                const float c = acc[i][j] * (float)(1.0 / (a * b));
                amax_bits = max(amax_bits, as_u32(c) & 0x7fffffffu);
                const int64_t o = gm * N + gn;
                switch (ep.out_kind) {
                    case OUT_F32: ((float*)C)[o] = c; break;
                    case OUT_BF16: ((unsigned short*)C)[o] = (unsigned short)bf16_bits(c); break;
                    case OUT_E4M3: ((uint8_t*)C)[o] = (uint8_t)encode_bits<FP8_E4M3>(c * sD); break;
                    default: ((uint8_t*)C)[o] = (uint8_t)encode_bits<FP8_E5M2>(c * sD); break;
                }
            }
        }
    if (ep.amax_out) wave_amax_commit(amax_bits, ep.amax_out);
}

template <int FA, int FB>
int launch_generic(const GemmArgs& g)
{
    const int64_t tiles = ((g.N + GT - 1) / GT) * ((g.M + GT - 1) / GT);
    if (tiles > 0x7fffffffll)
        return fail(FP8_ERR_UNSUPPORTED, "gemm (generic kernel): %lld tiles of 64 x 64 exceed the grid limit", (long long)tiles);
    const dim3 grid((unsigned)tiles);
    hipLaunchKernelGGL((gemm_generic_kernel<FA, FB>), grid, dim3(256), 0, g.stream, g.A, g.B, g.C, g.M, g.N, g.K,
                       g.ep, g.transA, g.transB);
    return check_launch("gemm (generic kernel)");
}

__global__ void zero_fill_kernel(unsigned char* p, size_t nbytes)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < nbytes; i += stride) p[i] = 0;
}

__global__ void zero_cell_kernel(unsigned* p) { *p = 0u; }

// The knob FP8_KNOB_GEMM_KERNEL = 1 forces the generic kernel, = 2 the any-shape matrix-core kernel.
bool force_generic() { return knob(FP8_KNOB_GEMM_KERNEL) == 1; }
bool force_mfma_any() { return knob(FP8_KNOB_GEMM_KERNEL) == 2; }

inline bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

}  // namespace

// Which kernel a (non-empty, K > 0) problem takes.
GemmPlan plan_gemm(const GemmArgs& g)
{
    const int64_t M = g.M, N = g.N, K = g.K;
    GemmPlan plan{!force_generic() && mfma_any_takes(g) ? GEMM_MFMA_ANY : GEMM_GENERIC, false, false, 0};
    const uint64_t ldmax = (uint64_t)(M > N ? (M > K ? M : K) : (N > K ? N : K));
    const bool fits32 = 256 * ldmax < (1ull << 32) && M < (1ll << 31) - TILE_M && N < (1ll << 31) - TILE_N &&
                        K < (1ll << 31) &&
                        // the grid holds one workgroup per tile: counted with the narrow tile, the larger count
                        ((M + TILE_M - 1) / TILE_M) * ((N + TILE_N / 2 - 1) / (TILE_N / 2)) < (1ll << 31);
    // The tiled kernel works on 256 x 256 tiles and clips the last ones: loads of rows / columns
    // beyond the edge are redirected to existing ones and their outputs are not stored.  What it
    // needs: K a multiple of 16 (it walks K in pairs of stages of 64 and fills a last, partial pair
    // up with zeros; rows of a K-contiguous operand start every K bytes); 16-byte aligned operands;
    // rows of an N-contiguous B and of an M-contiguous A that start on 16-byte boundaries (N % 16, M % 16).  Rows of C (and a
    // per-column factor vector) that do not start on 16-byte boundaries are served by the
    // element-wise stores of the epilogue: with B stored N x K any N goes (a vocabulary-sized
    // output layer, weights stored [out, in]).
    const bool c_lines = N % 16 == 0 && aligned16(g.C) && (!g.ep.b_per_col || aligned16(g.ep.sB_dev));
    const bool fast = !force_generic() && !force_mfma_any() && aligned16(g.A) && aligned16(g.B) && fits32 && K % 16 == 0 &&
                      (g.transB || N % 16 == 0) && (!g.transA || M % 16 == 0);
    if (!fast) return plan;
    // Tile width.  One workgroup per compute unit (256 of them) runs at a time.  The 256 x 128
    // tile sustains about 0.88 of the rate of the 256 x 256 tile (measured on 8192 x 49152 x
    // 12288: 0.80-0.92 over the layouts and modes), so it is chosen when it fills the rounds of
    // workgroups that much better (4096 x 6144: 384 wide tiles = 1.5 rounds, 768 narrow ones = 3).
    // The knob FP8_KNOB_TILE_N = 128 | 256 overrides the choice.
    auto fill = [&](int64_t bn) {
        const int64_t tiles = ((M + TILE_M - 1) / TILE_M) * ((N + bn - 1) / bn);
        return (double)tiles / (double)(((tiles + 255) / 256) * 256);
    };
    const int tn = knob(FP8_KNOB_TILE_N);
    const bool narrow = tn ? tn == 128 : 0.88 * fill(128) > fill(256);
    plan.kernel = narrow ? GEMM_TILED_128 : GEMM_TILED_256;
    plan.elementwise_stores = !c_lines;
    // Both widths in one launch (gemm_mixed_kernel): the first c tile columns of 256, the rest of N in
    // tiles of 128.  Chosen where a model of the run time says it beats the better single width by 3 %:
    // workgroups are handed to the 256 compute units in order, the wide ones first; a tile takes
    // a S + b microseconds, S = stages of 64 along K (fitted to one-round and three-round problems,
    // 4096 x 4096 and 4096 x 6144 over K = 512 .. 8192: fp16 mode 1.30 S + 9.4 wide, 0.70 S + 5.8
    // narrow; FP8 mode 0.65 S + 8.6 and 0.37 S + 4.7), and the change of width costs 3 + 32 / S
    // microseconds (measured: the mixed launch is that much slower than its two parts).  With these
    // figures it pays for long K (4096 x 6144 x 8192: 4 % in the fp16 mode, 7 % in the FP8 mode) and
    // not for short K, where the narrow tile is nearly as efficient as the wide one.  Problems of
    // more than 64 rounds are left alone (the last round is then under 2 %).
    // Knob FP8_KNOB_MIXED: 0 = by the model, 1 = never, 2 = wherever it is possible.
    const int mk = knob(FP8_KNOB_MIXED);
    const int64_t tiles_m = (M + TILE_M - 1) / TILE_M, wide_cols_all = (N + TILE_N - 1) / TILE_N;
    if (!tn && mk != 1 && g.splits <= 1 && N > TILE_N && tiles_m * wide_cols_all <= 64 * 256) {
        const double S = 2.0 * (double)((K + 2 * TILE_K - 1) / (2 * TILE_K));
        const double tw = g.acc == ACC_FP8 ? 0.65 * S + 8.6 : 1.30 * S + 9.4;
        const double tnar = g.acc == ACC_FP8 ? 0.37 * S + 4.7 : 0.70 * S + 5.8;
        const double change = 3.0 + 32.0 / S;
        // time until the last of Tw wide and then Tn narrow tiles ends on 256 units
        auto makespan = [&](int64_t Tw, int64_t Tn) {
            const int64_t q = Tw / 256, k = Tw % 256;          // k units get q + 1 wide tiles, the others q
            if (Tn == 0) return (double)(q + (k > 0)) * tw;
            double best = 1e300;
            for (int64_t r = 0; r <= Tn; ++r) {                // r narrow tiles on the units that are free first
                const int64_t late = r * tnar >= tw ? (int64_t)((r * tnar - tw) / tnar) : 0;     // and as many as fit on the others
                if ((256 - k) * r + k * late >= Tn) { best = (double)q * tw + (double)r * tnar; break; }
            }
            for (int64_t r = 1; r <= Tn; ++r) {                // or the last one ends on a unit that had q + 1 wide tiles
                const int64_t early = (int64_t)((tw + r * tnar) / tnar);
                if (k * r + (256 - k) * early >= Tn) { best = std::min(best, (double)(q + 1) * tw + (double)r * tnar); break; }
                if ((double)(q + 1) * tw + (double)r * tnar >= best) break;
            }
            return best;
        };
        const double uniform = std::min(makespan(tiles_m * wide_cols_all, 0), makespan(0, tiles_m * ((N + 127) / 128)));
        double best = 1e300;
        int64_t best_c = 0;
        for (int64_t c = 1; c * TILE_N < N; ++c) {
            const double t = makespan(tiles_m * c, tiles_m * ((N - c * TILE_N + 127) / 128)) + change;
            if (t < best) { best = t; best_c = c; }
        }
        if (best_c > 0 && (mk == 2 || best < 0.97 * uniform)) {
            plan.kernel = GEMM_TILED_MIXED;
            plan.wide_cols = (int)best_c;
        }
    }
    // The persistent form of the narrow tile (one workgroup per compute unit walks its tiles as one K
    // loop, see gemm_tiled.hip): for problems of more than one round of tiles without edge tiles, with
    // per-tensor factors and an fp32 / bf16 output.  It hides every tile's first loads and sends the
    // outputs straight from the registers, but its workgroups cannot even out their speeds over the
    // tiles as separately scheduled ones do.  Measured on 4096 x 6144 (768 tiles): with fp32 outputs
    // 3 - 6 % faster up to K = 4096 in both accumulation modes (the LDS turn of an fp32 tile takes two
    // passes); with bf16 outputs 2 % faster around K = 2048 in the fp16 mode, slower in the FP8 mode;
    // 1 - 2 % slower at K = 8192 throughout.  Knob FP8_KNOB_PERSIST: 0 = where it pays (below),
    // 1 = never, 2 = wherever it is possible.
    const int pk = knob(FP8_KNOB_PERSIST);
    const int64_t tiles = tiles_m * ((N + 127) / 128);
    const bool possible = plan.kernel == GEMM_TILED_128 && c_lines && M % TILE_M == 0 && N % 128 == 0 && K % (2 * TILE_K) == 0 && K >= 8 * TILE_K &&
                          !g.ep.a_per_row && !g.ep.b_per_col && g.ep.out_kind <= OUT_BF16 && !g.ep.amax_out && g.splits <= 1;
    const bool pays = tiles > 256 && (g.ep.out_kind == OUT_F32 ? K <= 64 * TILE_K
                                                               : g.acc == ACC_F16 && K >= 16 * TILE_K && K <= 32 * TILE_K);
    plan.persistent = possible && pk != 1 && (pk == 2 || pays);
    return plan;
}

int launch_tiled(const GemmArgs& g)
{
    typedef int (*tiled_fn)(const GemmArgs&);
    static const tiled_fn table[4][2] = {
        {FP8MM_TILED_NAME(0, 0), FP8MM_TILED_NAME(0, 1)}, {FP8MM_TILED_NAME(1, 0), FP8MM_TILED_NAME(1, 1)},
        {FP8MM_TILED_NAME(2, 0), FP8MM_TILED_NAME(2, 1)}, {FP8MM_TILED_NAME(3, 0), FP8MM_TILED_NAME(3, 1)}};
    return table[(g.transA ? 2 : 0) + (g.transB ? 1 : 0)][g.acc == ACC_FP8 ? 1 : 0](g);
}

int launch_gemm(const GemmArgs& g)
{
    const int64_t M = g.M, N = g.N, K = g.K;
    if (g.ep.amax_out) {                                     // written, not accumulated
        hipLaunchKernelGGL(zero_cell_kernel, dim3(1), dim3(1), 0, g.stream, (unsigned*)g.ep.amax_out);
        if (M == 0 || N == 0) return check_launch("gemm (amax init)");
    }
    if (M == 0 || N == 0) return FP8_OK;
    if (K == 0) {                                            // empty sums: every output is +0
        const size_t nbytes = (size_t)M * (size_t)N * (size_t)out_elem_size(g.ep.out_kind);
        hipLaunchKernelGGL(zero_fill_kernel, dim3(1024), dim3(256), 0, g.stream, (unsigned char*)g.C, nbytes);
        return check_launch("gemm (K = 0 fill)");
    }
    const GemmPlan plan = plan_gemm(g);
    if (plan.kernel == GEMM_MFMA_ANY) return launch_mfma_any(g);
    if (plan.kernel != GEMM_GENERIC) {
        GemmArgs gt = g;
        gt.ep.ragged_n = plan.elementwise_stores ? 1 : 0;
        gt.tile_n = plan.kernel == GEMM_TILED_128 ? 128 : 256;
        gt.wide_cols = plan.kernel == GEMM_TILED_MIXED ? plan.wide_cols : 0;
        gt.persist = plan.persistent;
        gt.splits = 1;
        return launch_tiled(gt);
    }
    if (g.fmtA == FP8_E4M3)
        return g.fmtB == FP8_E4M3 ? launch_generic<FP8_E4M3, FP8_E4M3>(g) : launch_generic<FP8_E4M3, FP8_E5M2>(g);
    return g.fmtB == FP8_E4M3 ? launch_generic<FP8_E5M2, FP8_E4M3>(g) : launch_generic<FP8_E5M2, FP8_E5M2>(g);
}

}  // namespace fp8mm
