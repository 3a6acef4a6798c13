// Declarations shared by the translation units of the GEMM (tiled kernel instances and the
// dispatcher with the generic kernel).
#pragma once

#include "common.hpp"
#include "fp8_decode.hpp"
#include "fp8_encode.hpp"

namespace fp8mm {

// Output kinds.  The first two are fp8_dtype_t; the FP8 kinds write one byte per output.
enum { OUT_F32 = 0, OUT_BF16 = 1, OUT_E4M3 = 2, OUT_E5M2 = 3 };
inline int out_elem_size(int kind) { return kind == OUT_F32 ? 4 : kind == OUT_BF16 ? 2 : 1; }

// How the products are formed and summed.
//   ACC_F16: operands widened to fp16 (exact for both FP8 formats), fp16 matrix-core
//            instructions.  These sum each instruction's products in a window of at least 24
//            bits: fp32-grade accumulation, at half the FP8 peak rate.
//   ACC_FP8: FP8 matrix-core instructions at the full FP8 rate.  The hardware adds each run of
//            8 products (the 8 bytes of a lane's register pair) after aligning them to the
//            largest and dropping what lies more than 13 bits below its leading bit, then
//            accumulates the runs in fp32.
enum { ACC_F16 = 0, ACC_FP8 = 1 };

// What happens to an accumulator on its way out (Section 2: the scaling factors are taken out
// once per dot product; results may be converted to FP8 before they are written):
//   c_ij = acc_ij / (sA_i * sB_j);  amax = max |c_ij|;  D_ij = cast_out(c_ij * sD)
// sA is one value or one per row of op(A), sB one value or one per column of op(B); sD applies
// to FP8 outputs only.
struct EpilogueArgs {
    float sA, sB;                 // host values, used where the device pointer is null
    const float* sA_dev;          // null, one value, or M values if a_per_row
    const float* sB_dev;          // null, one value, or N values if b_per_col
    const float* sD_dev;          // null (= 1) or one value
    float* amax_out;              // null or one cell, zeroed by the launcher, raised with atomicMax
    int out_kind;
    int a_per_row, b_per_col;
    int ragged_n;                 // set by the dispatcher for the tiled kernel: rows of C or the per-column
                                  // factors do not start on 16-byte boundaries, outputs are stored one by one
};

struct GemmArgs {
    const uint8_t* A; const uint8_t* B; void* C;
    int64_t M, N, K;
    int fmtA, fmtB;
    bool transA, transB;          // A stored K x M / B stored N x K
    int acc;                      // ACC_*
    int tile_n;                   // width of the tiled kernel's tile: 256, or 128 (chosen by the dispatcher)
    int wide_cols;                // tiled kernel: > 0 = both widths in one launch, this many tile columns of 256 first,
                                  // 128-wide tiles for the rest of N (chosen by the dispatcher)
    bool persist;                 // tiled kernel, narrow tile: the persistent form (one workgroup per compute unit walks
                                  // several tiles as one K loop); set by the dispatcher where its conditions hold
    int splits, pairs_per_split;  // tiled kernel only: splits > 1 cuts K into slices of pairs_per_split stage pairs
                                  // (128 bytes each); C is then a workspace of `splits` fp32 M x N matrices
    EpilogueArgs ep;
    hipStream_t stream;
};

// Tiled kernel, one translation unit per (storage orders, accumulation mode):
// layout = 2 * transA + transB.
#define FP8MM_TILED_NAME_(l, a) launch_tiled_l##l##_a##a
#define FP8MM_TILED_NAME(l, a) FP8MM_TILED_NAME_(l, a)
#define FP8MM_DECLARE_TILED(l) \
    int FP8MM_TILED_NAME(l, 0)(const GemmArgs& g); \
    int FP8MM_TILED_NAME(l, 1)(const GemmArgs& g);
FP8MM_DECLARE_TILED(0)
FP8MM_DECLARE_TILED(1)
FP8MM_DECLARE_TILED(2)
FP8MM_DECLARE_TILED(3)
#undef FP8MM_DECLARE_TILED

constexpr int TILE_M = 256, TILE_N = 256, TILE_K = 64;

int launch_gemm(const GemmArgs& g);

// The matrix-core kernel for any shape and alignment (gemm_mfma_any.hip): operands staged through
// registers; 128 x 128 tiles, or 256 x 256 tiles where those fill the chip (mfma_any_wide).  Takes
// every problem with M, N, K > 0 whose tile count fits the grid.
bool mfma_any_takes(const GemmArgs& g);
bool mfma_any_wide(const GemmArgs& g);
int launch_mfma_any(const GemmArgs& g);

// The tiled kernel instance for g's storage orders and accumulation mode, with g.tile_n, g.splits,
// g.pairs_per_split and g.ep.ragged_n as given (the caller has checked that the tiled kernel takes
// the problem).
int launch_tiled(const GemmArgs& g);

// Split-K (gemm_splitk.hip): K cut into `splits` slices of pairs_per_split stage pairs.
constexpr int kMaxSplitK = 64;
struct SplitPlan { int splits, pairs_per_split, tile_n; };
SplitPlan plan_splitk(const GemmArgs& g, int requested);
size_t splitk_workspace_bytes(const GemmArgs& g, const SplitPlan& sp);
int launch_gemm_splitk(const GemmArgs& g, const SplitPlan& sp, void* workspace);

// Argument checks shared by the GEMM entry points that take the arguments of fp8_gemm_ex; fills g.
// Returns FP8_OK or the status to return (the error text is set).
int fill_gemm_args(const char* who, GemmArgs& g, const uint8_t* A, int fmtA, int transA, const uint8_t* B, int fmtB,
                   int transB, void* C, int64_t M, int64_t N, int64_t K, int out_dtype, float sA, float sB,
                   const float* sA_dev, const float* sB_dev, int flags, void* stream);

// The dispatcher's decision for a problem with M, N, K > 0 (what launch_gemm acts on).
enum { GEMM_GENERIC = 1, GEMM_TILED_256 = 2, GEMM_TILED_128 = 3, GEMM_MFMA_ANY = 4, GEMM_TILED_MIXED = 5 };
struct GemmPlan { int kernel; bool elementwise_stores; bool persistent; int wide_cols; };
GemmPlan plan_gemm(const GemmArgs& g);

// ---- small device helpers used by the kernels -------------------------------------------------
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef _Float16 v2h __attribute__((ext_vector_type(2)));

// 8 FP8 bytes (two dwords) -> 8 fp16 values, exact (both formats embed in fp16; E4M3's NaN becomes NaN).
template <int FMT>
__device__ __forceinline__ v8h widen8(int lo, int hi)
{
    v2h p0, p1, p2, p3;
    if (FMT == FP8_E4M3) {
        p0 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8((unsigned)lo, 1.0f, false);
        p1 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8((unsigned)lo, 1.0f, true);
        p2 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8((unsigned)hi, 1.0f, false);
        p3 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8((unsigned)hi, 1.0f, true);
    } else {
        p0 = __builtin_amdgcn_cvt_scalef32_pk_f16_bf8((unsigned)lo, 1.0f, false);
        p1 = __builtin_amdgcn_cvt_scalef32_pk_f16_bf8((unsigned)lo, 1.0f, true);
        p2 = __builtin_amdgcn_cvt_scalef32_pk_f16_bf8((unsigned)hi, 1.0f, false);
        p3 = __builtin_amdgcn_cvt_scalef32_pk_f16_bf8((unsigned)hi, 1.0f, true);
    }
    return (v8h){p0.x, p0.y, p1.x, p1.y, p2.x, p2.y, p3.x, p3.y};
}

__device__ __forceinline__ float scale_value(const float* dev, float host) { return dev ? *dev : host; }

// Largest of `bits` (sign-stripped fp32 patterns; NaN patterns sort above infinity) over the wave,
// then one atomic per wave.
__device__ __forceinline__ void wave_amax_commit(unsigned bits, float* amax_out)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const unsigned o = (unsigned)__shfl_xor((int)bits, d, 64);
        bits = o > bits ? o : bits;
    }
    // most waves find the cell already large enough and skip the atomic (the lane index comes from
    // the execution mask count, not from threadIdx: nothing has to stay in a register for it)
    if (__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u)) == 0 &&
        bits > __hip_atomic_load((unsigned*)amax_out, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))
        atomicMax((unsigned*)amax_out, bits);
}

}  // namespace fp8mm
