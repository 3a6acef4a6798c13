/*
 * fp8mm.h -- C ABI of the MI355X (gfx950) scaled-FP8 matrix multiply library.
 *
 * The library implements, as hand-written HIP kernels, the per-tensor-scaled FP8
 * path of "FP8 Formats for Deep Learning" (arXiv 2209.05433):
 *
 *     amax  ->  scale  ->  cast to E4M3 / E5M2  ->  FP8 x FP8 GEMM (fp32 accumulate)
 *           ->  unscale epilogue to fp32 / bf16 / FP8
 *
 * and the variants of these steps that scaling recipes build on (transposed operands,
 * per-channel factors, single-pass cast with a factor from past maxima, strict and
 * stochastic conversion, dequantize).
 *
 * General rules for every entry point
 *   - Pointers are DEVICE pointers unless the name ends in _host.  The caller owns
 *     every buffer; the library allocates no device memory and keeps no state
 *     besides the thread-local error string.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All
 *     work is enqueued on it; no entry point synchronises the stream or the device.
 *     Every entry point may be recorded into a HIP graph (kernel launches only, no
 *     memset nodes); the first GEMM call of each kind on a device raises that kernel's
 *     LDS limit (hipFuncSetAttribute) and should be made outside a capture.
 *   - Output cells described as "written, not accumulated" are cleared by a small
 *     kernel on the same stream before they are raised with atomics.
 *   - The return value is an fp8_status_t; fp8_last_error() describes the reason of a
 *     failure.  FP8_ERR_INVALID_ARG and FP8_ERR_UNSUPPORTED are found on the host before
 *     anything is enqueued: nothing was launched, no output was written.  FP8_ERR_DEVICE
 *     reports what the HIP runtime said at a launch; kernels enqueued earlier in the same
 *     call (the clearing of a "written, not accumulated" cell) may already have run, and
 *     the outputs of the call are then unspecified.
 *   - Tensors are dense and contiguous.  Matrices are row-major.
 *   - bfloat16 data is the upper 16 bits of an IEEE single (uint16_t storage).
 */
#ifndef FP8MM_H
#define FP8MM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* The two 8-bit encodings (Section 3, Table 1): sign.exponent.mantissa =
 * 1.4.3 with bias 7, no infinities, one NaN pattern per sign, max 448 (E4M3);
 * 1.5.2 with bias 15, IEEE-style inf/NaN, max 57344 (E5M2). */
typedef enum { FP8_E4M3 = 0, FP8_E5M2 = 1 } fp8_format_t;

/* The wider types FP8 tensors are produced from and GEMM results are written in
 * (Section 2: FP8 tensors come from wider types; math on FP8 inputs yields
 * higher-precision outputs). */
typedef enum { FP8_F32 = 0, FP8_BF16 = 1 } fp8_dtype_t;

typedef enum {
    FP8_OK = 0,
    FP8_ERR_INVALID_ARG = 1,   /* null pointer, bad enum, negative size, misalignment */
    FP8_ERR_UNSUPPORTED = 2,   /* valid request this build has no kernel for */
    FP8_ERR_DEVICE = 3         /* the HIP runtime reported an error at launch */
} fp8_status_t;

/*
 * fp8_amax -- largest magnitude of a tensor (Section 2: the scaling factor is chosen
 * from the largest magnitude the tensor holds; Section 4.3: one factor per tensor).
 *   x        n elements of in_dtype (fp8_dtype_t); 4-byte aligned for F32, 2-byte for BF16
 *   amax_out one float, overwritten (not accumulated)
 * Any NaN element makes the result NaN; +-inf gives +inf; n == 0 gives 0 (x may be
 * NULL then).  Implemented with integer comparisons of the magnitude bits, which
 * order like the values (Section 3.1).
 */
int fp8_amax(const void* x, size_t n, int in_dtype, float* amax_out, void* stream);

/*
 * fp8_amax_scale -- fp8_amax and fp8_scale_from_amax in ONE kernel launch (Section 2: the factor
 * is chosen from the tensor's largest magnitude; amax and factor are those of the two calls, bit for
 * bit).  No cell is cleared beforehand: every workgroup leaves its maximum in the workspace and the
 * last one to finish reduces them and writes both results.  For the per-step path
 * amax -> scale -> cast, where two one-thread launches cost as much as casting a small tensor.
 *   amax_out   device, one fp32, overwritten;  scale_out  device, one fp32, or NULL (amax only)
 *   workspace  device, FP8_AMAX_WORKSPACE_BYTES bytes, 4-byte aligned.  It must be zero-filled
 *              once, before the first call that uses it; every call leaves its counters zero
 *              again, so calls that follow one another on a stream can share one workspace.
 *              Calls that may overlap (different streams) need a workspace each.
 * n == 0 gives amax 0 and scale 1.  Errors as fp8_amax.
 */
#define FP8_AMAX_WORKSPACE_BYTES 16384
int fp8_amax_scale(const void* x, size_t n, int in_dtype, int fmt, float* amax_out, float* scale_out,
                   void* workspace, void* stream);

/*
 * fp8_amax_scale_multi, fp8_quantize_multi -- the two steps above for up to FP8_MULTI_MAX tensors of
 * one element type in ONE launch each (both operands of a GEMM, say: Section 2's per-tensor
 * amax -> factor -> cast applies to each of them).  For small tensors a launch costs as much as the
 * kernel's work; results are those of the single-tensor calls, bit for bit.
 *   count      number of tensors, 0 .. FP8_MULTI_MAX
 *   x, n, fmt  HOST arrays of count entries: device pointer, element count and FP8 format of each
 *              tensor (read during the call; alignment of x[i] as for fp8_amax)
 *   amax_out, scale_out  DEVICE arrays of count floats (scale_out may be NULL for fp8_amax_scale_multi)
 *   workspace  device, count * FP8_AMAX_WORKSPACE_BYTES bytes, rules as for fp8_amax_scale
 *   scale_dev  device array of count factors (fp8_quantize_multi: as fp8_quantize_dscale per tensor)
 *   q_out      HOST array of count device pointers to the output bytes
 * Tensors that do not meet the conditions of the vector kernels (empty, not 16-byte aligned,
 * outputs of 384 MiB and more) are served by single-tensor launches inside the call.
 * Errors: FP8_ERR_INVALID_ARG for a bad count, NULL arrays, bad enums or misaligned pointers.
 */
#define FP8_MULTI_MAX 4
int fp8_amax_scale_multi(int count, const void* const* x, const size_t* n, int in_dtype, const int* fmt,
                         float* amax_out, float* scale_out, void* workspace, void* stream);
int fp8_quantize_multi(int count, const void* const* x, const size_t* n, int in_dtype, const int* fmt,
                       const float* scale_dev, uint8_t* const* q_out, void* stream);

/*
 * fp8_scale_from_amax_host / fp8_scale_from_amax -- scale = fmt_max / amax in IEEE
 * single precision, fmt_max = 448 (E4M3) or 57344 (E5M2) (Section 2: the maximum
 * magnitude is moved close to the largest representable one; Table 1, Max normal;
 * Section 3.2: the factor may be any real number, it is not rounded to a power of
 * two).  If amax is 0, NaN or inf, or the quotient is not finite, the scale is 1.
 * The device form reads amax[0] and writes scale_out[0] on `stream`.
 */
float fp8_scale_from_amax_host(float amax, int fmt);
int fp8_scale_from_amax(const float* amax, int fmt, float* scale_out, void* stream);

/*
 * fp8_quantize -- q[i] = FP8(fl32(x[i] * scale)) (Section 2: multiply by the scaling
 * factor, then cast; overflow saturates; Table 1 for the encodings).
 *   x      n elements of in_dtype
 *   fmt    fp8_format_t of the result
 *   scale  by value (fp8_quantize) or read from device memory (fp8_quantize_dscale,
 *          which lets amax -> scale -> cast run without a host round trip)
 *   q_out  n bytes, same element order as x
 * Rounding is to nearest, ties to the even code.  Finite values beyond the format's
 * maximum become the maximum; NaN becomes NaN (0x7F | sign); +-inf becomes NaN for
 * E4M3 and +-inf for E5M2 (Section 2, type conversion).  The sign of the input is
 * kept, also on results that round to zero.  n == 0 is valid and launches nothing.
 */
int fp8_quantize(const void* x, size_t n, int in_dtype, int fmt, float scale,
                 uint8_t* q_out, void* stream);
int fp8_quantize_dscale(const void* x, size_t n, int in_dtype, int fmt,
                        const float* scale, uint8_t* q_out, void* stream);

/*
 * fp8_quantize_ex -- fp8_quantize with both ways of passing the scale (scale_dev, if not
 * NULL, is read from device memory and `scale` is ignored) and conversion flags:
 *   FP8_QUANT_NOSAT  the strict conversion Section 2 allows for uses that must see
 *                    overflow: a value whose rounding lands beyond the largest finite value
 *                    becomes NaN (E4M3) or +-inf (E5M2) instead of the maximum.  Rounding is
 *                    done against the next point of the exponent/mantissa grid (480 / 65536),
 *                    so 464 still rounds to 448 and 61440 to inf.
 * Unknown flag bits are an FP8_ERR_INVALID_ARG.
 */
#define FP8_QUANT_NOSAT 1
int fp8_quantize_ex(const void* x, size_t n, int in_dtype, int fmt, float scale,
                    const float* scale_dev, int flags, uint8_t* q_out, void* stream);

/*
 * fp8_dequantize -- out[i] = decode(q[i]) / scale in IEEE single precision, written as fp32
 * or rounded to bf16 (Section 2: values are unscaled by the inverse of the scaling factor
 * after conversion from FP8; Section 4: the paper's own experiments cast to FP8 and back).
 *   q    n FP8 bytes of format fmt;   out  n elements of out_dtype
 *   scale by value, or from device memory if scale_dev is not NULL
 * NaN and inf codes decode to NaN and inf.  n == 0 launches nothing.
 */
int fp8_dequantize(const uint8_t* q, size_t n, int fmt, float scale, const float* scale_dev,
                   int out_dtype, void* out, void* stream);

/*
 * fp8_quantize_amax -- the cast of fp8_quantize_dscale and the amax of fp8_amax over the same
 * input, in one pass over x.  For recipes that pick the scaling factor before the tensor
 * exists (Section 2 leaves the choice of the factor to software), e.g. from the maxima of
 * earlier steps: the tensor is then read once instead of twice.
 *   scale_dev  device, one fp32: the factor applied in this call
 *   q_out      device, n bytes;  amax_out  device, one fp32 = max |x[i]| (NaN propagates);
 *              written, not accumulated; n == 0 gives 0
 * Same rounding, specials and errors as fp8_quantize / fp8_amax.
 */
int fp8_quantize_amax(const void* x, size_t n, int in_dtype, int fmt, const float* scale_dev,
                      uint8_t* q_out, float* amax_out, void* stream);

/*
 * fp8_quantize_sr -- the scaled cast with stochastic rounding in place of round-to-nearest
 * (Section 2 names stochastic rounding among the rounding modes left to the implementation and
 * does not define it; this definition is the library's).  y = fl32(x[i] * scale) of magnitude
 * below the format's largest value lies between adjacent FP8 values lo <= |y| < hi; with
 * T = floor(2^16 (|y| - lo) / (hi - lo)) the result is hi if T + r_i >= 2^16, else lo: hi with
 * probability T / 2^16, values on the grid never move.  Larger magnitudes saturate; sign, NaN and
 * inf as in fp8_quantize.  r_i = 16-bit field i % 8 (low half of word 0 first) of the output of
 * Philox4x32-10 (Salmon et al., SC 2011) for the counter (i / 8, 0, 0) -- i / 8 as a 64-bit
 * number in counter words 0 and 1 -- and the key (seed low word, seed high word): results depend
 * on (seed, i) alone, not on the launch shape.  scale_dev, if not NULL, replaces scale.
 */
int fp8_quantize_sr(const void* x, size_t n, int in_dtype, int fmt, float scale,
                    const float* scale_dev, uint64_t seed, uint8_t* q_out, void* stream);

/*
 * fp8_scale_from_amax_history -- scale = fmt_max / max(amax_history[0 .. len-1]) by the rule
 * of fp8_scale_from_amax (a NaN entry propagates into the maximum; a zero, NaN or infinite
 * maximum, or len == 0, gives 1).  amax_history: device, len fp32 values.
 * fp8_scale_from_amax_n -- n factors from n maxima, element by element (per-row scaling).
 */
int fp8_scale_from_amax_history(const float* amax_history, size_t len, int fmt,
                                float* scale_out, void* stream);
int fp8_scale_from_amax_n(const float* amax, size_t n, int fmt, float* scale_out, void* stream);

/*
 * fp8_amax_rows / fp8_quantize_rows -- one maximum / one scaling factor per row of a
 * rows x cols row-major matrix (Section 4.2: per-channel scaling factors for weights; a weight
 * stored [out x in] with one factor per output channel is the N x K form of operand B, and its
 * factors are the per-column factors of fp8_gemm_fused).
 *   amax_out   device, rows fp32:  amax_out[r] = max_c |x[r][c]| (NaN propagates; cols == 0: 0)
 *   scale_dev  device, rows fp32:  q[r][c] = FP8(fl32(x[r][c] * scale_dev[r]))
 * Same rounding, specials and errors as fp8_amax / fp8_quantize.
 */
int fp8_amax_rows(const void* x, int64_t rows, int64_t cols, int in_dtype, float* amax_out,
                  void* stream);
int fp8_quantize_rows(const void* x, int64_t rows, int64_t cols, int in_dtype, int fmt,
                      const float* scale_dev, uint8_t* q_out, void* stream);

/*
 * fp8_quantize_transpose -- the cast of fp8_quantize_dscale applied to a rows x cols row-major
 * matrix, written in both storage orders by one pass over x (Section 4.1: activations, weights
 * and activation gradients all feed GEMMs, and the backward pass consumes them transposed):
 *   q_out   device, rows x cols bytes, q[r][c] = FP8(fl32(x[r][c] * scale)); may be NULL
 *   qt_out  device, cols x rows bytes, qt[c][r] = q[r][c]
 * Any shape; rows and cols multiples of 16 with 16-byte aligned pointers take the tiled kernel.
 */
int fp8_quantize_transpose(const void* x, int64_t rows, int64_t cols, int in_dtype, int fmt,
                           const float* scale_dev, uint8_t* q_out, uint8_t* qt_out, void* stream);

/*
 * fp8_gemm -- C = (1 / (sA * sB)) * (A x B) with FP8 operands, fp32 accumulation
 * and the unscale applied once per output (Section 2: matrix multiplies on FP8
 * inputs produce single-precision results; unscaling is done once per dot product;
 * Section 3: E4M3 for activations and weights, E5M2 for gradients -- all four
 * operand format combinations are accepted).
 *   A  M x K bytes, row-major, format fmtA, quantised with scale sA
 *   B  K x N bytes, row-major, format fmtB, quantised with scale sB
 *   C  M x N elements of out_dtype (fp32, or bf16 rounded to nearest even), row-major
 * Every output satisfies |C - C_ref| <= 2^-20 * sum_k |a_ik b_kj| / (sA sB) + ulp/2,
 * C_ref being the exact product of the decoded operands: the FP8 bytes are widened
 * exactly to fp16 in registers and multiplied by the fp16 matrix-core instructions,
 * whose accumulation is fp32-grade.  M, N or K equal to 0 is valid (K == 0 writes
 * zeros).  Any shape is accepted.  The tiled matrix-core kernel takes those with K a
 * multiple of 16 and 16-byte aligned A and B whose operand rows start on 16-byte
 * boundaries: N a multiple of 16 where B is given as K x N, M a multiple of 16 where A is
 * given as K x M (see fp8_gemm_ex); with B given as N x K any N goes.  A C that is not
 * 16-byte aligned, or whose rows are not (N not a multiple of 16), is stored element by
 * element.  The other shapes and alignments take a second matrix-core kernel (register-staged
 * loads, 256 x 256 or 128 x 128 tiles, the same arithmetic and bound, 0.5 - 0.8 of the rate; see
 * fp8_gemm_plan).  fp8_gemm_dscale reads the two scales from device memory instead.
 */
int fp8_gemm(const uint8_t* A, int fmtA, float sA,
             const uint8_t* B, int fmtB, float sB,
             void* C, int64_t M, int64_t N, int64_t K, int out_dtype, void* stream);
int fp8_gemm_dscale(const uint8_t* A, int fmtA, const float* sA,
                    const uint8_t* B, int fmtB, const float* sB,
                    void* C, int64_t M, int64_t N, int64_t K, int out_dtype, void* stream);

/*
 * fp8_gemm_mfma8 -- the same product (same arguments, layouts and error behaviour)
 * formed by the FP8 matrix-core instructions of gfx950, at twice the peak rate of
 * fp8_gemm (Section 2 leaves the arithmetic of FP8-input instructions to the
 * processor).  The hardware adds each run of 8 products after aligning them to the
 * largest and dropping the bits more than 13 places below its leading bit, so the
 * guarantee is weaker: |C - C_ref| <= 2^-10 * sum_k |a_ik b_kj| / (sA sB) + ulp/2 in the
 * worst case, about 2^-17 of that sum for typical tensors.  Products whose runs of 8 span
 * less than 7 binades are exact, as with fp8_gemm.  Shapes outside the tiled kernel's
 * (see fp8_gemm) are computed exactly as fp8_gemm does.
 */
int fp8_gemm_mfma8(const uint8_t* A, int fmtA, float sA,
                   const uint8_t* B, int fmtB, float sB,
                   void* C, int64_t M, int64_t N, int64_t K, int out_dtype, void* stream);
int fp8_gemm_mfma8_dscale(const uint8_t* A, int fmtA, const float* sA,
                          const uint8_t* B, int fmtB, const float* sB,
                          void* C, int64_t M, int64_t N, int64_t K, int out_dtype, void* stream);

/*
 * fp8_gemm_ex -- the general form: C = (1 / (sA sB)) * op(A) x op(B), with each operand in
 * either storage order.  It covers the three GEMMs of a linear layer's training step
 * (Section 4.1: activations, weights and activation gradients are the GEMM inputs that are
 * cast to FP8), without a transposed copy of any operand:
 *     forward   Y  = X  W^T   X [tokens x in]   transA = 0;  W  [out x in]      transB = 1
 *     dgrad     dX = dY W     dY[tokens x out]  transA = 0;  W  [out x in]      transB = 0
 *     wgrad     dW = dY^T X   dY[tokens x out]  transA = 1;  X  [tokens x in]   transB = 0
 *   transA = 0: A is M x K row-major;   transA = 1: A is given as K x M row-major
 *   transB = 0: B is K x N row-major;   transB = 1: B is given as N x K row-major
 *   sA_dev / sB_dev: both NULL (scales by value) or both device pointers (values ignored)
 *   flags: FP8_GEMM_MFMA8 selects the FP8 matrix-core instructions (see fp8_gemm_mfma8)
 * Error bounds, shape rules and error behaviour are those of fp8_gemm / fp8_gemm_mfma8.
 */
#define FP8_GEMM_MFMA8 1
int fp8_gemm_ex(const uint8_t* A, int fmtA, int transA, const uint8_t* B, int fmtB, int transB,
                void* C, int64_t M, int64_t N, int64_t K, int out_dtype,
                float sA, float sB, const float* sA_dev, const float* sB_dev, int flags,
                void* stream);

/*
 * fp8_gemm_splitk -- fp8_gemm_ex for problems with few output tiles and a long K, above all the
 * weight gradient dW = dY^T X (Section 4.1: activation gradients and activations are GEMM inputs;
 * its K is the number of tokens).  K is cut into slices; every slice of every 256 x 256 tile is a
 * workgroup of its own, so that a 1024 x 1024 x 65536 problem occupies the whole chip instead of 16
 * compute units.  The slices' fp32 sums go to `workspace`; a second kernel adds them in slice order
 * (results are the same in every run), applies 1 / (sA sB) once per output (Section 2) and converts.
 * Arguments, bounds and error behaviour as fp8_gemm_ex, and:
 *   splits           0: the library chooses (about 256 / tiles, slices of at least 512 along K);
 *                    1..64: that many slices (fewer if K is too short to give each one 128)
 *   workspace        device, 4-byte aligned (16 for the fastest stores), at least
 *                    fp8_gemm_splitk_workspace_size(M, N, K, transA, transB, splits) bytes
 *                    = slices x M x N x 4; contents on entry are irrelevant, they are overwritten.
 *                    May be NULL where that size is 0 (one slice, or a problem the tiled kernel
 *                    does not take: the call is then fp8_gemm_ex).
 *   workspace_bytes  size of the workspace; too small is an FP8_ERR_INVALID_ARG, nothing launched
 * fp8_gemm_splitk_workspace_size assumes 16-byte aligned A and B (what the tiled kernel needs) and
 * returns 0 for M, N or K <= 0 or splits outside 0..64.
 */
size_t fp8_gemm_splitk_workspace_size(int64_t M, int64_t N, int64_t K, int transA, int transB, int splits);
int fp8_gemm_splitk(const uint8_t* A, int fmtA, int transA, const uint8_t* B, int fmtB, int transB,
                    void* C, int64_t M, int64_t N, int64_t K, int out_dtype,
                    float sA, float sB, const float* sA_dev, const float* sB_dev, int flags,
                    int splits, void* workspace, size_t workspace_bytes, void* stream);

/*
 * fp8_gemm_splitk_static -- fp8_gemm_splitk for callers that cannot allocate or carry a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The call
 * allocates nothing (no hipMalloc / hipFree, no allocating library routine): the slices' sums go
 * to a device array inside the library, FP8_SPLITK_STATIC_BYTES (64 MiB) per device, which every
 * device the library runs on holds until the process ends.  Results are those of fp8_gemm_splitk
 * with the same number of slices, bit for bit.
 *   splits  0: the library's choice, cut down to the slices the array holds (if it cannot hold
 *           two, the call is the plain fp8_gemm_ex);  1..64: that many slices -- if they need
 *           more than the array holds (slices x M x N x 4 bytes), FP8_ERR_UNSUPPORTED, nothing launched
 * All calls on one device share that device's array: calls that may overlap on a device (different
 * streams, different threads) race on it and must be serialised by the caller; calls that follow
 * one another on a stream are fine.  The first call on a device looks the array's address up
 * (hipGetSymbolAddress) and should be made outside a graph capture.
 */
#define FP8_SPLITK_STATIC_BYTES ((size_t)64 << 20)
int fp8_gemm_splitk_static(const uint8_t* A, int fmtA, int transA, const uint8_t* B, int fmtB, int transB,
                           void* C, int64_t M, int64_t N, int64_t K, int out_dtype,
                           float sA, float sB, const float* sA_dev, const float* sB_dev, int flags,
                           int splits, void* stream);

/*
 * fp8_gemm_fused -- the GEMM with the scale granularities and the output conversions that
 * training recipes build on:
 *     c_ij    = (sum_k a_ik b_kj) / (sA_i * sB_j)
 *     amax    = max_ij |c_ij|                                   (if amax_out is given)
 *     D_ij    = cast_out(c_ij)            for FP8_OUT_F32 / FP8_OUT_BF16
 *     D_ij    = encode_fmt(fl32(c_ij * sD))  for FP8_OUT_E4M3 / FP8_OUT_E5M2
 * Section 2: results of FP8 matrix products may be converted to FP8 before they are written
 * to memory, with a scaling factor of their own; Section 4.2 uses per-channel scaling factors
 * for weights; Section 4.3 / Section 2 leave the choice of the factor to software -- the
 * output amax is what a recipe that derives the next step's factor from past maxima needs.
 *   A, B, transA, transB, M, N, K, flags: as for fp8_gemm_ex
 *   D        device, M x N row-major, element type given by out_kind (1 byte for FP8 kinds)
 *   sA_dev   device, nsA values: nsA = 1 one factor for A, nsA = M one per row of op(A)
 *   sB_dev   device, nsB values: nsB = 1 one factor for B, nsB = N one per column of op(B)
 *   sD_dev   device, one value, or NULL for 1; FP8 output kinds only (else must be NULL)
 *   amax_out device, one fp32, or NULL.  Written, not accumulated: NaN if any c_ij is NaN,
 *            else the largest |c_ij| as computed (before the output scale and rounding)
 * The FP8 conversion is the one of fp8_quantize (nearest even, saturating, NaN -> NaN,
 * inf -> NaN for E4M3 / inf for E5M2).  c_ij meets the bound of fp8_gemm (fp8_gemm_mfma8 with
 * FP8_GEMM_MFMA8); an FP8 output byte is the encoding of a value within that bound of
 * c_ref * sD, so it can differ from the encoding of c_ref * sD itself only where that lies
 * within the bound of a rounding boundary.  Scales must be finite and non-zero.
 * Errors: as fp8_gemm; also FP8_ERR_INVALID_ARG for nsA not in {1, M}, nsB not in {1, N},
 * NULL scale pointers, a bad out_kind, or sD_dev with a non-FP8 output.
 */
typedef enum { FP8_OUT_F32 = 0, FP8_OUT_BF16 = 1, FP8_OUT_E4M3 = 2, FP8_OUT_E5M2 = 3 } fp8_out_t;
int fp8_gemm_fused(const uint8_t* A, int fmtA, int transA, const uint8_t* B, int fmtB, int transB,
                   void* D, int out_kind, int64_t M, int64_t N, int64_t K,
                   const float* sA_dev, int64_t nsA, const float* sB_dev, int64_t nsB,
                   const float* sD_dev, float* amax_out, int flags, void* stream);

/*
 * fp8_scaled_gemm -- the whole of Section 2's scheme for one product in ONE call: per-tensor amax and
 * factor of both operands (fmt_max / amax), their casts to FP8, the FP8 x FP8 product with
 * single-precision accumulation, and the factors taken out once per output.  It issues exactly the
 * launches of fp8_amax_scale_multi, fp8_quantize_multi and fp8_gemm_ex (factors read from scale_out)
 * in that order on `stream`, so every result is theirs bit for bit; what it saves is the host time
 * between three short dependent launches (4096 x 6144 x 2048: 0.147 - 0.155 -> 0.128 - 0.142 ms per step
 * over hosts; replaying the launches from a captured HIP graph, which a caller can do with either
 * form, gives 0.118).
 *   a, b        the operands in the wide type in_dtype, stored as fp8_gemm_ex stores A and B
 *               (a: M x K, or K x M if transA; b: K x N, or N x K if transB); alignment as for fp8_amax
 *   fmtA, fmtB  FP8 formats the operands are cast to
 *   qa_out, qb_out  M K and K N bytes: the FP8 operands, in the storage order of a and b (kept for
 *               the backward products)
 *   amax_out, scale_out  2 floats each: [0] for a, [1] for b
 *   workspace   2 * FP8_AMAX_WORKSPACE_BYTES bytes, rules as for fp8_amax_scale
 *   C, out_dtype, flags  as for fp8_gemm_ex
 * Errors: FP8_ERR_INVALID_ARG (bad enum or flag bits, negative dimension, NULL or misaligned
 * pointer), decided before anything is launched.
 */
int fp8_scaled_gemm(const void* a, const void* b, int in_dtype, int transA, int transB,
                    int64_t M, int64_t N, int64_t K, int fmtA, int fmtB,
                    uint8_t* qa_out, uint8_t* qb_out, float* amax_out, float* scale_out, void* workspace,
                    void* C, int out_dtype, int flags, void* stream);

/*
 * Which kernel the GEMM entry points would run for a problem (diagnostics; nothing is launched and
 * no pointer is dereferenced: only shapes, storage orders and pointer alignment decide).  Pass the
 * pointers of the intended call; sB_per_column is the per-column factor vector of fp8_gemm_fused or
 * NULL.  Returns FP8_PLAN_NO_GEMM if M, N or K is 0, otherwise one of FP8_PLAN_TILED_256x256,
 * FP8_PLAN_TILED_256x128 (the tiled matrix-core kernel, tile chosen for how well it fills the chip),
 * FP8_PLAN_TILED_MIXED (the same kernel with both tile widths in one launch: 256-wide tiles for the
 * first columns of the output, 128-wide ones for the rest, where that fills the rounds of workgroups
 * better than either width alone),
 * FP8_PLAN_MFMA_ANY (the matrix-core kernel for every other shape and alignment: an odd K, operand
 * rows that do not start on 16-byte boundaries, unaligned pointers; 0.5 - 0.8 of the tiled
 * kernel's rate, fifteen to twenty-five times that of plain FMAs; it computes in the default accumulation mode also under FP8_GEMM_MFMA8, which
 * meets that flag's bound a fortiori) or FP8_PLAN_FMA_KERNEL (plain FMAs: only when forced by
 * FP8_KNOB_GEMM_KERNEL or for outputs of more than 2^31 - 1 tiles of 128 x 128), ORed with
 * FP8_PLAN_ELEMENTWISE_STORES where the rows of the output do not start on 16-byte boundaries, and
 * with FP8_PLAN_PERSISTENT where the 256 x 128 kernel runs in its persistent form (answered for
 * per-tensor factors, an fp32 output and the default accumulation mode; with a bf16 output or
 * FP8_GEMM_MFMA8 the form is used over a narrower range of K, see FP8_KNOB_PERSIST).
 * A negative value is minus an fp8_status_t (bad arguments).  Section 2 fixes the arithmetic,
 * not the kernel: every plan computes the same product within the stated bounds.
 */
typedef enum { FP8_PLAN_NO_GEMM = 0, FP8_PLAN_FMA_KERNEL = 1, FP8_PLAN_TILED_256x256 = 2,
               FP8_PLAN_TILED_256x128 = 3, FP8_PLAN_MFMA_ANY = 4, FP8_PLAN_TILED_MIXED = 5,
               FP8_PLAN_ELEMENTWISE_STORES = 16,
               FP8_PLAN_PERSISTENT = 32 } fp8_plan_t;
int fp8_gemm_plan(const uint8_t* A, int transA, const uint8_t* B, int transB, const void* C,
                  int64_t M, int64_t N, int64_t K, const float* sB_per_column);

/*
 * Tuning knobs, for diagnostics, tests and benchmarks (the paper fixes the arithmetic, not the
 * kernels: no knob changes a result beyond the stated bounds).  Process-wide; each is seeded once
 * from the environment variable named below and changed with fp8_set_knob, which returns the
 * previous value (or minus an fp8_status_t for a bad knob or value).  Set them while no other
 * thread is inside a library call.
 *   FP8_KNOB_CAST_PATH    0 the FP8 conversion instructions of gfx950 (default), 1 the integer
 *                         rounding written from Table 1 (FP8MM_CAST_PATH=bits); both are bit-equal
 *   FP8_KNOB_TILE_N       0 the dispatcher chooses, 128 or 256 forces the tile width of the
 *                         tiled kernel and the form of the any-shape matrix-core kernel
 *                         (128 x 128 / 256 x 256 tiles) (FP8MM_TILE_N)
 *   FP8_KNOB_GROUP_M      tile rows per band of the tile order, 0 = default 8 (FP8MM_GROUP_M)
 *   FP8_KNOB_GEMM_KERNEL  0 the dispatcher chooses, 1 always the plain FMA kernel (FP8MM_GEMM=generic),
 *                         2 always the any-shape matrix-core kernel (FP8MM_GEMM=any)
 *   FP8_KNOB_SPLIT_K      0 fp8_gemm_splitk chooses its number of K slices, n > 0 forces n (FP8MM_SPLIT_K)
 *   FP8_KNOB_CAST_RUN     length of the contiguous run one workgroup of the cast kernel owns, in units
 *                         of 4096 elements; 0 = default (4: 16 384 elements) (FP8MM_CAST_RUN)
 *   FP8_KNOB_PERSIST      the persistent form of the matrix-core kernel (one workgroup per compute unit
 *                         walks several tiles as one K loop): 0 where the dispatcher finds it pays,
 *                         1 never, 2 wherever its conditions hold (FP8MM_PERSIST)
 *   FP8_KNOB_MIXED        both tile widths in one launch (FP8_PLAN_TILED_MIXED): 0 where the dispatcher's
 *                         model of the run time prefers it, 1 never, 2 wherever it is possible (FP8MM_MIXED)
 */
typedef enum { FP8_KNOB_CAST_PATH = 0, FP8_KNOB_TILE_N = 1, FP8_KNOB_GROUP_M = 2, FP8_KNOB_GEMM_KERNEL = 3,
               FP8_KNOB_SPLIT_K = 4, FP8_KNOB_CAST_RUN = 5, FP8_KNOB_PERSIST = 6, FP8_KNOB_MIXED = 7,
               FP8_KNOB_COUNT = 8 } fp8_knob_t;
int fp8_set_knob(int knob, int value);
int fp8_get_knob(int knob);

/* Text of the last error on the calling thread ("" if none).  Static storage. */
const char* fp8_last_error(void);

/* Library version string, static storage. */
const char* fp8_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FP8MM_H */
