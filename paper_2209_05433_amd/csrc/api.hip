// extern "C" entry points of libfp8mm: argument validation, then one launcher each.
#include "gemm_common.hpp"

#include <atomic>
#include <mutex>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

namespace fp8mm {

static thread_local char g_error[512] = "";

int fail(int code, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof g_error, fmt, ap);
    va_end(ap);
    return code;
}

void clear_error() { g_error[0] = '\0'; }

int check_launch(const char* what)
{
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(FP8_ERR_DEVICE, "%s: %s", what, hipGetErrorString(e));
    return FP8_OK;
}

// ---- tuning knobs -------------------------------------------------------------------------------
static std::atomic<int> g_knob[FP8_KNOB_COUNT];
static std::once_flag g_knob_once;

static void seed_knobs()
{
    const char* e;
    if ((e = getenv("FP8MM_CAST_PATH")) && strcmp(e, "bits") == 0) g_knob[FP8_KNOB_CAST_PATH] = 1;
    if ((e = getenv("FP8MM_TILE_N")) && (atoi(e) == 128 || atoi(e) == 256)) g_knob[FP8_KNOB_TILE_N] = atoi(e);
    if ((e = getenv("FP8MM_GROUP_M")) && atoi(e) > 0) g_knob[FP8_KNOB_GROUP_M] = atoi(e);
    if ((e = getenv("FP8MM_GEMM")) && e[0] == 'g') g_knob[FP8_KNOB_GEMM_KERNEL] = 1;
    if (e && e[0] == 'a') g_knob[FP8_KNOB_GEMM_KERNEL] = 2;
    if ((e = getenv("FP8MM_SPLIT_K")) && atoi(e) > 0) g_knob[FP8_KNOB_SPLIT_K] = atoi(e);
    if ((e = getenv("FP8MM_CAST_RUN")) && atoi(e) > 0 && atoi(e) <= 64) g_knob[FP8_KNOB_CAST_RUN] = atoi(e);
    if ((e = getenv("FP8MM_PERSIST")) && atoi(e) >= 0 && atoi(e) <= 2) g_knob[FP8_KNOB_PERSIST] = atoi(e);
    if ((e = getenv("FP8MM_MIXED")) && atoi(e) >= 0 && atoi(e) <= 2) g_knob[FP8_KNOB_MIXED] = atoi(e);
}

int knob(int which)
{
    std::call_once(g_knob_once, seed_knobs);
    return g_knob[which].load(std::memory_order_relaxed);
}

CastPath cast_path() { return knob(FP8_KNOB_CAST_PATH) == 1 ? kCastBits : kCastCvt; }

int fill_gemm_args(const char* who, GemmArgs& g, const uint8_t* A, int fmtA, int transA, const uint8_t* B, int fmtB,
                   int transB, void* C, int64_t M, int64_t N, int64_t K, int out_dtype, float sA, float sB,
                   const float* sA_dev, const float* sB_dev, int flags, void* stream)
{
    clear_error();
    if (flags & ~FP8_GEMM_MFMA8) return fail(FP8_ERR_INVALID_ARG, "%s: unknown flag bits 0x%x", who, flags & ~FP8_GEMM_MFMA8);
    if ((transA != 0 && transA != 1) || (transB != 0 && transB != 1)) return fail(FP8_ERR_INVALID_ARG, "%s: transA/transB must be 0 or 1", who);
    if ((sA_dev == nullptr) != (sB_dev == nullptr)) return fail(FP8_ERR_INVALID_ARG, "%s: give both scales on the device or neither", who);
    if (sA_dev && ((uintptr_t)sA_dev | (uintptr_t)sB_dev) % 4) return fail(FP8_ERR_INVALID_ARG, "%s: scale pointer is misaligned", who);
    if (!valid_format(fmtA) || !valid_format(fmtB))
        return fail(FP8_ERR_INVALID_ARG, "%s: operand formats (%d, %d) are not fp8_format_t", who, fmtA, fmtB);
    if (!valid_dtype(out_dtype)) return fail(FP8_ERR_INVALID_ARG, "%s: out_dtype %d is not an fp8_dtype_t", who, out_dtype);
    if (M < 0 || N < 0 || K < 0) return fail(FP8_ERR_INVALID_ARG, "%s: negative dimension (M=%lld N=%lld K=%lld)", who, (long long)M, (long long)N, (long long)K);
    if (M > 0 && N > 0) {
        if (!C) return fail(FP8_ERR_INVALID_ARG, "%s: C is NULL", who);
        if (K > 0 && (!A || !B)) return fail(FP8_ERR_INVALID_ARG, "%s: A or B is NULL", who);
        const uintptr_t osz = out_dtype == FP8_F32 ? 4 : 2;
        if ((uintptr_t)C % osz) return fail(FP8_ERR_INVALID_ARG, "%s: C is not aligned to its element size", who);
    }
    g = GemmArgs{};
    g.A = A; g.B = B; g.C = C; g.M = M; g.N = N; g.K = K; g.fmtA = fmtA; g.fmtB = fmtB;
    g.transA = transA != 0; g.transB = transB != 0; g.acc = (flags & FP8_GEMM_MFMA8) ? ACC_FP8 : ACC_F16;
    g.ep.sA = sA; g.ep.sB = sB; g.ep.sA_dev = sA_dev; g.ep.sB_dev = sB_dev;
    g.ep.out_kind = out_dtype;                      // fp8_dtype_t values are the first two output kinds
    g.splits = 1;
    g.stream = (hipStream_t)stream;
    return FP8_OK;
}

}  // namespace fp8mm

using namespace fp8mm;

extern "C" {

const char* fp8_last_error(void) { return g_error; }

const char* fp8_version(void) { return "fp8mm 0.2 (gfx950)"; }

int fp8_get_knob(int which)
{
    clear_error();
    if (which < 0 || which >= FP8_KNOB_COUNT) return -fail(FP8_ERR_INVALID_ARG, "fp8_get_knob: %d is not an fp8_knob_t", which);
    return knob(which);
}

int fp8_set_knob(int which, int value)
{
    clear_error();
    if (which < 0 || which >= FP8_KNOB_COUNT) return -fail(FP8_ERR_INVALID_ARG, "fp8_set_knob: %d is not an fp8_knob_t", which);
    bool ok = false;
    switch (which) {
        case FP8_KNOB_CAST_PATH: ok = value == 0 || value == 1; break;
        case FP8_KNOB_TILE_N: ok = value == 0 || value == 128 || value == 256; break;
        case FP8_KNOB_GROUP_M: ok = value >= 0 && value <= 4096; break;
        case FP8_KNOB_GEMM_KERNEL: ok = value >= 0 && value <= 2; break;
        case FP8_KNOB_SPLIT_K: ok = value >= 0 && value <= 64; break;
        case FP8_KNOB_CAST_RUN: ok = value >= 0 && value <= 64; break;
        case FP8_KNOB_PERSIST: ok = value >= 0 && value <= 2; break;
        case FP8_KNOB_MIXED: ok = value >= 0 && value <= 2; break;
    }
    if (!ok) return -fail(FP8_ERR_INVALID_ARG, "fp8_set_knob: value %d is not valid for knob %d", value, which);
    const int old = knob(which);                    // seeds from the environment first
    g_knob[which].store(value, std::memory_order_relaxed);
    return old;
}

int fp8_amax(const void* x, size_t n, int in_dtype, float* amax_out, void* stream)
{
    clear_error();
    if (!valid_dtype(in_dtype)) return fail(FP8_ERR_INVALID_ARG, "fp8_amax: in_dtype %d is not an fp8_dtype_t", in_dtype);
    if (!amax_out) return fail(FP8_ERR_INVALID_ARG, "fp8_amax: amax_out is NULL");
    if (n > 0 && !x) return fail(FP8_ERR_INVALID_ARG, "fp8_amax: x is NULL with n = %zu", n);
    const uintptr_t esz = in_dtype == FP8_F32 ? 4 : 2;
    if ((uintptr_t)x % esz) return fail(FP8_ERR_INVALID_ARG, "fp8_amax: x is not aligned to its element size");
    if ((uintptr_t)amax_out % 4) return fail(FP8_ERR_INVALID_ARG, "fp8_amax: amax_out is not 4-byte aligned");
    return launch_amax(x, n, in_dtype, amax_out, (hipStream_t)stream);
}

int fp8_amax_scale(const void* x, size_t n, int in_dtype, int fmt, float* amax_out, float* scale_out,
                   void* workspace, void* stream)
{
    const char* who = "fp8_amax_scale";
    clear_error();
    if (!valid_dtype(in_dtype)) return fail(FP8_ERR_INVALID_ARG, "%s: in_dtype %d is not an fp8_dtype_t", who, in_dtype);
    if (!valid_format(fmt)) return fail(FP8_ERR_INVALID_ARG, "%s: fmt %d is not an fp8_format_t", who, fmt);
    if (!amax_out) return fail(FP8_ERR_INVALID_ARG, "%s: amax_out is NULL", who);
    if (!workspace) return fail(FP8_ERR_INVALID_ARG, "%s: workspace is NULL", who);
    if (n > 0 && !x) return fail(FP8_ERR_INVALID_ARG, "%s: x is NULL with n = %zu", who, n);
    if ((uintptr_t)x % (in_dtype == FP8_F32 ? 4 : 2)) return fail(FP8_ERR_INVALID_ARG, "%s: x is not aligned to its element size", who);
    if (((uintptr_t)amax_out | (uintptr_t)scale_out | (uintptr_t)workspace) % 4)
        return fail(FP8_ERR_INVALID_ARG, "%s: amax_out, scale_out and workspace must be 4-byte aligned", who);
    return launch_amax_scale(x, n, in_dtype, fmt, amax_out, scale_out, workspace, (hipStream_t)stream);
}

int fp8_amax_scale_multi(int count, const void* const* x, const size_t* n, int in_dtype, const int* fmt,
                         float* amax_out, float* scale_out, void* workspace, void* stream)
{
    const char* who = "fp8_amax_scale_multi";
    clear_error();
    if (count < 0 || count > FP8_MULTI_MAX) return fail(FP8_ERR_INVALID_ARG, "%s: count %d is not in 0..%d", who, count, FP8_MULTI_MAX);
    if (count == 0) return FP8_OK;
    if (!x || !n || !fmt) return fail(FP8_ERR_INVALID_ARG, "%s: x, n or fmt is NULL", who);
    if (!valid_dtype(in_dtype)) return fail(FP8_ERR_INVALID_ARG, "%s: in_dtype %d is not an fp8_dtype_t", who, in_dtype);
    if (!amax_out || !workspace) return fail(FP8_ERR_INVALID_ARG, "%s: amax_out or workspace is NULL", who);
    if (((uintptr_t)amax_out | (uintptr_t)scale_out | (uintptr_t)workspace) % 4)
        return fail(FP8_ERR_INVALID_ARG, "%s: amax_out, scale_out and workspace must be 4-byte aligned", who);
    for (int i = 0; i < count; ++i) {
        if (!valid_format(fmt[i])) return fail(FP8_ERR_INVALID_ARG, "%s: fmt[%d] = %d is not an fp8_format_t", who, i, fmt[i]);
        if (n[i] > 0 && !x[i]) return fail(FP8_ERR_INVALID_ARG, "%s: x[%d] is NULL with n = %zu", who, i, n[i]);
        if ((uintptr_t)x[i] % (in_dtype == FP8_F32 ? 4 : 2)) return fail(FP8_ERR_INVALID_ARG, "%s: x[%d] is not aligned to its element size", who, i);
    }
    return launch_amax_scale_multi(count, x, n, in_dtype, fmt, amax_out, scale_out, workspace, (hipStream_t)stream);
}

int fp8_quantize_multi(int count, const void* const* x, const size_t* n, int in_dtype, const int* fmt,
                       const float* scale_dev, uint8_t* const* q_out, void* stream)
{
    const char* who = "fp8_quantize_multi";
    clear_error();
    if (count < 0 || count > FP8_MULTI_MAX) return fail(FP8_ERR_INVALID_ARG, "%s: count %d is not in 0..%d", who, count, FP8_MULTI_MAX);
    if (count == 0) return FP8_OK;
    if (!x || !n || !fmt || !q_out) return fail(FP8_ERR_INVALID_ARG, "%s: x, n, fmt or q_out is NULL", who);
    if (!valid_dtype(in_dtype)) return fail(FP8_ERR_INVALID_ARG, "%s: in_dtype %d is not an fp8_dtype_t", who, in_dtype);
    if (!scale_dev || (uintptr_t)scale_dev % 4) return fail(FP8_ERR_INVALID_ARG, "%s: scale_dev is NULL or misaligned", who);
    for (int i = 0; i < count; ++i) {
        if (!valid_format(fmt[i])) return fail(FP8_ERR_INVALID_ARG, "%s: fmt[%d] = %d is not an fp8_format_t", who, i, fmt[i]);
        if (n[i] > 0 && (!x[i] || !q_out[i])) return fail(FP8_ERR_INVALID_ARG, "%s: NULL tensor pointer %d with n = %zu", who, i, n[i]);
        if ((uintptr_t)x[i] % (in_dtype == FP8_F32 ? 4 : 2)) return fail(FP8_ERR_INVALID_ARG, "%s: x[%d] is not aligned to its element size", who, i);
    }
    return launch_quantize_multi(count, x, n, in_dtype, fmt, scale_dev, q_out, (hipStream_t)stream);
}

float fp8_scale_from_amax_host(float amax, int fmt)
{
    clear_error();
    if (!valid_format(fmt)) {
        fail(FP8_ERR_INVALID_ARG, "fp8_scale_from_amax_host: fmt %d is not an fp8_format_t", fmt);
        return 1.0f;
    }
    return scale_from_amax_host(amax, fmt);
}

int fp8_scale_from_amax(const float* amax, int fmt, float* scale_out, void* stream)
{
    clear_error();
    if (!valid_format(fmt)) return fail(FP8_ERR_INVALID_ARG, "fp8_scale_from_amax: fmt %d is not an fp8_format_t", fmt);
    if (!amax || !scale_out) return fail(FP8_ERR_INVALID_ARG, "fp8_scale_from_amax: NULL pointer");
    if (((uintptr_t)amax | (uintptr_t)scale_out) % 4) return fail(FP8_ERR_INVALID_ARG, "fp8_scale_from_amax: pointers must be 4-byte aligned");
    return launch_scale_from_amax(amax, fmt, scale_out, (hipStream_t)stream);
}

static int quantize_checked(const char* who, const void* x, size_t n, int in_dtype, int fmt, float scale,
                            const float* scale_dev, uint8_t* q_out, void* stream, bool saturate = true)
{
    clear_error();
    if (!valid_dtype(in_dtype)) return fail(FP8_ERR_INVALID_ARG, "%s: in_dtype %d is not an fp8_dtype_t", who, in_dtype);
    if (!valid_format(fmt)) return fail(FP8_ERR_INVALID_ARG, "%s: fmt %d is not an fp8_format_t", who, fmt);
    if (n > 0 && (!x || !q_out)) return fail(FP8_ERR_INVALID_ARG, "%s: NULL tensor pointer with n = %zu", who, n);
    const uintptr_t esz = in_dtype == FP8_F32 ? 4 : 2;
    if ((uintptr_t)x % esz) return fail(FP8_ERR_INVALID_ARG, "%s: x is not aligned to its element size", who);
    return launch_quantize(x, n, in_dtype, fmt, scale, scale_dev, saturate, q_out, (hipStream_t)stream);
}

int fp8_quantize(const void* x, size_t n, int in_dtype, int fmt, float scale, uint8_t* q_out, void* stream)
{
    return quantize_checked("fp8_quantize", x, n, in_dtype, fmt, scale, nullptr, q_out, stream);
}

int fp8_quantize_dscale(const void* x, size_t n, int in_dtype, int fmt, const float* scale,
                        uint8_t* q_out, void* stream)
{
    if (!scale || (uintptr_t)scale % 4) {
        clear_error();
        return fail(FP8_ERR_INVALID_ARG, "fp8_quantize_dscale: scale pointer is NULL or misaligned");
    }
    return quantize_checked("fp8_quantize_dscale", x, n, in_dtype, fmt, 0.0f, scale, q_out, stream);
}

int fp8_quantize_ex(const void* x, size_t n, int in_dtype, int fmt, float scale, const float* scale_dev,
                    int flags, uint8_t* q_out, void* stream)
{
    if (flags & ~FP8_QUANT_NOSAT) {
        clear_error();
        return fail(FP8_ERR_INVALID_ARG, "fp8_quantize_ex: unknown flag bits 0x%x", flags & ~FP8_QUANT_NOSAT);
    }
    if (scale_dev && (uintptr_t)scale_dev % 4) {
        clear_error();
        return fail(FP8_ERR_INVALID_ARG, "fp8_quantize_ex: scale_dev is misaligned");
    }
    return quantize_checked("fp8_quantize_ex", x, n, in_dtype, fmt, scale, scale_dev, q_out, stream,
                            !(flags & FP8_QUANT_NOSAT));
}

int fp8_dequantize(const uint8_t* q, size_t n, int fmt, float scale, const float* scale_dev,
                   int out_dtype, void* out, void* stream)
{
    clear_error();
    if (!valid_format(fmt)) return fail(FP8_ERR_INVALID_ARG, "fp8_dequantize: fmt %d is not an fp8_format_t", fmt);
    if (!valid_dtype(out_dtype)) return fail(FP8_ERR_INVALID_ARG, "fp8_dequantize: out_dtype %d is not an fp8_dtype_t", out_dtype);
    if (n > 0 && (!q || !out)) return fail(FP8_ERR_INVALID_ARG, "fp8_dequantize: NULL tensor pointer with n = %zu", n);
    if ((uintptr_t)out % (out_dtype == FP8_F32 ? 4 : 2)) return fail(FP8_ERR_INVALID_ARG, "fp8_dequantize: out is not aligned to its element size");
    if (scale_dev && (uintptr_t)scale_dev % 4) return fail(FP8_ERR_INVALID_ARG, "fp8_dequantize: scale_dev is misaligned");
    return launch_dequantize(q, n, fmt, scale, scale_dev, out_dtype, out, (hipStream_t)stream);
}

// ---- scaling-recipe variants of the amax / cast steps ------------------------------------------
static int check_tensor(const char* who, const void* x, int in_dtype, bool nonempty)
{
    if (!valid_dtype(in_dtype)) return fail(FP8_ERR_INVALID_ARG, "%s: in_dtype %d is not an fp8_dtype_t", who, in_dtype);
    if (nonempty && !x) return fail(FP8_ERR_INVALID_ARG, "%s: x is NULL", who);
    if ((uintptr_t)x % (in_dtype == FP8_F32 ? 4 : 2)) return fail(FP8_ERR_INVALID_ARG, "%s: x is not aligned to its element size", who);
    return FP8_OK;
}

static int check_f32_ptr(const char* who, const char* name, const void* p, bool required)
{
    if (required && !p) return fail(FP8_ERR_INVALID_ARG, "%s: %s is NULL", who, name);
    if ((uintptr_t)p % 4) return fail(FP8_ERR_INVALID_ARG, "%s: %s is misaligned", who, name);
    return FP8_OK;
}

int fp8_quantize_amax(const void* x, size_t n, int in_dtype, int fmt, const float* scale_dev,
                      uint8_t* q_out, float* amax_out, void* stream)
{
    const char* who = "fp8_quantize_amax";
    clear_error();
    if (!valid_format(fmt)) return fail(FP8_ERR_INVALID_ARG, "%s: fmt %d is not an fp8_format_t", who, fmt);
    if (int e = check_tensor(who, x, in_dtype, n > 0)) return e;
    if (n > 0 && !q_out) return fail(FP8_ERR_INVALID_ARG, "%s: q_out is NULL", who);
    if (int e = check_f32_ptr(who, "scale_dev", scale_dev, n > 0)) return e;
    if (int e = check_f32_ptr(who, "amax_out", amax_out, true)) return e;
    return launch_quantize_amax(x, n, in_dtype, fmt, scale_dev, q_out, amax_out, (hipStream_t)stream);
}

int fp8_quantize_sr(const void* x, size_t n, int in_dtype, int fmt, float scale, const float* scale_dev,
                    uint64_t seed, uint8_t* q_out, void* stream)
{
    const char* who = "fp8_quantize_sr";
    clear_error();
    if (!valid_format(fmt)) return fail(FP8_ERR_INVALID_ARG, "%s: fmt %d is not an fp8_format_t", who, fmt);
    if (int e = check_tensor(who, x, in_dtype, n > 0)) return e;
    if (n > 0 && !q_out) return fail(FP8_ERR_INVALID_ARG, "%s: q_out is NULL", who);
    if (int e = check_f32_ptr(who, "scale_dev", scale_dev, false)) return e;
    return launch_quantize_sr(x, n, in_dtype, fmt, scale, scale_dev, seed, q_out, (hipStream_t)stream);
}

int fp8_scale_from_amax_history(const float* amax_history, size_t len, int fmt, float* scale_out, void* stream)
{
    const char* who = "fp8_scale_from_amax_history";
    clear_error();
    if (!valid_format(fmt)) return fail(FP8_ERR_INVALID_ARG, "%s: fmt %d is not an fp8_format_t", who, fmt);
    if (int e = check_f32_ptr(who, "amax_history", amax_history, len > 0)) return e;
    if (int e = check_f32_ptr(who, "scale_out", scale_out, true)) return e;
    return launch_scale_from_history(amax_history, len, fmt, scale_out, (hipStream_t)stream);
}

int fp8_scale_from_amax_n(const float* amax, size_t n, int fmt, float* scale_out, void* stream)
{
    const char* who = "fp8_scale_from_amax_n";
    clear_error();
    if (!valid_format(fmt)) return fail(FP8_ERR_INVALID_ARG, "%s: fmt %d is not an fp8_format_t", who, fmt);
    if (int e = check_f32_ptr(who, "amax", amax, n > 0)) return e;
    if (int e = check_f32_ptr(who, "scale_out", scale_out, n > 0)) return e;
    return launch_scale_n(amax, n, fmt, scale_out, (hipStream_t)stream);
}

int fp8_amax_rows(const void* x, int64_t rows, int64_t cols, int in_dtype, float* amax_out, void* stream)
{
    const char* who = "fp8_amax_rows";
    clear_error();
    if (rows < 0 || cols < 0) return fail(FP8_ERR_INVALID_ARG, "%s: negative dimension (rows=%lld cols=%lld)", who, (long long)rows, (long long)cols);
    if (int e = check_tensor(who, x, in_dtype, rows > 0 && cols > 0)) return e;
    if (int e = check_f32_ptr(who, "amax_out", amax_out, rows > 0)) return e;
    return launch_amax_rows(x, rows, cols, in_dtype, amax_out, (hipStream_t)stream);
}

int fp8_quantize_rows(const void* x, int64_t rows, int64_t cols, int in_dtype, int fmt,
                      const float* scale_dev, uint8_t* q_out, void* stream)
{
    const char* who = "fp8_quantize_rows";
    clear_error();
    if (!valid_format(fmt)) return fail(FP8_ERR_INVALID_ARG, "%s: fmt %d is not an fp8_format_t", who, fmt);
    if (rows < 0 || cols < 0) return fail(FP8_ERR_INVALID_ARG, "%s: negative dimension (rows=%lld cols=%lld)", who, (long long)rows, (long long)cols);
    const bool work = rows > 0 && cols > 0;
    if (int e = check_tensor(who, x, in_dtype, work)) return e;
    if (work && !q_out) return fail(FP8_ERR_INVALID_ARG, "%s: q_out is NULL", who);
    if (int e = check_f32_ptr(who, "scale_dev", scale_dev, work)) return e;
    return launch_quantize_rows(x, rows, cols, in_dtype, fmt, scale_dev, q_out, (hipStream_t)stream);
}

int fp8_quantize_transpose(const void* x, int64_t rows, int64_t cols, int in_dtype, int fmt,
                           const float* scale_dev, uint8_t* q_out, uint8_t* qt_out, void* stream)
{
    const char* who = "fp8_quantize_transpose";
    clear_error();
    if (!valid_format(fmt)) return fail(FP8_ERR_INVALID_ARG, "%s: fmt %d is not an fp8_format_t", who, fmt);
    if (rows < 0 || cols < 0) return fail(FP8_ERR_INVALID_ARG, "%s: negative dimension (rows=%lld cols=%lld)", who, (long long)rows, (long long)cols);
    const bool work = rows > 0 && cols > 0;
    if (int e = check_tensor(who, x, in_dtype, work)) return e;
    if (work && !qt_out) return fail(FP8_ERR_INVALID_ARG, "%s: qt_out is NULL", who);
    if (int e = check_f32_ptr(who, "scale_dev", scale_dev, work)) return e;
    return launch_quantize_transpose(x, rows, cols, in_dtype, fmt, scale_dev, q_out, qt_out, (hipStream_t)stream);
}

static int gemm_checked(const char* who, const uint8_t* A, int fmtA, const uint8_t* B, int fmtB, void* C,
                        int64_t M, int64_t N, int64_t K, int out_dtype, float sA, float sB,
                        const float* sA_dev, const float* sB_dev, bool fp8_accumulate, void* stream,
                        bool transA = false, bool transB = false)
{
    GemmArgs g{};
    if (int e = fill_gemm_args(who, g, A, fmtA, transA, B, fmtB, transB, C, M, N, K, out_dtype, sA, sB, sA_dev, sB_dev,
                               fp8_accumulate ? FP8_GEMM_MFMA8 : 0, stream))
        return e;
    return launch_gemm(g);
}

int fp8_gemm(const uint8_t* A, int fmtA, float sA, const uint8_t* B, int fmtB, float sB,
             void* C, int64_t M, int64_t N, int64_t K, int out_dtype, void* stream)
{
    return gemm_checked("fp8_gemm", A, fmtA, B, fmtB, C, M, N, K, out_dtype, sA, sB, nullptr, nullptr, false, stream);
}

int fp8_gemm_mfma8(const uint8_t* A, int fmtA, float sA, const uint8_t* B, int fmtB, float sB,
                   void* C, int64_t M, int64_t N, int64_t K, int out_dtype, void* stream)
{
    return gemm_checked("fp8_gemm_mfma8", A, fmtA, B, fmtB, C, M, N, K, out_dtype, sA, sB, nullptr, nullptr, true, stream);
}

int fp8_gemm_dscale(const uint8_t* A, int fmtA, const float* sA, const uint8_t* B, int fmtB, const float* sB,
                    void* C, int64_t M, int64_t N, int64_t K, int out_dtype, void* stream)
{
    if (!sA || !sB || ((uintptr_t)sA | (uintptr_t)sB) % 4) {
        clear_error();
        return fail(FP8_ERR_INVALID_ARG, "fp8_gemm_dscale: scale pointer is NULL or misaligned");
    }
    return gemm_checked("fp8_gemm_dscale", A, fmtA, B, fmtB, C, M, N, K, out_dtype, 1.0f, 1.0f, sA, sB, false, stream);
}

int fp8_gemm_mfma8_dscale(const uint8_t* A, int fmtA, const float* sA, const uint8_t* B, int fmtB, const float* sB,
                          void* C, int64_t M, int64_t N, int64_t K, int out_dtype, void* stream)
{
    if (!sA || !sB || ((uintptr_t)sA | (uintptr_t)sB) % 4) {
        clear_error();
        return fail(FP8_ERR_INVALID_ARG, "fp8_gemm_mfma8_dscale: scale pointer is NULL or misaligned");
    }
    return gemm_checked("fp8_gemm_mfma8_dscale", A, fmtA, B, fmtB, C, M, N, K, out_dtype, 1.0f, 1.0f, sA, sB, true, stream);
}

int fp8_gemm_ex(const uint8_t* A, int fmtA, int transA, const uint8_t* B, int fmtB, int transB,
                void* C, int64_t M, int64_t N, int64_t K, int out_dtype,
                float sA, float sB, const float* sA_dev, const float* sB_dev, int flags, void* stream)
{
    GemmArgs g{};
    if (int e = fill_gemm_args("fp8_gemm_ex", g, A, fmtA, transA, B, fmtB, transB, C, M, N, K, out_dtype, sA, sB, sA_dev,
                               sB_dev, flags, stream))
        return e;
    return launch_gemm(g);
}

int fp8_gemm_fused(const uint8_t* A, int fmtA, int transA, const uint8_t* B, int fmtB, int transB,
                   void* D, int out_kind, int64_t M, int64_t N, int64_t K,
                   const float* sA_dev, int64_t nsA, const float* sB_dev, int64_t nsB,
                   const float* sD_dev, float* amax_out, int flags, void* stream)
{
    const char* who = "fp8_gemm_fused";
    clear_error();
    if (flags & ~FP8_GEMM_MFMA8) return fail(FP8_ERR_INVALID_ARG, "%s: unknown flag bits 0x%x", who, flags & ~FP8_GEMM_MFMA8);
    if ((transA != 0 && transA != 1) || (transB != 0 && transB != 1)) return fail(FP8_ERR_INVALID_ARG, "%s: transA/transB must be 0 or 1", who);
    if (!valid_format(fmtA) || !valid_format(fmtB))
        return fail(FP8_ERR_INVALID_ARG, "%s: operand formats (%d, %d) are not fp8_format_t", who, fmtA, fmtB);
    if (out_kind < FP8_OUT_F32 || out_kind > FP8_OUT_E5M2) return fail(FP8_ERR_INVALID_ARG, "%s: out_kind %d is not an fp8_out_t", who, out_kind);
    if (M < 0 || N < 0 || K < 0) return fail(FP8_ERR_INVALID_ARG, "%s: negative dimension (M=%lld N=%lld K=%lld)", who, (long long)M, (long long)N, (long long)K);
    if (!sA_dev || !sB_dev) return fail(FP8_ERR_INVALID_ARG, "%s: sA_dev or sB_dev is NULL", who);
    if (nsA != 1 && nsA != M) return fail(FP8_ERR_INVALID_ARG, "%s: nsA = %lld is neither 1 nor M", who, (long long)nsA);
    if (nsB != 1 && nsB != N) return fail(FP8_ERR_INVALID_ARG, "%s: nsB = %lld is neither 1 nor N", who, (long long)nsB);
    if (((uintptr_t)sA_dev | (uintptr_t)sB_dev | (uintptr_t)sD_dev | (uintptr_t)amax_out) % 4)
        return fail(FP8_ERR_INVALID_ARG, "%s: a scale or amax pointer is misaligned", who);
    if (sD_dev && out_kind < FP8_OUT_E4M3) return fail(FP8_ERR_INVALID_ARG, "%s: sD_dev applies to FP8 outputs only", who);
    if (M > 0 && N > 0) {
        if (!D) return fail(FP8_ERR_INVALID_ARG, "%s: D is NULL", who);
        if (K > 0 && (!A || !B)) return fail(FP8_ERR_INVALID_ARG, "%s: A or B is NULL", who);
        if ((uintptr_t)D % (uintptr_t)out_elem_size(out_kind)) return fail(FP8_ERR_INVALID_ARG, "%s: D is not aligned to its element size", who);
    }
    GemmArgs g{};
    g.A = A; g.B = B; g.C = D; g.M = M; g.N = N; g.K = K; g.fmtA = fmtA; g.fmtB = fmtB;
    g.transA = transA != 0; g.transB = transB != 0; g.acc = (flags & FP8_GEMM_MFMA8) ? ACC_FP8 : ACC_F16;
    g.ep.sA = 1.0f; g.ep.sB = 1.0f; g.ep.sA_dev = sA_dev; g.ep.sB_dev = sB_dev; g.ep.sD_dev = sD_dev;
    g.ep.amax_out = amax_out; g.ep.out_kind = out_kind;
    g.ep.a_per_row = nsA == M && M != 1;
    g.ep.b_per_col = nsB == N && N != 1;
    g.splits = 1;
    g.stream = (hipStream_t)stream;
    return launch_gemm(g);
}

int fp8_scaled_gemm(const void* a, const void* b, int in_dtype, int transA, int transB,
                    int64_t M, int64_t N, int64_t K, int fmtA, int fmtB,
                    uint8_t* qa_out, uint8_t* qb_out, float* amax_out, float* scale_out, void* workspace,
                    void* C, int out_dtype, int flags, void* stream)
{
    const char* who = "fp8_scaled_gemm";
    // every check of the three steps first: nothing is launched unless all of them can be
    GemmArgs g{};
    if (int e = fill_gemm_args(who, g, qa_out, fmtA, transA, qb_out, fmtB, transB, C, M, N, K, out_dtype, 1.0f, 1.0f,
                               scale_out, scale_out ? scale_out + 1 : nullptr, flags, stream))
        return e;
    if (!valid_dtype(in_dtype)) return fail(FP8_ERR_INVALID_ARG, "%s: in_dtype %d is not an fp8_dtype_t", who, in_dtype);
    if (!amax_out || !scale_out || !workspace) return fail(FP8_ERR_INVALID_ARG, "%s: amax_out, scale_out or workspace is NULL", who);
    if (((uintptr_t)amax_out | (uintptr_t)scale_out | (uintptr_t)workspace) % 4)
        return fail(FP8_ERR_INVALID_ARG, "%s: amax_out, scale_out and workspace must be 4-byte aligned", who);
    const void* x[2] = {a, b};
    const size_t n[2] = {(size_t)M * (size_t)K, (size_t)K * (size_t)N};
    const int fmt[2] = {fmtA, fmtB};
    uint8_t* q[2] = {qa_out, qb_out};
    for (int i = 0; i < 2; ++i) {
        if (n[i] > 0 && (!x[i] || !q[i])) return fail(FP8_ERR_INVALID_ARG, "%s: NULL operand or FP8 output %d with %zu elements", who, i, n[i]);
        if ((uintptr_t)x[i] % (in_dtype == FP8_F32 ? 4 : 2)) return fail(FP8_ERR_INVALID_ARG, "%s: operand %d is not aligned to its element size", who, i);
    }
    if (int e = launch_amax_scale_multi(2, x, n, in_dtype, fmt, amax_out, scale_out, workspace, (hipStream_t)stream)) return e;
    if (int e = launch_quantize_multi(2, x, n, in_dtype, fmt, scale_out, q, (hipStream_t)stream)) return e;
    return launch_gemm(g);
}

int fp8_gemm_plan(const uint8_t* A, int transA, const uint8_t* B, int transB, const void* C,
                  int64_t M, int64_t N, int64_t K, const float* sB_per_column)
{
    clear_error();
    if (M < 0 || N < 0 || K < 0) return -fail(FP8_ERR_INVALID_ARG, "fp8_gemm_plan: negative dimension (M=%lld N=%lld K=%lld)", (long long)M, (long long)N, (long long)K);
    if ((transA != 0 && transA != 1) || (transB != 0 && transB != 1)) return -fail(FP8_ERR_INVALID_ARG, "fp8_gemm_plan: transA/transB must be 0 or 1");
    if (M == 0 || N == 0 || K == 0) return FP8_PLAN_NO_GEMM;
    GemmArgs g{};
    g.A = A; g.B = B; g.C = const_cast<void*>(C); g.M = M; g.N = N; g.K = K;
    g.transA = transA != 0; g.transB = transB != 0;
    g.ep.sB_dev = sB_per_column; g.ep.b_per_col = sB_per_column != nullptr;
    const GemmPlan plan = plan_gemm(g);
    const int kernel = plan.kernel == GEMM_GENERIC ? FP8_PLAN_FMA_KERNEL
                     : plan.kernel == GEMM_MFMA_ANY ? FP8_PLAN_MFMA_ANY
                     : plan.kernel == GEMM_TILED_MIXED ? FP8_PLAN_TILED_MIXED
                     : plan.kernel == GEMM_TILED_128 ? FP8_PLAN_TILED_256x128 : FP8_PLAN_TILED_256x256;
    return kernel | (plan.elementwise_stores ? FP8_PLAN_ELEMENTWISE_STORES : 0) | (plan.persistent ? FP8_PLAN_PERSISTENT : 0);
}

}  // extern "C"
