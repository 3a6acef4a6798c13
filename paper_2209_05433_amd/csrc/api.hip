// extern "C" entry points of libfp8mm: argument validation, then one launcher each.
#include "common.hpp"

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

CastPath cast_path()
{
    const char* e = getenv("FP8MM_CAST_PATH");     // read per call: a test may switch it
    return (e && strcmp(e, "bits") == 0) ? kCastBits : kCastCvt;
}

}  // namespace fp8mm

using namespace fp8mm;

extern "C" {

const char* fp8_last_error(void) { return g_error; }

const char* fp8_version(void) { return "fp8mm 0.1 (gfx950)"; }

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

static int gemm_checked(const char* who, const uint8_t* A, int fmtA, const uint8_t* B, int fmtB, void* C,
                        int64_t M, int64_t N, int64_t K, int out_dtype, float sA, float sB,
                        const float* sA_dev, const float* sB_dev, bool fp8_accumulate, void* stream,
                        bool transA = false, bool transB = false)
{
    clear_error();
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
    return launch_gemm(A, fmtA, B, fmtB, C, M, N, K, out_dtype, sA, sB, sA_dev, sB_dev, transA, transB, fp8_accumulate, (hipStream_t)stream);
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
    clear_error();
    if (flags & ~FP8_GEMM_MFMA8) return fail(FP8_ERR_INVALID_ARG, "fp8_gemm_ex: unknown flag bits 0x%x", flags & ~FP8_GEMM_MFMA8);
    if ((transA != 0 && transA != 1) || (transB != 0 && transB != 1)) return fail(FP8_ERR_INVALID_ARG, "fp8_gemm_ex: transA/transB must be 0 or 1");
    if ((sA_dev == nullptr) != (sB_dev == nullptr)) return fail(FP8_ERR_INVALID_ARG, "fp8_gemm_ex: give both scales on the device or neither");
    if (sA_dev && ((uintptr_t)sA_dev | (uintptr_t)sB_dev) % 4) return fail(FP8_ERR_INVALID_ARG, "fp8_gemm_ex: scale pointer is misaligned");
    return gemm_checked("fp8_gemm_ex", A, fmtA, B, fmtB, C, M, N, K, out_dtype, sA, sB, sA_dev, sB_dev,
                        (flags & FP8_GEMM_MFMA8) != 0, stream, transA != 0, transB != 0);
}

}  // extern "C"
