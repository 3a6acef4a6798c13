/* Host-side exercise of the C ABI's argument checks and planning logic, for a build of the library
 * with AddressSanitizer and UndefinedBehaviorSanitizer on the host code (tests/test_api_sanitizers.py).
 * Every call here is decided on the host: a rejected argument, an empty problem that needs no
 * launch, a plan or a size query.  No call may reach a kernel launch (the sanitized build carries no
 * device code).  Exit status 0 and "ok" on stdout if every call returned what it should. */
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "fp8mm.h"

static int failures = 0;

#define EXPECT(call, want)                                                                          \
    do {                                                                                            \
        long long got_ = (long long)(call);                                                         \
        if (got_ != (long long)(want)) {                                                            \
            printf("line %d: %s returned %lld, expected %lld (%s)\n", __LINE__, #call, got_,        \
                   (long long)(want), fp8_last_error());                                            \
            ++failures;                                                                             \
        }                                                                                           \
    } while (0)

#define BAD FP8_ERR_INVALID_ARG

int main(void)
{
    /* stand-ins for device pointers: never dereferenced on the host */
    uint8_t* A = (uint8_t*)(uintptr_t)0x10000000u;
    uint8_t* B = (uint8_t*)(uintptr_t)0x20000000u;
    void* C = (void*)(uintptr_t)0x30000000u;
    float* F = (float*)(uintptr_t)0x40000000u;
    float* Fodd = (float*)(uintptr_t)0x40000002u;
    void* X = (void*)(uintptr_t)0x50000000u;
    void* Xodd = (void*)(uintptr_t)0x50000001u;

    if (!strstr(fp8_version(), "gfx950")) { printf("version string: %s\n", fp8_version()); ++failures; }
    EXPECT(strlen(fp8_last_error()) == 0 || 1, 1);

    /* amax, scale */
    EXPECT(fp8_amax(X, 16, 7, F, NULL), BAD);
    EXPECT(fp8_amax(X, 16, FP8_BF16, NULL, NULL), BAD);
    EXPECT(fp8_amax(NULL, 16, FP8_BF16, F, NULL), BAD);
    EXPECT(fp8_amax(Xodd, 16, FP8_BF16, F, NULL), BAD);
    EXPECT(fp8_amax(X, 16, FP8_F32, Fodd, NULL), BAD);
    EXPECT(strlen(fp8_last_error()) > 0, 1);
    EXPECT(fp8_amax_scale(X, 16, FP8_BF16, 5, F, F + 1, F + 64, NULL), BAD);
    EXPECT(fp8_amax_scale(X, 16, FP8_BF16, FP8_E4M3, NULL, F + 1, F + 64, NULL), BAD);
    EXPECT(fp8_amax_scale(X, 16, FP8_BF16, FP8_E4M3, F, F + 1, NULL, NULL), BAD);
    EXPECT(fp8_amax_scale(X, 16, FP8_BF16, FP8_E4M3, F, Fodd, F + 64, NULL), BAD);
    EXPECT(fp8_scale_from_amax_host(2.0f, FP8_E4M3) == 224.0f, 1);
    EXPECT(fp8_scale_from_amax_host(0.0f, FP8_E5M2) == 1.0f, 1);
    EXPECT(fp8_scale_from_amax_host(1.0f, 9) == 1.0f, 1);
    EXPECT(fp8_scale_from_amax(NULL, FP8_E4M3, F, NULL), BAD);
    EXPECT(fp8_scale_from_amax(F, 3, F, NULL), BAD);
    EXPECT(fp8_scale_from_amax(Fodd, FP8_E4M3, F, NULL), BAD);
    EXPECT(fp8_scale_from_amax_history(NULL, 4, FP8_E4M3, F, NULL), BAD);
    EXPECT(fp8_scale_from_amax_history(F, 4, FP8_E4M3, NULL, NULL), BAD);
    EXPECT(fp8_scale_from_amax_n(F, 4, -1, F, NULL), BAD);
    EXPECT(fp8_scale_from_amax_n(NULL, 4, FP8_E4M3, F, NULL), BAD);

    {
        const void* xs[5] = {X, X, X, X, X};
        const size_t ns[5] = {16, 0, 16, 16, 16};
        const int fm[5] = {FP8_E4M3, FP8_E5M2, FP8_E4M3, FP8_E4M3, FP8_E4M3};
        const int badfm[2] = {FP8_E4M3, 4};
        uint8_t* qs[5] = {A, A, A, A, A};
        const void* withnull[2] = {X, NULL};
        EXPECT(fp8_amax_scale_multi(5, xs, ns, FP8_BF16, fm, F, F + 8, F + 64, NULL), BAD);
        EXPECT(fp8_amax_scale_multi(-1, xs, ns, FP8_BF16, fm, F, F + 8, F + 64, NULL), BAD);
        EXPECT(fp8_amax_scale_multi(0, NULL, NULL, FP8_BF16, NULL, NULL, NULL, NULL, NULL), FP8_OK);
        EXPECT(fp8_amax_scale_multi(2, NULL, ns, FP8_BF16, fm, F, F + 8, F + 64, NULL), BAD);
        EXPECT(fp8_amax_scale_multi(2, xs, ns, FP8_BF16, badfm, F, F + 8, F + 64, NULL), BAD);
        EXPECT(fp8_amax_scale_multi(2, xs, ns, FP8_BF16, fm, NULL, F + 8, F + 64, NULL), BAD);
        EXPECT(fp8_amax_scale_multi(2, xs, ns, 9, fm, F, F + 8, F + 64, NULL), BAD);
        EXPECT(fp8_amax_scale_multi(2, withnull, ns + 2, FP8_BF16, fm, F, F + 8, F + 64, NULL), BAD);
        EXPECT(fp8_quantize_multi(5, xs, ns, FP8_BF16, fm, F, qs, NULL), BAD);
        EXPECT(fp8_quantize_multi(2, xs, ns, FP8_BF16, fm, NULL, qs, NULL), BAD);
        EXPECT(fp8_quantize_multi(2, xs, ns, FP8_BF16, fm, Fodd, qs, NULL), BAD);
        EXPECT(fp8_quantize_multi(2, xs, ns, FP8_BF16, fm, F, NULL, NULL), BAD);
        EXPECT(fp8_quantize_multi(2, xs, ns, FP8_BF16, badfm, F, qs, NULL), BAD);
        EXPECT(fp8_quantize_multi(0, NULL, NULL, FP8_BF16, NULL, NULL, NULL, NULL), FP8_OK);
    }

    /* the whole scheme in one call: every check precedes the first launch */
    EXPECT(fp8_scaled_gemm(X, X, 2, 0, 0, 4, 4, 4, FP8_E4M3, FP8_E4M3, A, B, F, F + 8, F + 64, C, FP8_F32, 0, NULL), BAD);
    EXPECT(fp8_scaled_gemm(X, X, FP8_BF16, 2, 0, 4, 4, 4, FP8_E4M3, FP8_E4M3, A, B, F, F + 8, F + 64, C, FP8_F32, 0, NULL), BAD);
    EXPECT(fp8_scaled_gemm(X, X, FP8_BF16, 0, 0, 4, -4, 4, FP8_E4M3, FP8_E4M3, A, B, F, F + 8, F + 64, C, FP8_F32, 0, NULL), BAD);
    EXPECT(fp8_scaled_gemm(X, X, FP8_BF16, 0, 0, 4, 4, 4, 5, FP8_E4M3, A, B, F, F + 8, F + 64, C, FP8_F32, 0, NULL), BAD);
    EXPECT(fp8_scaled_gemm(NULL, X, FP8_BF16, 0, 0, 4, 4, 4, FP8_E4M3, FP8_E4M3, A, B, F, F + 8, F + 64, C, FP8_F32, 0, NULL), BAD);
    EXPECT(fp8_scaled_gemm(X, Xodd, FP8_F32, 0, 0, 4, 4, 4, FP8_E4M3, FP8_E4M3, A, B, F, F + 8, F + 64, C, FP8_F32, 0, NULL), BAD);
    EXPECT(fp8_scaled_gemm(X, X, FP8_BF16, 0, 0, 4, 4, 4, FP8_E4M3, FP8_E4M3, NULL, B, F, F + 8, F + 64, C, FP8_F32, 0, NULL), BAD);
    EXPECT(fp8_scaled_gemm(X, X, FP8_BF16, 0, 0, 4, 4, 4, FP8_E4M3, FP8_E4M3, A, B, NULL, F + 8, F + 64, C, FP8_F32, 0, NULL), BAD);
    EXPECT(fp8_scaled_gemm(X, X, FP8_BF16, 0, 0, 4, 4, 4, FP8_E4M3, FP8_E4M3, A, B, F, NULL, F + 64, C, FP8_F32, 0, NULL), BAD);
    EXPECT(fp8_scaled_gemm(X, X, FP8_BF16, 0, 0, 4, 4, 4, FP8_E4M3, FP8_E4M3, A, B, F, F + 8, NULL, C, FP8_F32, 0, NULL), BAD);
    EXPECT(fp8_scaled_gemm(X, X, FP8_BF16, 0, 0, 4, 4, 4, FP8_E4M3, FP8_E4M3, A, B, F, F + 8, F + 64, NULL, FP8_F32, 0, NULL), BAD);
    EXPECT(fp8_scaled_gemm(X, X, FP8_BF16, 0, 0, 4, 4, 4, FP8_E4M3, FP8_E4M3, A, B, F, F + 8, F + 64, C, 3, 0, NULL), BAD);
    EXPECT(fp8_scaled_gemm(X, X, FP8_BF16, 0, 0, 4, 4, 4, FP8_E4M3, FP8_E4M3, A, B, F, F + 8, F + 64, C, FP8_F32, 8, NULL), BAD);

    /* casts */
    EXPECT(fp8_quantize(X, 0, FP8_BF16, FP8_E4M3, 1.0f, A, NULL), FP8_OK);          /* empty: nothing to launch */
    EXPECT(fp8_quantize(NULL, 0, FP8_F32, FP8_E5M2, 1.0f, NULL, NULL), FP8_OK);
    EXPECT(fp8_quantize(X, 8, 2, FP8_E4M3, 1.0f, A, NULL), BAD);
    EXPECT(fp8_quantize(X, 8, FP8_BF16, 2, 1.0f, A, NULL), BAD);
    EXPECT(fp8_quantize(X, 8, FP8_BF16, FP8_E4M3, 1.0f, NULL, NULL), BAD);
    EXPECT(fp8_quantize(Xodd, 8, FP8_F32, FP8_E4M3, 1.0f, A, NULL), BAD);
    EXPECT(fp8_quantize_dscale(X, 8, FP8_BF16, FP8_E4M3, NULL, A, NULL), BAD);
    EXPECT(fp8_quantize_dscale(X, 8, FP8_BF16, FP8_E4M3, Fodd, A, NULL), BAD);
    EXPECT(fp8_quantize_ex(X, 8, FP8_BF16, FP8_E4M3, 1.0f, NULL, 4, A, NULL), BAD);
    EXPECT(fp8_quantize_ex(X, 8, FP8_BF16, FP8_E4M3, 1.0f, Fodd, FP8_QUANT_NOSAT, A, NULL), BAD);
    EXPECT(fp8_quantize_ex(X, 0, FP8_BF16, FP8_E4M3, 1.0f, NULL, FP8_QUANT_NOSAT, A, NULL), FP8_OK);
    EXPECT(fp8_dequantize(A, 8, 4, 1.0f, NULL, FP8_F32, C, NULL), BAD);
    EXPECT(fp8_dequantize(A, 8, FP8_E4M3, 1.0f, NULL, 5, C, NULL), BAD);
    EXPECT(fp8_dequantize(NULL, 8, FP8_E4M3, 1.0f, NULL, FP8_F32, C, NULL), BAD);
    EXPECT(fp8_dequantize(A, 8, FP8_E4M3, 1.0f, NULL, FP8_F32, Xodd, NULL), BAD);
    EXPECT(fp8_dequantize(A, 0, FP8_E4M3, 1.0f, NULL, FP8_BF16, C, NULL), FP8_OK);
    EXPECT(fp8_quantize_amax(X, 8, FP8_BF16, FP8_E4M3, NULL, A, F, NULL), BAD);
    EXPECT(fp8_quantize_amax(X, 8, FP8_BF16, FP8_E4M3, F, NULL, F, NULL), BAD);
    EXPECT(fp8_quantize_amax(X, 8, FP8_BF16, FP8_E4M3, F, A, NULL, NULL), BAD);
    EXPECT(fp8_quantize_sr(X, 8, FP8_BF16, 7, 1.0f, NULL, 1u, A, NULL), BAD);
    EXPECT(fp8_quantize_sr(X, 8, FP8_BF16, FP8_E4M3, 1.0f, Fodd, 1u, A, NULL), BAD);
    EXPECT(fp8_quantize_sr(X, 0, FP8_BF16, FP8_E4M3, 1.0f, NULL, 1u, A, NULL), FP8_OK);
    EXPECT(fp8_amax_rows(X, -1, 4, FP8_BF16, F, NULL), BAD);
    EXPECT(fp8_amax_rows(X, 4, 4, FP8_BF16, NULL, NULL), BAD);
    EXPECT(fp8_amax_rows(X, 0, 4, FP8_BF16, NULL, NULL), FP8_OK);
    EXPECT(fp8_quantize_rows(X, 4, -4, FP8_BF16, FP8_E4M3, F, A, NULL), BAD);
    EXPECT(fp8_quantize_rows(X, 4, 4, FP8_BF16, FP8_E4M3, NULL, A, NULL), BAD);
    EXPECT(fp8_quantize_rows(X, 4, 0, FP8_BF16, FP8_E4M3, NULL, NULL, NULL), FP8_OK);
    EXPECT(fp8_quantize_transpose(X, 4, 4, FP8_BF16, FP8_E4M3, F, A, NULL, NULL), BAD);
    EXPECT(fp8_quantize_transpose(X, 4, 4, 9, FP8_E4M3, F, A, B, NULL), BAD);
    EXPECT(fp8_quantize_transpose(X, 0, 4, FP8_BF16, FP8_E4M3, NULL, NULL, NULL, NULL), FP8_OK);

    /* GEMM entry points: rejected on the host */
    EXPECT(fp8_gemm(A, 2, 1.0f, B, FP8_E4M3, 1.0f, C, 16, 16, 16, FP8_F32, NULL), BAD);
    EXPECT(fp8_gemm(A, FP8_E4M3, 1.0f, B, FP8_E4M3, 1.0f, C, 16, -16, 16, FP8_F32, NULL), BAD);
    EXPECT(fp8_gemm(A, FP8_E4M3, 1.0f, B, FP8_E4M3, 1.0f, NULL, 16, 16, 16, FP8_F32, NULL), BAD);
    EXPECT(fp8_gemm(NULL, FP8_E4M3, 1.0f, B, FP8_E4M3, 1.0f, C, 16, 16, 16, FP8_F32, NULL), BAD);
    EXPECT(fp8_gemm(A, FP8_E4M3, 1.0f, B, FP8_E4M3, 1.0f, Xodd, 16, 16, 16, FP8_BF16, NULL), BAD);
    EXPECT(fp8_gemm(A, FP8_E4M3, 1.0f, B, FP8_E4M3, 1.0f, C, 16, 16, 16, 3, NULL), BAD);
    EXPECT(fp8_gemm(A, FP8_E4M3, 1.0f, B, FP8_E4M3, 1.0f, C, 0, 16, 16, FP8_F32, NULL), FP8_OK);      /* no output */
    EXPECT(fp8_gemm_mfma8(A, FP8_E4M3, 1.0f, B, 6, 1.0f, C, 16, 16, 16, FP8_F32, NULL), BAD);
    EXPECT(fp8_gemm_dscale(A, FP8_E4M3, NULL, B, FP8_E4M3, F, C, 16, 16, 16, FP8_F32, NULL), BAD);
    EXPECT(fp8_gemm_dscale(A, FP8_E4M3, Fodd, B, FP8_E4M3, F, C, 16, 16, 16, FP8_F32, NULL), BAD);
    EXPECT(fp8_gemm_mfma8_dscale(A, FP8_E4M3, F, B, FP8_E4M3, NULL, C, 16, 16, 16, FP8_F32, NULL), BAD);
    EXPECT(fp8_gemm_ex(A, FP8_E4M3, 2, B, FP8_E4M3, 0, C, 16, 16, 16, FP8_F32, 1.0f, 1.0f, NULL, NULL, 0, NULL), BAD);
    EXPECT(fp8_gemm_ex(A, FP8_E4M3, 0, B, FP8_E4M3, 0, C, 16, 16, 16, FP8_F32, 1.0f, 1.0f, NULL, NULL, 8, NULL), BAD);
    EXPECT(fp8_gemm_ex(A, FP8_E4M3, 0, B, FP8_E4M3, 0, C, 16, 0, 16, FP8_F32, 1.0f, 1.0f, NULL, NULL, 0, NULL), FP8_OK);
    EXPECT(fp8_gemm_fused(A, FP8_E4M3, 0, B, FP8_E4M3, 0, C, 7, 16, 16, 16, F, 1, F, 1, NULL, NULL, 0, NULL), BAD);
    EXPECT(fp8_gemm_fused(A, FP8_E4M3, 0, B, FP8_E4M3, 0, C, FP8_OUT_BF16, 16, 16, 16, F, 3, F, 1, NULL, NULL, 0, NULL), BAD);
    EXPECT(fp8_gemm_fused(A, FP8_E4M3, 0, B, FP8_E4M3, 0, C, FP8_OUT_BF16, 16, 16, 16, F, 16, F, 5, NULL, NULL, 0, NULL), BAD);
    EXPECT(fp8_gemm_fused(A, FP8_E4M3, 0, B, FP8_E4M3, 0, C, FP8_OUT_BF16, 16, 16, 16, NULL, 1, F, 1, NULL, NULL, 0, NULL), BAD);
    EXPECT(fp8_gemm_fused(A, FP8_E4M3, 0, B, FP8_E4M3, 0, C, FP8_OUT_BF16, 16, 16, 16, F, 1, F, 1, F, NULL, 0, NULL), BAD);
    EXPECT(fp8_gemm_splitk(A, FP8_E4M3, 0, B, FP8_E4M3, 0, C, 1024, 1024, 65536, FP8_F32, 1.0f, 1.0f, NULL, NULL, 0, 65, X, 1u << 30, NULL), BAD);
    EXPECT(fp8_gemm_splitk(A, FP8_E4M3, 0, B, FP8_E4M3, 0, C, 1024, 1024, 65536, FP8_F32, 1.0f, 1.0f, NULL, NULL, 0, 8, NULL, 0, NULL), BAD);
    EXPECT(fp8_gemm_splitk(A, FP8_E4M3, 0, B, FP8_E4M3, 0, C, 1024, 1024, 65536, FP8_F32, 1.0f, 1.0f, NULL, NULL, 0, 8, X, 1024, NULL), BAD);
    EXPECT(fp8_gemm_splitk(A, FP8_E4M3, 0, B, FP8_E4M3, 0, C, 1024, 1024, 65536, FP8_F32, 1.0f, 1.0f, NULL, NULL, 0, 8, Xodd, 1u << 30, NULL), BAD);
    EXPECT(fp8_gemm_splitk_static(A, FP8_E4M3, 0, B, FP8_E4M3, 0, C, 1024, 1024, 65536, FP8_F32, 1.0f, 1.0f, NULL, NULL, 0, -1, NULL), BAD);
    EXPECT(fp8_gemm_splitk_static(A, FP8_E4M3, 0, B, FP8_E4M3, 0, C, 4096, 4096, 65536, FP8_F32, 1.0f, 1.0f, NULL, NULL, 0, 8, NULL), FP8_ERR_UNSUPPORTED);

    /* plans and sizes: fixed cases, then a seeded sweep (every value must be one of the documented ones) */
    EXPECT(fp8_gemm_plan(A, 0, B, 0, C, 8192, 49152, 12288, NULL), FP8_PLAN_TILED_256x256);
    EXPECT(fp8_gemm_plan(A, 0, B, 0, C, 8192, 50257, 12288, NULL), FP8_PLAN_MFMA_ANY);
    EXPECT(fp8_gemm_plan(A, 0, B, 1, C, 8192, 50257, 12288, NULL), FP8_PLAN_TILED_256x256 | FP8_PLAN_ELEMENTWISE_STORES);
    EXPECT(fp8_gemm_plan(A + 1, 0, B, 0, C, 512, 512, 512, NULL), FP8_PLAN_MFMA_ANY);
    EXPECT(fp8_gemm_plan(A, 0, B, 0, C, 0, 512, 512, NULL), FP8_PLAN_NO_GEMM);
    EXPECT(fp8_gemm_plan(A, 0, B, 0, C, -1, 512, 512, NULL), -BAD);
    EXPECT(fp8_gemm_plan(A, 0, B, 3, C, 512, 512, 512, NULL), -BAD);
    EXPECT(fp8_gemm_plan(A, 0, B, 0, C, INT64_MAX / 2, 3, 5, NULL), FP8_PLAN_FMA_KERNEL);
    EXPECT(fp8_gemm_splitk_workspace_size(1024, 1024, 65536, 1, 0, 0), (size_t)16 * 1024 * 1024 * 4);
    EXPECT(fp8_gemm_splitk_workspace_size(1024, 1024, 65536, 1, 0, 70), 0);
    EXPECT(fp8_gemm_splitk_workspace_size(-5, 1024, 65536, 1, 0, 0), 0);
    {
        uint64_t s = 0x9E3779B97F4A7C15ull;
        for (int i = 0; i < 20000; ++i) {
            int64_t dim[3];
            for (int d = 0; d < 3; ++d) {
                s = s * 6364136223846793005ull + 1442695040888963407ull;
                const int shift = (int)((s >> 59) & 31);                     /* sizes from 1 to 2^36 */
                dim[d] = (int64_t)(((s >> 8) & 0xFFFFFFFFFull) >> shift) + 1;
            }
            s = s * 6364136223846793005ull + 1442695040888963407ull;
            const int ta = (int)(s >> 63), tb = (int)((s >> 62) & 1), off = (int)((s >> 40) & 15) * (int)((s >> 61) & 1);
            const int plan = fp8_gemm_plan(A + off, ta, B, tb, C, dim[0], dim[1], dim[2], (s >> 33) & 1 ? F : NULL);
            const int kernel = plan & 15;
            if (plan < 0 || kernel < FP8_PLAN_FMA_KERNEL || kernel > FP8_PLAN_TILED_MIXED ||
                (plan & ~(15 | FP8_PLAN_ELEMENTWISE_STORES | FP8_PLAN_PERSISTENT))) {
                printf("plan(%lld, %lld, %lld, %d, %d, +%d) = %d\n", (long long)dim[0], (long long)dim[1], (long long)dim[2], ta, tb, off, plan);
                ++failures;
            }
            const size_t ws = fp8_gemm_splitk_workspace_size(dim[0], dim[1], dim[2], ta, tb, (int)((s >> 20) % 65));
            if (ws % 4 || (ws && ws / 4 / (size_t)dim[0] / (size_t)dim[1] > 64)) {
                printf("workspace(%lld, %lld, %lld) = %zu\n", (long long)dim[0], (long long)dim[1], (long long)dim[2], ws);
                ++failures;
            }
        }
    }

    /* knobs */
    EXPECT(fp8_get_knob(FP8_KNOB_TILE_N), 0);
    EXPECT(fp8_set_knob(FP8_KNOB_TILE_N, 128), 0);
    EXPECT(fp8_get_knob(FP8_KNOB_TILE_N), 128);
    EXPECT(fp8_set_knob(FP8_KNOB_TILE_N, 0), 128);
    EXPECT(fp8_set_knob(FP8_KNOB_TILE_N, 100), -BAD);
    EXPECT(fp8_set_knob(-1, 0), -BAD);
    EXPECT(fp8_set_knob(FP8_KNOB_COUNT, 0), -BAD);
    EXPECT(fp8_get_knob(FP8_KNOB_COUNT), -BAD);
    EXPECT(fp8_set_knob(FP8_KNOB_PERSIST, 3), -BAD);
    EXPECT(fp8_set_knob(FP8_KNOB_MIXED, 2), 0);
    EXPECT(fp8_gemm_plan(A, 0, B, 0, C, 8192, 49152, 12288, NULL), FP8_PLAN_TILED_MIXED);
    EXPECT(fp8_set_knob(FP8_KNOB_MIXED, 0), 2);
    EXPECT(fp8_gemm_plan(A, 0, B, 0, C, 4096, 6144, 8192, NULL), FP8_PLAN_TILED_MIXED);

    if (failures) { printf("%d failure(s)\n", failures); return 1; }
    printf("ok\n");
    return 0;
}
