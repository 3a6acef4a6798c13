/* Driver for the sanitizer build of the CPU oracle (test infrastructure): calls every exported
 * routine of oracle/fp8_oracle.c on small, ragged and empty inputs and prints one checksum per
 * routine, which the test compares with the checksums of the ordinary build.  Compiled together
 * with fp8_oracle.c under -fsanitize=address,undefined; any report fails the test. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

double fp8o_decode(int fmt, uint8_t b);
uint8_t fp8o_encode(int fmt, float y, int saturating);
uint8_t fp8o_encode_sr(int fmt, float y, uint32_t r16);
void fp8o_philox4x32(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);
uint32_t fp8o_sr_bits(uint64_t seed, uint64_t i);
float fp8o_amax(const void *x, size_t n, int in_dtype);
float fp8o_scale_from_amax(float amax, int fmt);
void fp8o_quantize(const void *x, size_t n, int in_dtype, int fmt, float scale, int saturating, uint8_t *q);
void fp8o_dequantize(const uint8_t *q, size_t n, int fmt, float scale, double *out);
void fp8o_quantize_sr(const void *x, size_t n, int in_dtype, int fmt, float scale, uint64_t seed, uint8_t *q);
void fp8o_gemm_points(const uint8_t *A, int fmtA, const uint8_t *B, int fmtB, int64_t M, int64_t N, int64_t K,
                      const int64_t *pi, const int64_t *pj, int64_t npts, double *S, double *T);
void fp8o_gemm_rows(const uint8_t *A, int fmtA, const uint8_t *B, int fmtB, int64_t M, int64_t N, int64_t K,
                    const int64_t *rows, int64_t nrows, double *S, double *T);
int fp8o_gemm_block_sums(const uint8_t *A, int fmtA, const uint8_t *B, int fmtB, int64_t M, int64_t N, int64_t K,
                         const double *r, int64_t block, double *BR, double *BT, double *SR, double *TR);

static uint64_t lcg = 88172645463325252ull;
static uint32_t rnd(void) { lcg ^= lcg << 13; lcg ^= lcg >> 7; lcg ^= lcg << 17; return (uint32_t)(lcg >> 16); }

static uint64_t fnv(uint64_t h, const void *p, size_t n)
{
    const unsigned char *c = (const unsigned char *)p;
    size_t i;
    for (i = 0; i < n; ++i) { h ^= c[i]; h *= 1099511628211ull; }
    return h;
}

int main(void)
{
    const uint64_t H0 = 1469598103934665603ull;
    int fmt, sat, dt;
    uint64_t h;

    /* decode: all 256 patterns of both formats */
    h = H0;
    for (fmt = 0; fmt < 2; ++fmt) {
        int b;
        for (b = 0; b < 256; ++b) { double v = fp8o_decode(fmt, (uint8_t)b); if (v != v) v = -12345.0; h = fnv(h, &v, sizeof v); }
    }
    printf("decode %016llx\n", (unsigned long long)h);

    /* encode: random bit patterns (specials and subnormals included), both modes */
    h = H0;
    for (fmt = 0; fmt < 2; ++fmt)
        for (sat = 0; sat < 2; ++sat) {
            int i;
            for (i = 0; i < 200000; ++i) {
                uint32_t u = rnd() ^ (rnd() << 16);
                float y; uint8_t q;
                memcpy(&y, &u, 4);
                q = fp8o_encode(fmt, y, sat);
                h = fnv(h, &q, 1);
            }
        }
    printf("encode %016llx\n", (unsigned long long)h);

    /* amax, scale, quantize, dequantize, stochastic cast over sizes 0, 1, ragged */
    h = H0;
    {
        static const size_t sizes[] = {0, 1, 7, 64, 1001, 4099};
        size_t si;
        for (si = 0; si < sizeof sizes / sizeof sizes[0]; ++si) {
            const size_t n = sizes[si];
            float *xf = (float *)malloc(n * sizeof(float) + 1);
            uint16_t *xb = (uint16_t *)malloc(n * sizeof(uint16_t) + 1);
            uint8_t *q = (uint8_t *)malloc(n + 1);
            double *d = (double *)malloc(n * sizeof(double) + 1);
            size_t i;
            for (i = 0; i < n; ++i) {
                uint32_t u = rnd() ^ (rnd() << 16);
                if ((u & 0x7f800000u) == 0x7f800000u && (i % 50)) u &= 0x3fffffffu;   /* a few specials stay */
                memcpy(&xf[i], &u, 4);
                xb[i] = (uint16_t)(u >> 16);
            }
            for (dt = 0; dt < 2; ++dt) {
                const void *x = dt == 0 ? (const void *)xf : (const void *)xb;
                float a = fp8o_amax(x, n, dt);
                if (a != a) a = -1.0f;
                h = fnv(h, &a, 4);
                for (fmt = 0; fmt < 2; ++fmt) {
                    float s = fp8o_scale_from_amax(a, fmt);
                    h = fnv(h, &s, 4);
                    for (sat = 0; sat < 2; ++sat) { fp8o_quantize(x, n, dt, fmt, s, sat, q); h = fnv(h, q, n); }
                    fp8o_quantize(x, n, dt, fmt, 0.37f, 1, q);
                    h = fnv(h, q, n);
                    fp8o_dequantize(q, n, fmt, 0.37f, d);
                    for (i = 0; i < n; ++i) if (d[i] != d[i]) d[i] = -7.0;
                    h = fnv(h, d, n * sizeof(double));
                    fp8o_quantize_sr(x, n, dt, fmt, 0.37f, 0x123456789abcdefull + n, q);
                    h = fnv(h, q, n);
                }
            }
            free(xf); free(xb); free(q); free(d);
        }
    }
    printf("cast %016llx\n", (unsigned long long)h);

    /* generator */
    h = H0;
    {
        uint32_t ctr[4] = {1, 2, 3, 4}, key[2] = {5, 6}, out[4];
        int i;
        for (i = 0; i < 1000; ++i) { ctr[0] = (uint32_t)i; fp8o_philox4x32(ctr, key, out); h = fnv(h, out, sizeof out); }
        for (i = 0; i < 1000; ++i) { uint32_t b = fp8o_sr_bits(77, (uint64_t)i * 3); h = fnv(h, &b, 4); }
        for (i = 0; i < 20000; ++i) {
            uint32_t u = rnd() ^ (rnd() << 16); float y; uint8_t q;
            memcpy(&y, &u, 4);
            q = fp8o_encode_sr(i & 1, y, rnd() & 0xffff);
            h = fnv(h, &q, 1);
        }
    }
    printf("sr %016llx\n", (unsigned long long)h);

    /* GEMM reference: rows, points, block sums on ragged shapes, all format mixes */
    h = H0;
    {
        static const int64_t shapes[][3] = {{1, 1, 1}, {3, 5, 2}, {17, 9, 33}, {8, 40, 64}};
        size_t s;
        for (s = 0; s < sizeof shapes / sizeof shapes[0]; ++s) {
            const int64_t M = shapes[s][0], N = shapes[s][1], K = shapes[s][2];
            uint8_t *A = (uint8_t *)malloc((size_t)(M * K)), *B = (uint8_t *)malloc((size_t)(K * N));
            double *S = (double *)malloc((size_t)(M * N) * sizeof(double)), *T = (double *)malloc((size_t)(M * N) * sizeof(double));
            int64_t *rows = (int64_t *)malloc((size_t)M * sizeof(int64_t));
            int64_t pi[4], pj[4], i;
            double Sp[4], Tp[4];
            for (i = 0; i < M * K; ++i) A[i] = (uint8_t)((rnd() % 0x60) | ((rnd() & 1) << 7));
            for (i = 0; i < K * N; ++i) B[i] = (uint8_t)((rnd() % 0x60) | ((rnd() & 1) << 7));
            for (i = 0; i < M; ++i) rows[i] = M - 1 - i;
            for (i = 0; i < 4; ++i) { pi[i] = (int64_t)(rnd() % (uint32_t)M); pj[i] = (int64_t)(rnd() % (uint32_t)N); }
            for (fmt = 0; fmt < 4; ++fmt) {
                const int64_t block = 4, nb = (N + block - 1) / block;
                double *r = (double *)malloc((size_t)N * sizeof(double));
                double *BR = (double *)malloc((size_t)(K * nb) * sizeof(double)), *BT = (double *)malloc((size_t)(K * nb) * sizeof(double));
                double *SR = (double *)malloc((size_t)(M * nb) * sizeof(double)), *TR = (double *)malloc((size_t)(M * nb) * sizeof(double));
                fp8o_gemm_rows(A, fmt & 1, B, fmt >> 1, M, N, K, rows, M, S, T);
                h = fnv(h, S, (size_t)(M * N) * sizeof(double));
                h = fnv(h, T, (size_t)(M * N) * sizeof(double));
                fp8o_gemm_points(A, fmt & 1, B, fmt >> 1, M, N, K, pi, pj, 4, Sp, Tp);
                h = fnv(h, Sp, sizeof Sp);
                h = fnv(h, Tp, sizeof Tp);
                for (i = 0; i < N; ++i) r[i] = (rnd() & 1) ? 1.0 : -1.0;
                if (fp8o_gemm_block_sums(A, fmt & 1, B, fmt >> 1, M, N, K, r, block, BR, BT, SR, TR)) return 3;
                h = fnv(h, SR, (size_t)(M * nb) * sizeof(double));
                h = fnv(h, TR, (size_t)(M * nb) * sizeof(double));
                free(r); free(BR); free(BT); free(SR); free(TR);
            }
            free(A); free(B); free(S); free(T); free(rows);
        }
    }
    printf("gemm %016llx\n", (unsigned long long)h);
    return 0;
}
