/*
 * fp8_oracle.c -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, obviously-correct CPU statement of the scaled-FP8 matrix
 * multiply path of "FP8 Formats for Deep Learning" (arXiv 2209.05433):
 * amax -> scale -> cast to E4M3/E5M2 -> FP8 x FP8 dot products -> unscale.
 * Only tests, the smoke check and the bench's cpu_baseline leg may call it.
 * The product (the HIP library) never links, includes or calls this file,
 * and this file includes nothing from the product.
 *
 * Every function states the passage of the paper it follows.  Where the
 * paper is silent the reading taken is written at the function.
 *
 * Conventions of this repository that the paper does not fix ("parity
 * unpinned", they occur in none of the benchmark workloads):
 *   - the scale returned for a zero / non-finite amax (also from a history of maxima),
 *   - the stochastic-rounding rule fp8o_encode_sr (Section 2 names the mode without defining
 *     it; the rule's properties and its generator's published vectors are pinned, the choice
 *     of the rule itself is this repository's).
 *
 * Build: gcc -O2 -fopenmp -shared -fPIC (no -ffast-math: IEEE semantics are
 * part of the definition).  OpenMP only spreads independent outer-loop
 * iterations over host cores; no arithmetic is reordered by it.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { FMT_E4M3 = 0, FMT_E5M2 = 1 };
enum { DT_F32 = 0, DT_BF16 = 1 };

/* Field widths and bias: Table 1, row "Exponent bias", and the S.E.M notation
 * of Section 3 (E4M3 = 1.4.3 bits, E5M2 = 1.5.2 bits). */
static int fmt_ebits(int fmt) { return fmt == FMT_E4M3 ? 4 : 5; }
static int fmt_mbits(int fmt) { return fmt == FMT_E4M3 ? 3 : 2; }
static int fmt_bias(int fmt)  { return fmt == FMT_E4M3 ? 7 : 15; }

/*
 * decode: the real value of one FP8 byte (Table 1; Section 3.1).
 *   E4M3: exponent field all ones AND mantissa all ones is NaN; there are no
 *         infinities; every other pattern with exponent 1111 is an ordinary
 *         normal number (256 ... 448).
 *   E5M2: IEEE-style: exponent 11111 with mantissa 00 is +-inf, otherwise NaN.
 *   exponent field 0: subnormal, (-1)^S * 2^(1-bias) * M / 2^mbits  (zero if M=0)
 *   otherwise       : normal,    (-1)^S * 2^(E-bias) * (1 + M / 2^mbits)
 */
double fp8o_decode(int fmt, uint8_t b)
{
    const int eb = fmt_ebits(fmt), mb = fmt_mbits(fmt), bias = fmt_bias(fmt);
    const int S = b >> 7;
    const int E = (b >> mb) & ((1 << eb) - 1);
    const int M = b & ((1 << mb) - 1);
    const int Eall = (1 << eb) - 1, Mall = (1 << mb) - 1;
    const double sgn = S ? -1.0 : 1.0;
    double mag;

    if (fmt == FMT_E4M3) {
        if (E == Eall && M == Mall) return S ? -NAN : NAN;
    } else {
        if (E == Eall) return M == 0 ? sgn * INFINITY : (S ? -NAN : NAN);
    }
    if (E == 0)
        mag = ldexp((double)M / (double)(1 << mb), 1 - bias);
    else
        mag = ldexp(1.0 + (double)M / (double)(1 << mb), E - bias);
    return sgn * mag;
}

/* Number of non-negative finite codes: 0x00..0x7E for E4M3 (the only
 * non-finite magnitude code is 0x7F), 0x00..0x7B for E5M2 (0x7C is inf,
 * 0x7D..0x7F are NaN).  Table 1 rows "Infinities", "NaN", "Max normal". */
static int fmt_nfinite(int fmt) { return fmt == FMT_E4M3 ? 127 : 124; }

/*
 * encode: nearest representable value of a single-precision number, round to
 * nearest with ties to the even code, written as a search over the list of
 * representable magnitudes that decode() defines.
 *
 *  - Specials (Section 2, type-conversion paragraph): NaN -> NaN; for E4M3
 *    +-inf -> NaN as well (it has no inf); for E5M2 +-inf -> +-inf.  This
 *    holds in saturating mode too: saturation (Section 2, scaling paragraph)
 *    is said of values that overflow, i.e. finite ones.
 *  - saturating != 0: a finite magnitude at or above the largest finite value
 *    becomes that value (448 / 57344).
 *  - saturating == 0 (the optional strict mode of Section 2): the magnitude is
 *    rounded against the next value the exponent/mantissa grid would hold
 *    (480 / 65536); if rounding lands there the result is NaN (E4M3) or inf
 *    (E5M2).
 *  - The sign bit of the input is kept, also when the magnitude rounds to
 *    zero (IEEE reading of the signed zeros of Section 3.1).
 *  - NaN payload for E5M2: mantissa 11 (Table 1 allows three; the code a widely used library cast
 *    emits, which a test compares with).
 *
 * All comparisons are exact: a float and every FP8 value are exact doubles,
 * and so are 2*m and lo+hi.
 */
uint8_t fp8o_encode(int fmt, float y, int saturating)
{
    const int nfin = fmt_nfinite(fmt);
    const uint8_t sign = signbit(y) ? 0x80 : 0x00;
    const uint8_t nan_code = 0x7F;
    const uint8_t inf_code = 0x7C;              /* E5M2 only */
    const uint8_t max_code = (uint8_t)(nfin - 1);
    double m, vmax;
    int lo, hi;

    if (isnan(y)) return sign | nan_code;
    if (isinf(y)) return sign | (fmt == FMT_E4M3 ? nan_code : inf_code);

    m = fabs((double)y);
    vmax = fp8o_decode(fmt, max_code);
    if (m >= vmax) {
        double next, mid;
        if (saturating || m == vmax) return sign | max_code;
        /* strict mode: the grid point one step above the maximum */
        next = vmax + (vmax - fp8o_decode(fmt, (uint8_t)(max_code - 1)));
        mid = 0.5 * (vmax + next);
        if (m < mid) return sign | max_code;
        if (m == mid && (max_code & 1) == 0) return sign | max_code;
        return sign | (fmt == FMT_E4M3 ? nan_code : inf_code);
    }
    /* bisection for adjacent codes lo, hi=lo+1 with decode(lo) <= m < decode(hi) */
    lo = 0;
    hi = max_code;
    while (hi - lo > 1) {
        int mid = (lo + hi) / 2;
        if (fp8o_decode(fmt, (uint8_t)mid) <= m) lo = mid; else hi = mid;
    }
    {
        const double vlo = fp8o_decode(fmt, (uint8_t)lo);
        const double vhi = fp8o_decode(fmt, (uint8_t)hi);
        const double twice = 2.0 * m, sum = vlo + vhi;
        int code;
        if (twice < sum) code = lo;
        else if (twice > sum) code = hi;
        else code = (lo & 1) ? hi : lo;          /* tie: the even code */
        return sign | (uint8_t)code;
    }
}

/*
 * Stochastic rounding (Section 2 lists it as a rounding mode an implementation may choose; the
 * paper gives no definition, this one is the reading of this repository).  A finite value of
 * magnitude m below the largest finite value lies between adjacent FP8 values lo <= m < hi.  With
 * t = (m - lo) / (hi - lo) and T = floor(t * 2^16), the result is hi if T + r >= 2^16 and lo
 * otherwise, where r is a 16-bit random integer: hi is taken with probability T / 2^16, values
 * on the grid never move.  Magnitudes at or above the largest finite value saturate; the sign
 * and the special values are handled as in fp8o_encode.
 */
uint8_t fp8o_encode_sr(int fmt, float y, uint32_t r16)
{
    const int nfin = fmt_nfinite(fmt);
    const uint8_t sign = signbit(y) ? 0x80 : 0x00;
    const uint8_t max_code = (uint8_t)(nfin - 1);
    double m, vlo, vhi, t;
    int lo, hi;

    if (isnan(y) || isinf(y)) return fp8o_encode(fmt, y, 1);
    m = fabs((double)y);
    if (m >= fp8o_decode(fmt, max_code)) return sign | max_code;
    lo = 0;
    hi = max_code;
    while (hi - lo > 1) {
        int mid = (lo + hi) / 2;
        if (fp8o_decode(fmt, (uint8_t)mid) <= m) lo = mid; else hi = mid;
    }
    vlo = fp8o_decode(fmt, (uint8_t)lo);
    vhi = fp8o_decode(fmt, (uint8_t)hi);
    t = (m - vlo) / (vhi - vlo);            /* exact: the spacing is a power of two */
    return sign | (uint8_t)((floor(t * 65536.0) + (double)(r16 & 0xFFFFu) >= 65536.0) ? hi : lo);
}

/*
 * Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3",
 * SC 2011): ten rounds of two 32x32 -> 64 bit multiplications whose halves are crossed over and
 * mixed with a key that is bumped by Weyl constants every round.
 */
void fp8o_philox4x32(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    int round;
    for (round = 0; round < 10; ++round) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n1 = (uint32_t)p1;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        const uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* The 16 random bits of element i for a 64-bit seed: block i / 8 of the generator keyed by the
 * seed, counter = (block, 0, 0) as a 128-bit number; 16-bit field i % 8 of its 128 output bits,
 * low half of word 0 first. */
uint32_t fp8o_sr_bits(uint64_t seed, uint64_t i)
{
    const uint64_t block = i / 8;
    const uint32_t ctr[4] = {(uint32_t)block, (uint32_t)(block >> 32), 0u, 0u};
    const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t w[4];
    const unsigned f = (unsigned)(i % 8);
    fp8o_philox4x32(ctr, key, w);
    return (w[f / 2] >> (16 * (f % 2))) & 0xFFFFu;
}

/* bfloat16 is the upper half of a single-precision number: widening is exact. */
static float bf16_to_f32(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

static float load_elem(const void *x, size_t i, int in_dtype)
{
    if (in_dtype == DT_BF16) return bf16_to_f32(((const uint16_t *)x)[i]);
    return ((const float *)x)[i];
}

/*
 * amax: the largest magnitude in the tensor (Section 2: the scale is chosen
 * from the largest magnitude the tensor holds; Section 4.3: one per tensor).
 * Reading where the paper is silent: any NaN element makes the result NaN;
 * infinities give +inf; the result is never negative zero; empty -> 0.
 */
float fp8o_amax(const void *x, size_t n, int in_dtype)
{
    float best = 0.0f;
    int saw_nan = 0;
    size_t i;
#pragma omp parallel
    {
        float loc = 0.0f;
        int loc_nan = 0;
#pragma omp for nowait
        for (i = 0; i < n; ++i) {
            float a = fabsf(load_elem(x, i, in_dtype));
            if (isnan(a)) loc_nan = 1;
            else if (a > loc) loc = a;
        }
#pragma omp critical
        {
            if (loc_nan) saw_nan = 1;
            if (loc > best) best = loc;
        }
    }
    return saw_nan ? NAN : best;
}

/*
 * scale: the factor that moves amax onto the largest finite value of the
 * format (Section 2; Table 1 "Max normal"), one IEEE single-precision
 * division.  Any real value is allowed (Section 3.2), so no rounding to a
 * power of two and no margin.  Repository convention where the paper is
 * silent: amax zero, NaN or inf, or a quotient that is not finite -> 1.
 */
float fp8o_scale_from_amax(float amax, int fmt)
{
    const float fmax = fmt == FMT_E4M3 ? 448.0f : 57344.0f;
    float s;
    if (!(amax > 0.0f) || isinf(amax)) return 1.0f;
    s = fmax / amax;
    if (!isfinite(s)) return 1.0f;
    return s;
}

/*
 * quantize: q[i] = encode(fl32(x[i] * scale))  (Section 2: values are
 * multiplied by the scaling factor before the cast, and overflow saturates).
 * Reading where the paper is silent: the product is rounded once to single
 * precision before the FP8 rounding.  A 24x24-bit product is exact in double,
 * so the conversion to float below is that single rounding.
 */
void fp8o_quantize(const void *x, size_t n, int in_dtype, int fmt, float scale,
                   int saturating, uint8_t *q)
{
    size_t i;
#pragma omp parallel for
    for (i = 0; i < n; ++i) {
        double p = (double)load_elem(x, i, in_dtype) * (double)scale;
        q[i] = fp8o_encode(fmt, (float)p, saturating);
    }
}

/* Inverse of the cast for one tensor: decode, then undo the scaling by the
 * reciprocal of the scale (Section 2, scaling paragraph). */
void fp8o_dequantize(const uint8_t *q, size_t n, int fmt, float scale, double *out)
{
    size_t i;
#pragma omp parallel for
    for (i = 0; i < n; ++i) out[i] = fp8o_decode(fmt, q[i]) / (double)scale;
}

/* Scaled cast with stochastic rounding: q[i] = encode_sr(fl32(x[i] * scale), bits(seed, i)). */
void fp8o_quantize_sr(const void *x, size_t n, int in_dtype, int fmt, float scale, uint64_t seed,
                      uint8_t *q)
{
    size_t i;
#pragma omp parallel for
    for (i = 0; i < n; ++i) {
        double p = (double)load_elem(x, i, in_dtype) * (double)scale;
        q[i] = fp8o_encode_sr(fmt, (float)p, fp8o_sr_bits(seed, (uint64_t)i));
    }
}

/*
 * GEMM reference (Section 2: FP8-input matrix multiplies produce
 * higher-precision outputs; Section 3: the formats of the operands).
 * For every requested output (i, j), in double precision:
 *     S = sum_k decode(A[i,k]) * decode(B[k,j])
 *     T = sum_k |decode(A[i,k]) * decode(B[k,j])|
 * A is M x K row-major, B is K x N row-major.  Each product of two FP8 values
 * is exact in double.  The unscale factor is applied by the caller.
 */
static void decode_table(int fmt, double lut[256])
{
    int b;
    for (b = 0; b < 256; ++b) lut[b] = fp8o_decode(fmt, (uint8_t)b);
}

/* Sampled outputs: npts pairs (pi[p], pj[p]). */
void fp8o_gemm_points(const uint8_t *A, int fmtA, const uint8_t *B, int fmtB,
                      int64_t M, int64_t N, int64_t K,
                      const int64_t *pi, const int64_t *pj, int64_t npts,
                      double *S, double *T)
{
    double va[256], vb[256];       /* decode() of every byte value */
    int64_t p;
    (void)M;
    decode_table(fmtA, va);
    decode_table(fmtB, vb);
#pragma omp parallel for schedule(dynamic, 16)
    for (p = 0; p < npts; ++p) {
        const uint8_t *arow = A + pi[p] * K;
        const uint8_t *bcol = B + pj[p];
        double s = 0.0, t = 0.0;
        int64_t k;
        for (k = 0; k < K; ++k) {
            double prod = va[arow[k]] * vb[bcol[k * N]];
            s += prod;
            t += fabs(prod);
        }
        S[p] = s;
        T[p] = t;
    }
}

/* Whole rows: rows[r] for r < nrows; S and T are nrows x N row-major.
 * Every output still adds its K products in ascending k. */
void fp8o_gemm_rows(const uint8_t *A, int fmtA, const uint8_t *B, int fmtB,
                    int64_t M, int64_t N, int64_t K,
                    const int64_t *rows, int64_t nrows, double *S, double *T)
{
    double va[256], vb[256];
    int64_t r;
    (void)M;
    decode_table(fmtA, va);
    decode_table(fmtB, vb);
#pragma omp parallel for schedule(dynamic, 1)
    for (r = 0; r < nrows; ++r) {
        const uint8_t *arow = A + rows[r] * K;
        double *s = S + r * N, *t = T + r * N;
        int64_t j, k;
        for (j = 0; j < N; ++j) { s[j] = 0.0; t[j] = 0.0; }
        for (k = 0; k < K; ++k) {
            const double a = va[arow[k]];
            const uint8_t *brow = B + k * N;
            for (j = 0; j < N; ++j) {
                double prod = a * vb[brow[j]];
                s[j] += prod;
                t[j] += fabs(prod);
            }
        }
    }
}

/* Signed block sums of the reference product, for the whole-matrix check of problems whose
 * every output the loops above cannot reach.  With r one multiplier (+-1) per column and block t =
 * columns [t * block, (t + 1) * block):
 *     SR[i][t] = sum_{j in block t} r[j] * S[i][j] = sum_k decode(A[i,k]) * BR[k][t],
 *     BR[k][t] = sum_{j in block t} r[j] * decode(B[k,j]),
 * and the same with magnitudes for TR (|r[j]| = 1 is assumed: TR[i][t] = sum_j T[i][j]).
 * Plain reassociation of the definition (every term is exact in double); SR, TR are M x nb. */
int fp8o_gemm_block_sums(const uint8_t *A, int fmtA, const uint8_t *B, int fmtB,
                         int64_t M, int64_t N, int64_t K, const double *r, int64_t block,
                         double *BR, double *BT, double *SR, double *TR)
{
    double va[256], vb[256];
    const int64_t nb = (N + block - 1) / block;
    int64_t k, i;
    int nonfinite = 0;             /* set if an operand byte decodes to inf or NaN: sums are then meaningless */
    decode_table(fmtA, va);
    decode_table(fmtB, vb);
#pragma omp parallel for schedule(static)
    for (k = 0; k < K; ++k) {
        const uint8_t *brow = B + k * N;
        int64_t j;
        for (j = 0; j < nb; ++j) { BR[k * nb + j] = 0.0; BT[k * nb + j] = 0.0; }
        for (j = 0; j < N; ++j) {
            const double b = vb[brow[j]];
            const int64_t t = j / block;
            BR[k * nb + t] += r[j] * b;
            BT[k * nb + t] += fabs(b);
        }
        for (j = 0; j < nb; ++j)
            if (!isfinite(BT[k * nb + j])) {
#pragma omp atomic write
                nonfinite = 1;
            }
    }
#pragma omp parallel for schedule(static)
    for (i = 0; i < M; ++i) {
        const uint8_t *arow = A + i * K;
        double *s = SR + i * nb, *t = TR + i * nb;
        int64_t kk, j;
        for (j = 0; j < nb; ++j) { s[j] = 0.0; t[j] = 0.0; }
        for (kk = 0; kk < K; ++kk) {
            const double a = va[arow[kk]], aa = fabs(a);
            const double *br = BR + kk * nb, *bt = BT + kk * nb;
            for (j = 0; j < nb; ++j) {
                s[j] += a * br[j];
                t[j] += aa * bt[j];
            }
        }
        for (j = 0; j < nb; ++j)
            if (!isfinite(t[j])) {
#pragma omp atomic write
                nonfinite = 1;
            }
    }
    return nonfinite;
}

int fp8o_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        n = omp_get_num_threads();
    }
#endif
    return n;
}
