// Variants of the amax / cast kernels for gfx950 (MI355X) that scaling recipes beyond the plain
// two-pass per-tensor one build on (arXiv 2209.05433: Section 2 leaves the choice of the scaling
// factor to software; Section 4.2 uses per-channel factors for weights; Section 4.1: activations,
// weights and activation gradients are all GEMM inputs, so a tensor is consumed in both storage
// orders during training):
//   - cast + amax in one pass, for a factor chosen beforehand from past maxima (3 bytes per bf16
//     element instead of 5);
//   - the factor from a history of maxima;
//   - per-row amax, per-row factors, per-row cast;
//   - cast that also writes the transposed bytes;
//   - cast with stochastic rounding (Section 2 names it as a rounding mode left to the
//     implementation), random bits from a counter-based generator so that results depend on
//     (seed, element index) alone.
// Except for the stochastic mode the rounding itself is the routine of the plain cast
// (fp8_encode.hpp).
#include "cast_common.hpp"

namespace fp8mm {
namespace {

// Packed running maximum (see vec_mag_max) -> sign-stripped fp32 bits.
template <int DT>
__device__ __forceinline__ unsigned run_to_bits(unsigned run)
{
    if (DT == FP8_F32) return run;
    const u16x2 p = __builtin_bit_cast(u16x2, run);
    return (unsigned)(p.x > p.y ? p.x : p.y) << 16;
}

// Raises *cell to at least `bits`.  Most workgroups find the cell already large enough and skip
// the atomic, so thousands of workgroups do not queue on one address.
__device__ __forceinline__ void raise_cell(unsigned* cell, unsigned bits)
{
    if (bits > __hip_atomic_load(cell, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(cell, bits);
}

// ------------------------------------------------------------------------------------------
// cast + amax in one pass
// ------------------------------------------------------------------------------------------
template <int DT, int FMT, bool NTS>
__global__ __launch_bounds__(kThreads) void quantize_amax_kernel(const void* __restrict__ x, size_t n,
                                                                const float* __restrict__ scale_dev,
                                                                uint8_t* __restrict__ q,
                                                                unsigned* __restrict__ amax_bits, bool vec)
{
    constexpr int VPI = DT == FP8_BF16 ? 2 : 4;     // 16-byte vectors per 16 elements
    const float s = *scale_dev;
    unsigned run = 0;
    size_t done = 0;
    if (vec) {
        const size_t nitem = n / 16;
        const size_t per = (nitem + gridDim.x - 1) / gridDim.x;
        const size_t lo = (size_t)blockIdx.x * per;
        const size_t hi = lo + per < nitem ? lo + per : nitem;
        if (lo < hi)
            cast_run<DT, FMT, kCastCvt, NTS, true>((const u32x4*)x, (typename Piece<DT>::type*)q, VPI * lo, VPI * hi, s, run);
        done = nitem * 16;
    }
    unsigned r = run_to_bits<DT>(run);
    const size_t stride = (size_t)gridDim.x * kThreads;
    for (size_t t = done + (size_t)blockIdx.x * kThreads + threadIdx.x; t < n; t += stride) {
        const unsigned m = scalar_mag<DT>(x, t);
        r = r > m ? r : m;
        q[t] = (uint8_t)encode_bits<FMT>(load_scalar<DT>(x, t) * s);
    }
    r = block_max_u32(r);
    if (threadIdx.x == 0) raise_cell(amax_bits, r);
}

// ------------------------------------------------------------------------------------------
// factors from maxima
// ------------------------------------------------------------------------------------------
// One factor from the largest entry of a history of maxima (NaN entries propagate, and a NaN
// maximum gives the factor 1 like every degenerate maximum).
__global__ __launch_bounds__(kThreads) void scale_from_history_kernel(const float* __restrict__ hist, size_t len, int fmt,
                                                                     float* __restrict__ out)
{
    unsigned r = 0;
    for (size_t i = threadIdx.x; i < len; i += kThreads) {
        const unsigned m = as_u32(hist[i]) & 0x7fffffffu;
        r = r > m ? r : m;
    }
    r = block_max_u32(r);
    if (threadIdx.x == 0) *out = scale_rule(as_f32(r), fmt);
}

__global__ __launch_bounds__(kThreads) void scale_n_kernel(const float* __restrict__ amax, size_t n, int fmt,
                                                          float* __restrict__ out)
{
    const size_t stride = (size_t)gridDim.x * kThreads;
    for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride) out[i] = scale_rule(amax[i], fmt);
}

// ------------------------------------------------------------------------------------------
// per-row amax and cast: one workgroup per row at a time
// ------------------------------------------------------------------------------------------
template <int DT>
__global__ __launch_bounds__(kThreads) void amax_rows_kernel(const void* __restrict__ x, int64_t rows, int64_t cols,
                                                            float* __restrict__ amax_out, bool vec)
{
    constexpr int PV = Elem<DT>::per_vec;
    for (int64_t row = blockIdx.x; row < rows; row += gridDim.x) {
        const char* xr = (const char*)x + (size_t)row * (size_t)cols * Elem<DT>::size;
        unsigned run = 0;
        int64_t done = 0;
        if (vec) {
            const u32x4* xv = (const u32x4*)xr;
            const int64_t nvec = cols / PV;
            for (int64_t i = threadIdx.x; i < nvec; i += kThreads) run = vec_mag_max<DT>(__builtin_nontemporal_load(&xv[i]), run);
            done = nvec * PV;
        }
        unsigned r = run_to_bits<DT>(run);
        for (int64_t t = done + threadIdx.x; t < cols; t += kThreads) {
            const unsigned m = scalar_mag<DT>(xr, (size_t)t);
            r = r > m ? r : m;
        }
        r = block_max_u32(r);
        if (threadIdx.x == 0) amax_out[row] = as_f32(r);
        __syncthreads();                    // the reduction's staging cells are reused by the next row
    }
}

template <int DT, int FMT>
__global__ __launch_bounds__(kThreads) void quantize_rows_kernel(const void* __restrict__ x, int64_t rows, int64_t cols,
                                                                const float* __restrict__ scale_dev,
                                                                uint8_t* __restrict__ q, bool vec)
{
    constexpr int VPI = DT == FP8_BF16 ? 2 : 4;
    for (int64_t row = blockIdx.x; row < rows; row += gridDim.x) {
        const char* xr = (const char*)x + (size_t)row * (size_t)cols * Elem<DT>::size;
        uint8_t* qr = q + (size_t)row * (size_t)cols;
        const float s = scale_dev[row];
        int64_t done = 0;
        if (vec) {                              // cols is a multiple of 16: whole groups of vectors
            const int64_t nitem = cols / 16;
            unsigned unused = 0;
            cast_run<DT, FMT, kCastCvt, false, false>((const u32x4*)xr, (typename Piece<DT>::type*)qr, 0, (size_t)(VPI * nitem), s, unused);
            done = nitem * 16;
        }
        for (int64_t t = done + threadIdx.x; t < cols; t += kThreads)
            qr[t] = (uint8_t)encode_bits<FMT>(load_scalar<DT>(xr, (size_t)t) * s);
    }
}

// ------------------------------------------------------------------------------------------
// cast + transpose.  One workgroup per tile of 128 rows x 512 bytes of x (256 bf16 or 128 fp32
// columns).  A lane converts 8 (bf16) or 4 (fp32) consecutive elements of a row; the bytes go out to q
// straight from the registers (the lanes of a tile row cover its 256 or 128 bytes) and into an LDS
// copy of the tile.  The transposed tile comes out of that copy through the transposing LDS read of
// gfx950 (ds_read_b64_tr_b8: 16 lanes read an 8 x 16 byte block and each receives one column of it),
// two per lane = 16 consecutive bytes of a row of q^T; the pieces are put back into the buffer as the
// tile of q^T and stored 16 bytes per lane, 8 lanes per row: whole 128-byte lines (written as they
// come out of the transposing reads, every store instruction would touch 16 lines for a half each:
// 3-14 % slower, measured).  Non-temporal stores change nothing here (measured on four shapes).
//
// Tile order.  A tile's 128-byte pieces of q^T lie `rows` bytes apart.  Where that distance is a
// power of two (4 KB and up) they all fall on the same few memory channels, and so do those of every
// tile of the same tile row: walking the tiles along the rows of x then loses 15-20 % of the rate
// (measured on 16384 x 16384 against 16640 x 16640).  There the tiles are walked diagonally instead
// (tile row and tile column both change from one workgroup to the next); elsewhere along the rows of
// x, which keeps the pieces of neighbouring tiles together in time and is 3-12 % faster than the
// diagonal walk on such shapes (3 x 2^k rows included: 49152 x 12288 5.1 against 4.8 TB/s).
// Measured, bf16 -> E4M3 with both outputs, bytes moved / time: 16384 x 16384 4.2 -> 5.2 TB/s with
// the diagonal walk and the 256-column tile, 18432 x 16384 5.1 -> 5.4, 12288 x 49152 4.8 -> 5.0;
// with q^T written to the places of q (no scatter) the same
// kernel reaches 5.4, the plain cast 5.9 (cold).
// ------------------------------------------------------------------------------------------
constexpr int TT = 128;                       // tile rows; also the tile columns of the fp32 form
constexpr int QT_PITCH = TT + 16;             // LDS row pitch of the q^T tile (16-byte pad spreads the rows over the banks)

typedef int v2i __attribute__((ext_vector_type(2)));
#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))

template <int DT> struct TransposeTile { static constexpr int cols = DT == FP8_BF16 ? 256 : 128; };

template <int DT, int FMT>
__global__ __launch_bounds__(kThreads) void quantize_transpose_kernel(const void* __restrict__ x, int64_t rows, int64_t cols,
                                                                     const float* __restrict__ scale_dev,
                                                                     uint8_t* __restrict__ q, uint8_t* __restrict__ qt,
                                                                     int tiles_r, int tiles_c, bool diagonal)
{
    constexpr int TC = TransposeTile<DT>::cols;          // tile columns
    constexpr int PITCH = TC + 16;                       // LDS row pitch of the tile of q
    constexpr int EPL = DT == FP8_BF16 ? 8 : 4;          // elements per lane per load (16 bytes)
    constexpr int LPR = TC / EPL;                        // lanes per tile row
    constexpr int RPP = kThreads / LPR;                  // tile rows per pass of the workgroup
    constexpr int PASSES = TT / RPP;
    constexpr int LDS_BYTES = TT * PITCH > TC * QT_PITCH ? TT * PITCH : TC * QT_PITCH;
    __shared__ __attribute__((aligned(16))) uint8_t tile[LDS_BYTES];
    const float s = *scale_dev;
    const int b = blockIdx.x;
    int ti, tj;
    if (diagonal) { ti = b % tiles_r; tj = (b / tiles_r + ti) % tiles_c; }
    else { ti = b / tiles_c; tj = b % tiles_c; }
    const int64_t r0 = (int64_t)ti * TT, c0 = (int64_t)tj * TC;
    const int tid = threadIdx.x;
    const int lr = tid / LPR, lc = (tid % LPR) * EPL;    // lane's row within a pass, first column

    // load everything first (PASSES 16-byte loads in flight per lane), then convert
    u32x4 v[PASSES];
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
        const int64_t r = r0 + p * RPP + lr, c = c0 + lc;
        v[p] = (u32x4){0u, 0u, 0u, 0u};
        if (r < rows && c < cols)
            v[p] = __builtin_nontemporal_load((const u32x4*)((const char*)x + ((size_t)r * (size_t)cols + (size_t)c) * Elem<DT>::size));
    }
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
        const int tr = p * RPP + lr;
        unsigned b0, b1 = 0;
        if (DT == FP8_BF16) {
            b0 = encode4<FMT>(as_f32(v[p].x << 16) * s, as_f32(v[p].x & 0xffff0000u) * s,
                              as_f32(v[p].y << 16) * s, as_f32(v[p].y & 0xffff0000u) * s);
            b1 = encode4<FMT>(as_f32(v[p].z << 16) * s, as_f32(v[p].z & 0xffff0000u) * s,
                              as_f32(v[p].w << 16) * s, as_f32(v[p].w & 0xffff0000u) * s);
            *LDS_PTR(v2i, tile + tr * PITCH + lc) = (v2i){(int)b0, (int)b1};
        } else {
            b0 = encode4<FMT>(as_f32(v[p].x) * s, as_f32(v[p].y) * s, as_f32(v[p].z) * s, as_f32(v[p].w) * s);
            *LDS_PTR(unsigned, tile + tr * PITCH + lc) = b0;
        }
        // q straight from the registers: the lanes of one tile row cover its bytes
        const int64_t r = r0 + tr, c = c0 + lc;
        if (q && r < rows && c < cols) {
            uint8_t* dst = q + (size_t)r * (size_t)cols + (size_t)c;
            if (DT == FP8_BF16) *(u32x2*)dst = (u32x2){b0, b1}; else *(unsigned*)dst = b0;
        }
    }
    __syncthreads();
    // q^T: the transposing reads hand a lane 16 consecutive tile rows of one tile column = 16 bytes of
    // a row of q^T; a wave instruction covers 16 columns x 64 rows, wave w owns the columns
    // (TC / 4) w .. (TC / 4) (w + 1) - 1.  Stored like that a wave instruction would write 64-byte
    // halves of 16 different lines; instead the pieces go back into the (by then idle) buffer as the
    // tile of q^T and leave 16 bytes per lane, 8 lanes per 128-byte row.
    const int w = tid >> 6, l = tid & 63;
    const int g = l >> 4, t16 = l & 15;
    constexpr int CBW = TC / 64;                                  // blocks of 16 columns per wave
    u32x4 piece[CBW][2];
#pragma unroll
    for (int cb = 0; cb < CBW; ++cb)
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int tc0 = w * (TC / 4) + cb * 16;           // first tile column of the 16-lane group's block
            const int tr0 = half * 64 + g * 16;               // first tile row of the lane's 16 bytes
            // lanes 2 k and 2 k + 1 of a group address the two 8-byte halves of tile row tr0 + k (+ 8)
            const uint8_t* src = tile + (tr0 + (t16 >> 1)) * PITCH + tc0 + (t16 & 1) * 8;
            const v2i lo = __builtin_amdgcn_ds_read_tr8_b64_v2i32(LDS_PTR(v2i, src));
            const v2i hi = __builtin_amdgcn_ds_read_tr8_b64_v2i32(LDS_PTR(v2i, src + 8 * PITCH));
            piece[cb][half] = (u32x4){(unsigned)lo.x, (unsigned)lo.y, (unsigned)hi.x, (unsigned)hi.y};
        }
    __syncthreads();                                          // every wave has read what it needs of the tile
#pragma unroll
    for (int cb = 0; cb < CBW; ++cb)
#pragma unroll
        for (int half = 0; half < 2; ++half)
            *LDS_PTR(u32x4, tile + (w * (TC / 4) + cb * 16 + t16) * QT_PITCH + half * 64 + g * 16) = piece[cb][half];
    __syncthreads();
#pragma unroll
    for (int p = 0; p < TC / 32; ++p) {
        const int tc = p * 32 + (tid >> 3), trc = (tid & 7) * 16;         // row of the q^T tile, first byte in it
        const int64_t orow = c0 + tc, ocol = r0 + trc;                    // position in q^T (cols x rows)
        if (orow < cols && ocol < rows)
            *(u32x4*)(qt + (size_t)orow * (size_t)rows + (size_t)ocol) = *LDS_PTR(u32x4, tile + tc * QT_PITCH + trc);
    }
}

// Any shape and alignment: one element per lane, both outputs written directly.
template <int DT, int FMT>
__global__ __launch_bounds__(kThreads) void quantize_transpose_scalar_kernel(const void* __restrict__ x, int64_t rows, int64_t cols,
                                                                            const float* __restrict__ scale_dev,
                                                                            uint8_t* __restrict__ q, uint8_t* __restrict__ qt)
{
    const float s = *scale_dev;
    const size_t n = (size_t)rows * (size_t)cols, stride = (size_t)gridDim.x * kThreads;
    for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride) {
        const uint8_t b = (uint8_t)encode_bits<FMT>(load_scalar<DT>(x, i) * s);
        if (q) q[i] = b;
        qt[(i % (size_t)cols) * (size_t)rows + i / (size_t)cols] = b;
    }
}

// ------------------------------------------------------------------------------------------
// cast with stochastic rounding.  For lo <= |y| < hi adjacent FP8 values, t = (|y| - lo)/(hi - lo),
// T = floor(t * 2^16): the result is hi iff T + r >= 2^16, r = 16 random bits of the element.
// In the bits of y: for results in the normal range T is the 16 bits below the kept mantissa and
// the carry of T + r is added to the truncated code (a mantissa carry bumps the exponent as it
// should); below the smallest normal value the grid is uniform, |y| / step is taken as a fixed-point
// number with 16 fraction bits and r is added to it.
// ------------------------------------------------------------------------------------------
template <int FMT>
__device__ __forceinline__ unsigned encode_sr_bits(float y, unsigned r16)
{
    constexpr int MB = FMT == FP8_E4M3 ? 3 : 2;
    constexpr int BIAS = FMT == FP8_E4M3 ? 7 : 15;
    constexpr unsigned DROP = 23 - MB;
    constexpr unsigned REBIAS = (unsigned)(127 - BIAS) << 23;
    constexpr unsigned MIN_NORMAL = (unsigned)(127 + 1 - BIAS) << 23;
    constexpr unsigned TO_FIXED = (unsigned)(127 + 16 - (1 - BIAS - MB)) << 23;     // 2^16 / step
    constexpr unsigned MAX_BITS = FMT == FP8_E4M3 ? 0x43E00000u : 0x47600000u;
    constexpr unsigned MAX_CODE = FMT == FP8_E4M3 ? 0x7Eu : 0x7Bu;
    constexpr unsigned INF_CODE = FMT == FP8_E4M3 ? 0x7Fu : 0x7Cu;
    const unsigned u = as_u32(y);
    const unsigned a = u & 0x7fffffffu;
    const unsigned sign = (u >> 24) & 0x80u;
    const unsigned T = (a >> (DROP - 16)) & 0xffffu;
    const unsigned normal = ((a - REBIAS) >> DROP) + ((T + r16) >> 16);
    const unsigned fixed = (unsigned)(as_f32(a < MIN_NORMAL ? a : 0u) * as_f32(TO_FIXED));   // truncates
    const unsigned sub = (fixed + r16) >> 16;
    unsigned code = a < MIN_NORMAL ? sub : normal;
    code = a >= MAX_BITS ? MAX_CODE : code;
    code = a >= 0x7f800000u ? INF_CODE : code;
    code = a > 0x7f800000u ? 0x7Fu : code;
    return sign | code;
}

// The same rule through the converter instructions of gfx950 (v_cvt_sr_fp8_f32 / v_cvt_sr_bf8_f32:
// the random operand's upper bits are added below the kept mantissa; with the 16 random bits in
// its upper half and zeros below, the carry is exactly that of T + r; subnormal results included.
// Checked against the integer form on the GPU test inputs and on constructed carry boundaries).
// The instructions do not saturate (a magnitude beyond the largest value comes out as NaN / inf), so
// the value is clamped first; NaN and infinities take the integer form.
// Four scaled values and their four 16-bit fields (r01 = fields 0, 1; r23 = fields 2, 3) -> 4 bytes.
template <int FMT>
__device__ __forceinline__ unsigned encode_sr4(float y0, float y1, float y2, float y3, unsigned r01, unsigned r23)
{
    if (is_special(y0) | is_special(y1) | is_special(y2) | is_special(y3))
        return encode_sr_bits<FMT>(y0, r01 & 0xffffu) | (encode_sr_bits<FMT>(y1, r01 >> 16) << 8) |
               (encode_sr_bits<FMT>(y2, r23 & 0xffffu) << 16) | (encode_sr_bits<FMT>(y3, r23 >> 16) << 24);
    constexpr float FMAX = FMT == FP8_E4M3 ? 448.0f : 57344.0f;
    y0 = __builtin_amdgcn_fmed3f(y0, FMAX, -FMAX); y1 = __builtin_amdgcn_fmed3f(y1, FMAX, -FMAX);
    y2 = __builtin_amdgcn_fmed3f(y2, FMAX, -FMAX); y3 = __builtin_amdgcn_fmed3f(y3, FMAX, -FMAX);
    int w = 0;
    if (FMT == FP8_E4M3) {
        w = __builtin_amdgcn_cvt_sr_fp8_f32(y0, r01 << 16, w, 0);
        w = __builtin_amdgcn_cvt_sr_fp8_f32(y1, r01 & 0xffff0000u, w, 1);
        w = __builtin_amdgcn_cvt_sr_fp8_f32(y2, r23 << 16, w, 2);
        w = __builtin_amdgcn_cvt_sr_fp8_f32(y3, r23 & 0xffff0000u, w, 3);
    } else {
        w = __builtin_amdgcn_cvt_sr_bf8_f32(y0, r01 << 16, w, 0);
        w = __builtin_amdgcn_cvt_sr_bf8_f32(y1, r01 & 0xffff0000u, w, 1);
        w = __builtin_amdgcn_cvt_sr_bf8_f32(y2, r23 << 16, w, 2);
        w = __builtin_amdgcn_cvt_sr_bf8_f32(y3, r23 & 0xffff0000u, w, 3);
    }
    return (unsigned)w;
}

// Philox4x32-10 (Salmon et al., SC 2011): counter (c0, c1, 0, 0), key (k0, k1).
__device__ __forceinline__ void philox4x32_10(unsigned c0, unsigned c1, unsigned k0, unsigned k1, unsigned (&out)[4])
{
    unsigned c2 = 0u, c3 = 0u;
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const unsigned hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        const unsigned hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        c0 = hi1 ^ c1 ^ k0;
        c1 = lo1;
        c2 = hi0 ^ c3 ^ k1;
        c3 = lo0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// Element e uses the 16-bit field e % 8 (low half of word 0 first) of generator block e / 8.
// The unit of work is one generator block = 8 elements: one 16-byte vector of bf16 input (a wave's
// load instruction reads 1 KB of consecutive bytes) or two adjacent ones of fp32, 8 bytes of output.
// Workgroups own contiguous runs of blocks; a lane takes blocks kThreads apart, four in flight.
template <int DT, int FMT>
__global__ __launch_bounds__(kThreads) void quantize_sr_kernel(const void* __restrict__ x, size_t n, float scale,
                                                              const float* __restrict__ scale_dev,
                                                              unsigned seed_lo, unsigned seed_hi,
                                                              uint8_t* __restrict__ q, bool vec)
{
    constexpr int V = DT == FP8_BF16 ? 1 : 2;       // 16-byte vectors per block
    constexpr int U = 4;
    const float s = scale_dev ? *scale_dev : scale;
    size_t done = 0;
    if (vec) {
        const u32x4* xv = (const u32x4*)x;
        u32x2* qp = (u32x2*)q;
        const size_t nblock = n / 8;
        const size_t per = (nblock + gridDim.x - 1) / gridDim.x;
        const size_t lo = (size_t)blockIdx.x * per;
        const size_t hi = lo + per < nblock ? lo + per : nblock;
        auto emit = [&](size_t block, const u32x4 (&v)[V]) {
            float y[8];
            if (DT == FP8_BF16) {
#pragma unroll
                for (int d = 0; d < 4; ++d) { y[2 * d] = as_f32(v[0][d] << 16) * s; y[2 * d + 1] = as_f32(v[0][d] & 0xffff0000u) * s; }
            } else {
#pragma unroll
                for (int d = 0; d < 8; ++d) y[d] = as_f32(v[V - 1 < d / 4 ? V - 1 : d / 4][d & 3]) * s;
            }
            unsigned w[4];
            philox4x32_10((unsigned)block, (unsigned)(block >> 32), seed_lo, seed_hi, w);
            qp[block] = (u32x2){encode_sr4<FMT>(y[0], y[1], y[2], y[3], w[0], w[1]),
                                encode_sr4<FMT>(y[4], y[5], y[6], y[7], w[2], w[3])};
        };
        size_t b = lo + threadIdx.x;
        for (; b + (U - 1) * kThreads < hi; b += U * kThreads) {
            u32x4 v[U][V];
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int k = 0; k < V; ++k) v[u][k] = __builtin_nontemporal_load(&xv[V * (b + (size_t)u * kThreads) + k]);
#pragma unroll
            for (int u = 0; u < U; ++u) emit(b + (size_t)u * kThreads, v[u]);
        }
        for (; b < hi; b += kThreads) {
            u32x4 v[V];
#pragma unroll
            for (int k = 0; k < V; ++k) v[k] = __builtin_nontemporal_load(&xv[V * b + k]);
            emit(b, v);
        }
        done = nblock * 8;
    }
    const size_t stride = (size_t)gridDim.x * kThreads;
    for (size_t t = done + (size_t)blockIdx.x * kThreads + threadIdx.x; t < n; t += stride) {
        const size_t block = t / 8;
        unsigned w[4];
        philox4x32_10((unsigned)block, (unsigned)(block >> 32), seed_lo, seed_hi, w);
        const unsigned f = (unsigned)(t % 8);
        const unsigned r = (w[f / 2] >> (16 * (f % 2))) & 0xffffu;
        q[t] = (uint8_t)encode_sr_bits<FMT>(load_scalar<DT>(x, t) * s, r);
    }
}

#define FP8MM_DISPATCH_DT_FMT(KERNEL, grid, ...)                                                           \
    do {                                                                                                   \
        if (in_dtype == FP8_F32) {                                                                         \
            if (fmt == FP8_E4M3) hipLaunchKernelGGL((KERNEL<FP8_F32, FP8_E4M3>), grid, dim3(kThreads), 0, stream, __VA_ARGS__); \
            else hipLaunchKernelGGL((KERNEL<FP8_F32, FP8_E5M2>), grid, dim3(kThreads), 0, stream, __VA_ARGS__);                 \
        } else {                                                                                           \
            if (fmt == FP8_E4M3) hipLaunchKernelGGL((KERNEL<FP8_BF16, FP8_E4M3>), grid, dim3(kThreads), 0, stream, __VA_ARGS__); \
            else hipLaunchKernelGGL((KERNEL<FP8_BF16, FP8_E5M2>), grid, dim3(kThreads), 0, stream, __VA_ARGS__);                \
        }                                                                                                  \
    } while (0)

}  // namespace

int launch_quantize_amax(const void* x, size_t n, int in_dtype, int fmt, const float* scale_dev, uint8_t* q_out,
                         float* amax_out, hipStream_t stream)
{
    unsigned* bits = (unsigned*)amax_out;
    hipLaunchKernelGGL(store_u32_kernel, dim3(1), dim3(1), 0, stream, bits, 0u);
    if (n == 0) return check_launch("quantize_amax init");
    const bool vec = aligned16(x) && aligned16(q_out);
    // Measured (bf16, E4M3): up to a few hundred MB of output 512 workgroups (one atomic each) and
    // ordinary stores are best (2^28 elements: 134 us, against 142 with 16384 workgroups and 148 with
    // non-temporal stores); an output beyond the memory-side cache goes out non-temporally from many
    // short runs (6.04 10^8 elements: 329 us against 367).
    const bool nts = n >= kStreamingStoreBytes;
    const dim3 grid(vec ? grid_for((n / 16 + 3) / 4, nts ? kCastBlocks : 512) : grid_for(n, 2048));
#define FP8MM_QA(DT, FMT)                                                                                                   \
    do {                                                                                                                    \
        if (nts) hipLaunchKernelGGL((quantize_amax_kernel<DT, FMT, true>), grid, dim3(kThreads), 0, stream, x, n, scale_dev, q_out, bits, vec); \
        else hipLaunchKernelGGL((quantize_amax_kernel<DT, FMT, false>), grid, dim3(kThreads), 0, stream, x, n, scale_dev, q_out, bits, vec);    \
    } while (0)
    if (in_dtype == FP8_F32) { if (fmt == FP8_E4M3) FP8MM_QA(FP8_F32, FP8_E4M3); else FP8MM_QA(FP8_F32, FP8_E5M2); }
    else { if (fmt == FP8_E4M3) FP8MM_QA(FP8_BF16, FP8_E4M3); else FP8MM_QA(FP8_BF16, FP8_E5M2); }
#undef FP8MM_QA
    return check_launch("quantize_amax");
}

int launch_quantize_sr(const void* x, size_t n, int in_dtype, int fmt, float scale, const float* scale_dev,
                       uint64_t seed, uint8_t* q_out, hipStream_t stream)
{
    if (n == 0) return FP8_OK;
    const bool vec = aligned16(x) && aligned16(q_out);
    const dim3 grid(vec ? grid_for((n / 8 + 3) / 4, kCastBlocks) : grid_for(n, 2048));     // 4 blocks of 8 elements per lane
    FP8MM_DISPATCH_DT_FMT(quantize_sr_kernel, grid, x, n, scale, scale_dev, (unsigned)seed, (unsigned)(seed >> 32), q_out, vec);
    return check_launch("quantize_sr");
}

int launch_scale_from_history(const float* hist, size_t len, int fmt, float* scale_out, hipStream_t stream)
{
    hipLaunchKernelGGL(scale_from_history_kernel, dim3(1), dim3(kThreads), 0, stream, hist, len, fmt, scale_out);
    return check_launch("scale_from_amax_history");
}

int launch_scale_n(const float* amax, size_t n, int fmt, float* scale_out, hipStream_t stream)
{
    if (n == 0) return FP8_OK;
    hipLaunchKernelGGL(scale_n_kernel, dim3(grid_for(n, 1024)), dim3(kThreads), 0, stream, amax, n, fmt, scale_out);
    return check_launch("scale_from_amax_n");
}

int launch_amax_rows(const void* x, int64_t rows, int64_t cols, int in_dtype, float* amax_out, hipStream_t stream)
{
    if (rows == 0) return FP8_OK;
    const size_t esz = in_dtype == FP8_F32 ? 4 : 2;
    const bool vec = aligned16(x) && ((size_t)cols * esz) % 16 == 0;
    const dim3 grid((unsigned)(rows < 65536 ? rows : 65536));
    if (in_dtype == FP8_F32) hipLaunchKernelGGL(amax_rows_kernel<FP8_F32>, grid, dim3(kThreads), 0, stream, x, rows, cols, amax_out, vec);
    else hipLaunchKernelGGL(amax_rows_kernel<FP8_BF16>, grid, dim3(kThreads), 0, stream, x, rows, cols, amax_out, vec);
    return check_launch("amax_rows");
}

int launch_quantize_rows(const void* x, int64_t rows, int64_t cols, int in_dtype, int fmt, const float* scale_dev,
                         uint8_t* q_out, hipStream_t stream)
{
    if (rows == 0 || cols == 0) return FP8_OK;
    const bool vec = aligned16(x) && aligned16(q_out) && cols % 16 == 0;
    const dim3 grid((unsigned)(rows < 65536 ? rows : 65536));
    FP8MM_DISPATCH_DT_FMT(quantize_rows_kernel, grid, x, rows, cols, scale_dev, q_out, vec);
    return check_launch("quantize_rows");
}

int launch_quantize_transpose(const void* x, int64_t rows, int64_t cols, int in_dtype, int fmt, const float* scale_dev,
                              uint8_t* q_out, uint8_t* qt_out, hipStream_t stream)
{
    if (rows == 0 || cols == 0) return FP8_OK;
    const int tcols = in_dtype == FP8_BF16 ? TransposeTile<FP8_BF16>::cols : TransposeTile<FP8_F32>::cols;
    const int64_t tiles_r = (rows + TT - 1) / TT, tiles_c = (cols + tcols - 1) / tcols;
    const bool vec = aligned16(x) && aligned16(qt_out) && (!q_out || aligned16(q_out)) && rows % 16 == 0 && cols % 16 == 0 &&
                     tiles_r * tiles_c < (1ll << 31);
    if (vec) {
        const dim3 grid((unsigned)(tiles_r * tiles_c));
        const bool diagonal = rows >= 4096 && (rows & (rows - 1)) == 0;      // see "Tile order" at the kernel
        FP8MM_DISPATCH_DT_FMT(quantize_transpose_kernel, grid, x, rows, cols, scale_dev, q_out, qt_out, (int)tiles_r, (int)tiles_c, diagonal);
    } else {
        const dim3 grid(grid_for((size_t)rows * (size_t)cols, 4096));
        FP8MM_DISPATCH_DT_FMT(quantize_transpose_scalar_kernel, grid, x, rows, cols, scale_dev, q_out, qt_out);
    }
    return check_launch("quantize_transpose");
}

}  // namespace fp8mm
