// Matrix-core GEMM for any shape and any alignment, for gfx950 (MI355X).
//
//   c[M x N] = (op(A)[M x K] x op(B)[K x N]) / (sA sB),   D = cast_out(c)
//
// The tiled kernel (gemm_tiled.hip) fills its LDS with direct global->LDS loads of aligned 16-byte
// chunks and therefore wants K in multiples of 16 and operand rows that start on 16-byte
// boundaries.  This kernel serves everything else (an odd K, an odd leading dimension such as a
// vocabulary size with the weight stored [in, out], operands at any address) at a fraction of the
// tiled kernel's rate instead of the small fraction of a per cent that plain FMAs give:
//   - 128 x 128 output tile per workgroup of 4 waves (64 x 64 per wave as 2 x 2 blocks of 32 x 32),
//     K walked in stages of 64;
//   - a thread fetches 2 x 16 bytes of each operand per stage into registers with unaligned vector
//     loads (byte by byte, with zeros beyond the edges, where the 16 bytes would leave the row), one
//     stage ahead of the products, widens them exactly to fp16 (both FP8 formats embed in fp16) and
//     writes them to LDS in one layout for every storage order: 64 consecutive-K halves per row of
//     op(A) / column of op(B).  An operand that is contiguous along M / N in memory is transposed by
//     that write (32 two-byte writes per thread and stage);
//   - fragments are plain 16-byte LDS reads, the products v_mfma_f32_32x32x16_f16 with fp32
//     accumulation: the arithmetic of the tiled kernel's default mode, so the same error bound
//     holds (arXiv 2209.05433, Section 2: FP8 operands, single-precision accumulation, factors
//     taken out once per output);
//   - the epilogue is that of the generic kernel, element by element (any N, any output alignment).
// 32 KB of LDS and about 100 registers per lane: several workgroups share a compute unit and hide
// each other's barriers and load latencies; nothing in this form is pipelined by hand.  Problems of
// many tiles take the wide form further down (256 x 256 tiles, one workgroup per compute unit).
#include "gemm_common.hpp"

#include <atomic>
#include <type_traits>

namespace fp8mm {
namespace {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 v4h __attribute__((ext_vector_type(4)));

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))

constexpr int FT = 128;                 // tile edge
constexpr int FK = 64;                  // K per stage
constexpr int NV = FK / 32;             // 16-byte vectors per thread, operand and stage
constexpr int FPITCH = 2 * FK;          // bytes per LDS row: FK halves = 8 chunks of 16 bytes
constexpr int FGROUP = 8;               // tile rows per band of the tile order

// fp32 -> bf16 bits, round to nearest even; NaN stays NaN.
__device__ __forceinline__ unsigned bf16_bits_any(float f)
{
    const unsigned u = as_u32(f);
    const unsigned r = (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
    return (u & 0x7fffffffu) > 0x7f800000u ? ((u >> 16) | 0x40u) : r;
}

// 16 bytes p[0..15] if `whole`, else p[j] for j < count and zeros beyond (count may be <= 0).
__device__ __forceinline__ u32x4 load16_guarded(const uint8_t* p, bool whole, int64_t count)
{
    u32x4 v = {0u, 0u, 0u, 0u};
    if (whole) {
        __builtin_memcpy(&v, p, 16);                     // no alignment assumed: the target loads 16 bytes from any address
    } else {
#pragma unroll
        for (int j = 0; j < 16; ++j)
            if (j < count) v[j >> 2] |= (unsigned)p[j] << (8 * (j & 3));
    }
    return v;
}

// Vector v (of NV) of the thread's bytes of one operand for the stage that starts at k0.  `ext` = rows
// of op(A) / columns of op(B), t0 = first one of the tile.
//   KC (contiguous along K: element (r, k) at base[r K + k]): row 64 v + tid / 4, K bytes 16 (tid % 4) ..
//      (four lanes cover the 64 bytes of a row: a wave's load touches 16 rows, not 32)
//   MC (contiguous along M / N: element (r, k) at base[k ext + r]): K-row 32 v + tid / 8, rows 16 (tid % 8) ..
template <bool KC>
__device__ __forceinline__ u32x4 fetch_stage(const uint8_t* base, int64_t ext, int64_t K, int64_t t0, int64_t k0, int tid, int v)
{
    if (KC) {
        const int64_t r = t0 + 64 * v + (tid >> 2), k = k0 + (tid & 3) * 16;
        if (r >= ext) return (u32x4){0u, 0u, 0u, 0u};
        return load16_guarded(base + r * K + k, k + 16 <= K, K - k);
    }
    const int64_t k = k0 + 32 * v + (tid >> 3), r = t0 + (tid & 7) * 16;
    if (k >= K) return (u32x4){0u, 0u, 0u, 0u};
    return load16_guarded(base + k * ext + r, r + 16 <= ext, ext - r);
}

// LDS image of an operand: row = row of op(A) / column of op(B) inside the tile, FK halves along K
// per row as 8 chunks of 16 bytes; chunk c of row `row` sits at position c ^ swz(row).  The first
// term of swz is the swizzle of the tiled kernel's K-contiguous slabs (same row length, same
// 16-byte fragment reads: conflict-free there); the second spreads the 8 column groups of a
// transposing write (rows 16 apart, which otherwise meet in one bank: measured, 75 % of the active
// LDS cycles were conflict cycles and the LDS was busy 90 % of the time) and is constant over the
// 16 rows that one pass of a fragment read covers.
__device__ __forceinline__ int swz(int row) { return ((row >> 1) ^ (row >> 4)) & 7; }

// The thread's 16 bytes, widened, into the image.
template <int FMT, bool KC>
__device__ __forceinline__ void store_stage(uint8_t* img, u32x4 x, int tid, int v)
{
    const v8h lo = widen8<FMT>((int)x.x, (int)x.y), hi = widen8<FMT>((int)x.z, (int)x.w);
    if (KC) {
        const int row = 64 * v + (tid >> 2), c = 2 * (tid & 3);   // chunks c, c + 1
        uint8_t* dst = img + row * FPITCH;
        *LDS_PTR(v8h, dst + ((c ^ swz(row)) * 16)) = lo;
        *LDS_PTR(v8h, dst + (((c + 1) ^ swz(row)) * 16)) = hi;
    } else {
        const int k = 32 * v + (tid >> 3), row0 = (tid & 7) * 16;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int row = row0 + j;
            *LDS_PTR(_Float16, img + row * FPITCH + (((k >> 3) ^ swz(row)) * 16) + (k & 7) * 2) = j < 8 ? lo[j] : hi[j - 8];
        }
    }
}

// Workgroup id -> tile.  Ids go round-robin over the 8 XCDs (each with its own L2); XCD x gets one
// contiguous run of the order below, so that the tiles it works on at a time share a few row slabs
// of A and column slabs of B in its L2 (dealt out id by id, every XCD streamed all of B once per
// band: 47 GB of L2 fills for 0.7 GB of operands, measured).  Order: bands of FGROUP tile rows,
// down the rows of a band first, then to the next tile column.
__device__ __forceinline__ void tile_of(int64_t bid, int64_t tiles_m, int64_t tiles_n, int64_t& tm, int64_t& tn)
{
    const int64_t total = tiles_m * tiles_n;
    const int64_t x = bid % 8, idx = bid / 8, base = total / 8, rem = total % 8;
    const int64_t p = x * base + (x < rem ? x : rem) + idx;
    const int64_t band_tiles = FGROUP * tiles_n;
    const int64_t band = p / band_tiles, q = p - band * band_tiles;
    const int64_t rows = tiles_m - band * FGROUP < FGROUP ? tiles_m - band * FGROUP : FGROUP;
    tm = band * FGROUP + q % rows;
    tn = q / rows;
}

// Epilogue of both kernels: c = acc / (sA sB) element by element, as in the generic kernel (any N,
// any output alignment).  acc[nb][mb] is the wave's block of 32 columns nb x 32 rows mb; wave_m /
// wave_n = first row / column of the wave's part of C; lane (r, h) holds, per accumulator quad, 4
// consecutive columns of row r of a block.
// Block row MB and, by recursion, those after it: the index into acc is a constant whatever the
// optimizer makes of the loops (an accumulator array indexed by a loop that was not unrolled would
// go to scratch memory).  A lane's columns are col0 + (a constant per element): one row pointer per
// block row and constant offsets, so that no element needs address registers of its own.
template <int OUT, int NBLK, int MB>
__device__ __forceinline__ void store_block_rows(const v16f (&acc)[NBLK][NBLK], void* __restrict__ C, int64_t M, int64_t N,
                                                 int64_t wave_m, int64_t col0, int r, const EpilogueArgs& ep,
                                                 float sA_host, float sB_host, float r_uniform, float sD, bool uniform,
                                                 unsigned& amax_bits)
{
    typedef std::conditional_t<OUT == OUT_F32, float, std::conditional_t<OUT == OUT_BF16, unsigned short, uint8_t>> out_t;
    const int64_t gm = wave_m + MB * 32 + r, cols_left = N - col0;
    if (gm < M) {
        const double a = ep.a_per_row ? (double)ep.sA_dev[gm] : (double)scale_value(ep.sA_dev, sA_host);
        out_t* __restrict__ rowp = (out_t*)C + gm * N + col0;
#pragma unroll
        for (int nb = 0; nb < NBLK; ++nb)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int off = nb * 32 + 8 * (e >> 2) + (e & 3);          // column col0 + off
                if (off >= cols_left) continue;
                float rcp = r_uniform;
                if (!uniform) {
                    const double b = ep.b_per_col ? (double)ep.sB_dev[col0 + off] : (double)scale_value(ep.sB_dev, sB_host);
                    rcp = (float)(1.0 / (a * b));
                }
                const float c = acc[nb][MB][e] * rcp;
                amax_bits = max(amax_bits, as_u32(c) & 0x7fffffffu);
                if (OUT == OUT_F32) rowp[off] = (out_t)c;
                else if (OUT == OUT_BF16) rowp[off] = (out_t)bf16_bits_any(c);
                else if (OUT == OUT_E4M3) rowp[off] = (out_t)encode_bits<FP8_E4M3>(c * sD);
                else rowp[off] = (out_t)encode_bits<FP8_E5M2>(c * sD);
            }
    }
    if constexpr (MB + 1 < NBLK)
        store_block_rows<OUT, NBLK, MB + 1>(acc, C, M, N, wave_m, col0, r, ep, sA_host, sB_host, r_uniform, sD, uniform, amax_bits);
}

template <int OUT, int NBLK>
__device__ __forceinline__ void store_outputs_as(const v16f (&acc)[NBLK][NBLK], void* __restrict__ C, int64_t M, int64_t N,
                                                 int64_t wave_m, int64_t wave_n, int r, int h, const EpilogueArgs& ep)
{
    const float sA_host = ep.sA, sB_host = ep.sB;     // by value: a choice between two memory locations would cost scratch
    const bool uniform = !ep.a_per_row && !ep.b_per_col;
    const float r_uniform = uniform ? (float)(1.0 / ((double)scale_value(ep.sA_dev, sA_host) * (double)scale_value(ep.sB_dev, sB_host))) : 0.0f;
    const float sD = (OUT >= OUT_E4M3) ? scale_value(ep.sD_dev, 1.0f) : 1.0f;
    unsigned amax_bits = 0;
    store_block_rows<OUT, NBLK, 0>(acc, C, M, N, wave_m, wave_n + 4 * h, r, ep, sA_host, sB_host, r_uniform, sD, uniform, amax_bits);
    if (ep.amax_out) wave_amax_commit(amax_bits, ep.amax_out);
}

template <int NBLK>
__device__ __forceinline__ void store_outputs(const v16f (&acc)[NBLK][NBLK], void* __restrict__ C, int64_t M, int64_t N,
                                              int64_t wave_m, int64_t wave_n, int r, int h, const EpilogueArgs& ep)
{
    switch (ep.out_kind) {
        case OUT_F32: store_outputs_as<OUT_F32>(acc, C, M, N, wave_m, wave_n, r, h, ep); break;
        case OUT_BF16: store_outputs_as<OUT_BF16>(acc, C, M, N, wave_m, wave_n, r, h, ep); break;
        case OUT_E4M3: store_outputs_as<OUT_E4M3>(acc, C, M, N, wave_m, wave_n, r, h, ep); break;
        default: store_outputs_as<OUT_E5M2>(acc, C, M, N, wave_m, wave_n, r, h, ep); break;
    }
}

int64_t tile_count(const GemmArgs& g, int64_t edge) { return ((g.M + edge - 1) / edge) * ((g.N + edge - 1) / edge); }

template <int FMT_A, int FMT_B, bool A_KC, bool B_KC>
__global__ __launch_bounds__(256) void gemm_mfma_any_kernel(
    const uint8_t* __restrict__ A, const uint8_t* __restrict__ B, void* __restrict__ C,
    int64_t M, int64_t N, int64_t K, EpilogueArgs ep)
{
    __shared__ __attribute__((aligned(16))) uint8_t As[FT * FPITCH];
    __shared__ __attribute__((aligned(16))) uint8_t Bs[FT * FPITCH];
    const int tid = threadIdx.x;
    const int w = tid >> 6, l = tid & 63;
    const int wm = w >> 1, wn = w & 1, r = l & 31, h = l >> 5;
    const int64_t tiles_m = (M + FT - 1) / FT, tiles_n = (N + FT - 1) / FT;
    int64_t tm, tn;
    tile_of(blockIdx.x, tiles_m, tiles_n, tm, tn);
    const int64_t m0 = tm * FT, n0 = tn * FT;

    v16f acc[2][2];                                   // [block of 32 columns][block of 32 rows]
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    u32x4 ra[NV], rb[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        ra[v] = fetch_stage<A_KC>(A, M, K, m0, 0, tid, v);
        rb[v] = fetch_stage<B_KC>(B, N, K, n0, 0, tid, v);
    }
    for (int64_t k0 = 0; k0 < K; k0 += FK) {
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            store_stage<FMT_A, A_KC>(As, ra[v], tid, v);
            store_stage<FMT_B, B_KC>(Bs, rb[v], tid, v);
        }
        __syncthreads();
        if (k0 + FK < K) {                            // the next stage's bytes travel while this one is multiplied
#pragma unroll                                        // (a second register set, two stages ahead, cost a wave of
            for (int v = 0; v < NV; ++v) {            // occupancy and measured 4 % slower)
                ra[v] = fetch_stage<A_KC>(A, M, K, m0, k0 + FK, tid, v);
                rb[v] = fetch_stage<B_KC>(B, N, K, n0, k0 + FK, tid, v);
            }
        }
        // lane (r, h) supplies row / column r of a block and, per instruction, the 8 halves 8 h .. 8 h + 7
        // of its 16; D[i][j] gets i from operand 0 (B: columns of C) and j from operand 1 (A: rows of C),
        // so a lane ends up with 4 consecutive columns of one row of C per accumulator quad
#pragma unroll
        for (int s = 0; s < FK / 16; ++s) {
            v8h af[2], bf[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int ra_ = wm * 64 + i * 32 + r, rb_ = wn * 64 + i * 32 + r;
                const int c = 2 * h + (s & 1) + 4 * (s >> 1);      // which 8 of the 64 halves: any assignment that is
                af[i] = *LDS_PTR(v8h, As + ra_ * FPITCH + ((c ^ swz(ra_)) * 16));    // the same for A and B will do;
                bf[i] = *LDS_PTR(v8h, Bs + rb_ * FPITCH + ((c ^ swz(rb_)) * 16));    // this one is the tiled kernel's
            }
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                for (int mb = 0; mb < 2; ++mb)
                    acc[nb][mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(bf[nb], af[mb], acc[nb][mb], 0, 0, 0);
        }
        __syncthreads();
    }

    store_outputs<2>(acc, C, M, N, m0 + wm * 64, n0 + wn * 64, r, h, ep);
}

// ---- the wide form ------------------------------------------------------------------------------
// For problems of many tiles: a 256 x 256 tile per workgroup (128 x 128 per wave as 4 x 4 blocks,
// half the LDS reads per product of the 2 x 2 form), one workgroup per compute unit, so nobody
// hides a workgroup's waits but itself:
//   - the LDS holds two stages of both images (128 KB); stage s is multiplied out of one half
//     while stage s + 1 is written into the other;
//   - two register sets: the bytes of stage s + 2 are requested before stage s is multiplied; a
//     stage later they are widened and written to LDS in eight pieces, issued between the matrix
//     instructions of the first three of that stage's four K sub-steps;
//   - one barrier per stage, before its last K sub-step, during which the first fragments of the
//     next stage are already read (see the kernel);
//   - an operand that is contiguous along M / N is fetched as 4 consecutive K rows x 16 tile rows per
//     thread and turned round in registers (byte permutes), so that the image gets 8-byte writes
//     (4 halves along K) instead of 2-byte ones;
//   - stages that lie inside K, of tiles that lie inside C, run a loop without a single test.
constexpr int WT = 256;                         // tile edge
constexpr int WNV = WT * FK / 16 / 256;         // 16-byte vectors per thread, operand and stage: 4
constexpr int W_IMG = WT * FPITCH;              // one operand, one stage: 32 KB
constexpr int W_LDS = 4 * W_IMG;

// Sixteen zero bytes in device memory, never written: what a lane of the wide form loads in place of
// a piece that is not wholly inside its row.
__device__ __attribute__((aligned(16))) uint8_t g_any_zero_chunk[16];

// Where vector v (of WNV) of the thread's bytes for the stage that starts at k0 lies, and how many
// of its 16 bytes exist (16 = all; <= 0 = none: the piece lies beyond the edge of the operand):
//   KC: as in fetch_stage (row 64 v + tid / 4, K bytes 16 (tid % 4) ..);
//   MC: K-row 4 (tid / 16) + v, tile rows 16 (tid % 16) .. : 16 lanes cover the 256 bytes of a K-row.
template <bool KC>
__device__ __forceinline__ const uint8_t* piece_wide(const uint8_t* base, int64_t ext, int64_t K, int64_t t0, int64_t k0, int tid, int v,
                                                     int64_t& count)
{
    if (KC) {
        const int64_t r = t0 + 64 * v + (tid >> 2), k = k0 + (tid & 3) * 16;
        count = r < ext ? K - k : 0;
        return base + r * K + k;
    }
    const int64_t k = k0 + 4 * (tid >> 4) + v, r = t0 + (tid & 15) * 16;
    count = k < K ? ext - r : 0;
    return base + k * ext + r;
}

// The thread's WNV vectors of one operand for the stage that starts at k0.  First one 16-byte load per
// vector, unconditionally (whole pieces from the operand, the others from the zero chunk); only then
// the pieces that straddle an edge, byte by byte.  In that order the number of loads issued after
// any earlier load has a known minimum, and the waits for the stage fetched before this one leave
// this stage's loads in flight.  (With each piece's choice between one load and its bytes made in
// place, every wait for older bytes also waited for the loads just issued.)
template <bool KC>
__device__ __forceinline__ void fetch_wide(u32x4 (&x)[WNV], const uint8_t* base, int64_t ext, int64_t K, int64_t t0, int64_t k0, int tid)
{
    const uint8_t* p[WNV];
    int64_t count[WNV];
#pragma unroll
    for (int v = 0; v < WNV; ++v) {
        p[v] = piece_wide<KC>(base, ext, K, t0, k0, tid, v, count[v]);
        __builtin_memcpy(&x[v], count[v] >= 16 ? p[v] : g_any_zero_chunk, 16);
    }
#pragma unroll
    for (int v = 0; v < WNV; ++v)
        if (count[v] > 0 && count[v] < 16) {
            u32x4 e = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int j = 0; j < 16; ++j)
                if (j < count[v]) e[j >> 2] |= (unsigned)p[v][j] << (8 * (j & 3));
            x[v] = e;
        }
}

// Piece q (of 2 WNV) of the thread's share of writing an operand's stage into its image; d = q / 2.
//   KC: 8 of the 16 bytes of vector d, placed as in store_stage.
//   MC: byte j of x[v] is the element of tile row 16 (tid % 16) + j at K index 4 (tid / 16) + v; the
//       piece takes the tile rows 4 d + 2 (q % 2) and the one after it: 4 x 2 bytes (K index x tile
//       row) are turned into 2 words, one per tile row with K ascending, widened, and written as
//       4 halves (8 bytes) per row.
template <int FMT, bool KC>
__device__ __forceinline__ void store_wide_piece(uint8_t* img, const u32x4 (&x)[WNV], int tid, int q)
{
    const int d = q >> 1, second = q & 1;
    if (KC) {
        const int row = 64 * d + (tid >> 2), c = 2 * (tid & 3) + second;
        const v8h hv = second ? widen8<FMT>((int)x[d].z, (int)x[d].w) : widen8<FMT>((int)x[d].x, (int)x[d].y);
        *LDS_PTR(v8h, img + row * FPITCH + ((c ^ swz(row)) * 16)) = hv;
        return;
    }
    const int kg = tid >> 4, row = (tid & 15) * 16 + 4 * d + 2 * second;
    const int chunk = kg >> 1, inner = (kg & 1) * 8;          // 8 halves per 16-byte chunk: K indices 4 kg .. 4 kg + 3
    const unsigned sel = second ? 0x07030602u : 0x05010400u;  // bytes 2, 3 / 0, 1 of both words, interleaved
    const unsigned t = __builtin_amdgcn_perm(x[1][d], x[0][d], sel), u = __builtin_amdgcn_perm(x[3][d], x[2][d], sel);
    const unsigned w0 = __builtin_amdgcn_perm(u, t, 0x05040100u), w1 = __builtin_amdgcn_perm(u, t, 0x07060302u);
    const v8h hv = widen8<FMT>((int)w0, (int)w1);
    *LDS_PTR(v4h, img + (row + 0) * FPITCH + ((chunk ^ swz(row + 0)) * 16) + inner) = (v4h){hv[0], hv[1], hv[2], hv[3]};
    *LDS_PTR(v4h, img + (row + 1) * FPITCH + ((chunk ^ swz(row + 1)) * 16) + inner) = (v4h){hv[4], hv[5], hv[6], hv[7]};
}

template <int FMT_A, int FMT_B, bool A_KC, bool B_KC>
__global__ __launch_bounds__(256) void gemm_mfma_any_wide_kernel(
    const uint8_t* __restrict__ A, const uint8_t* __restrict__ B, void* __restrict__ C,
    int64_t M, int64_t N, int64_t K, EpilogueArgs ep)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];     // [stage parity][A image, B image]
    const int tid = threadIdx.x;
    const int w = tid >> 6, l = tid & 63;
    const int wm = w >> 1, wn = w & 1, r = l & 31, h = l >> 5;
    const int64_t tiles_m = (M + WT - 1) / WT, tiles_n = (N + WT - 1) / WT;
    int64_t tm, tn;
    tile_of(blockIdx.x, tiles_m, tiles_n, tm, tn);
    const int64_t m0 = tm * WT, n0 = tn * WT;
    const int64_t stages = (K + FK - 1) / FK;

    v16f acc[4][4];                                   // [block of 32 columns][block of 32 rows]
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    auto fetch = [&](u32x4 (&xa)[WNV], u32x4 (&xb)[WNV], int64_t stage) __attribute__((always_inline)) {
        fetch_wide<A_KC>(xa, A, M, K, m0, stage * FK, tid);
        fetch_wide<B_KC>(xb, B, N, K, n0, stage * FK, tid);
    };
    // the same for a stage that lies wholly inside K, of a tile that lies wholly inside C: no tests,
    // and addresses as a base per stage (the same for the whole workgroup) plus the thread's offset
    // of each vector within the tile's stage (fits 32 bits: see mfma_any_wide)
    unsigned offa[WNV], offb[WNV];
#pragma unroll
    for (int v = 0; v < WNV; ++v) {
        offa[v] = A_KC ? (unsigned)(64 * v + (tid >> 2)) * (unsigned)K + (tid & 3) * 16 : (unsigned)(4 * (tid >> 4) + v) * (unsigned)M + (tid & 15) * 16;
        offb[v] = B_KC ? (unsigned)(64 * v + (tid >> 2)) * (unsigned)K + (tid & 3) * 16 : (unsigned)(4 * (tid >> 4) + v) * (unsigned)N + (tid & 15) * 16;
    }
    const uint8_t* tile_a = A + (A_KC ? m0 * K : m0);
    const uint8_t* tile_b = B + (B_KC ? n0 * K : n0);
    auto fetch_inside = [&](u32x4 (&xa)[WNV], u32x4 (&xb)[WNV], int64_t stage) __attribute__((always_inline)) {
        const uint8_t* sa = tile_a + stage * FK * (A_KC ? 1 : M);
        const uint8_t* sb = tile_b + stage * FK * (B_KC ? 1 : N);
#pragma unroll
        for (int v = 0; v < WNV; ++v) {
            __builtin_memcpy(&xa[v], sa + offa[v], 16);
            __builtin_memcpy(&xb[v], sb + offb[v], 16);
        }
    };
    // lane (r, h): fragments of the K indices 16 s .. 16 s + 15 of the stage in half `parity`.  Block i
    // of the wave is row r0 + 32 i of the image, chunk c = 2 h + (s & 1) + 4 (s >> 1) at position
    // c ^ swz(row).  Adding 32 i to the row flips swz by 2 i, and c is 2 h with constant bits flipped, so
    // an address is one value per lane with three bits flipped by a constant, plus a constant: two
    // registers hold what would otherwise be an address per block and sub-step.
    const unsigned lane_a = (unsigned)((wm * 128 + r) * FPITCH) + (unsigned)(((2 * h) ^ swz(wm * 128 + r)) << 4);
    const unsigned lane_b = (unsigned)((wn * 128 + r) * FPITCH) + (unsigned)(((2 * h) ^ swz(wn * 128 + r)) << 4) + W_IMG;
    auto read_frags = [&](int parity, int s, v8h (&af)[4], v8h (&bf)[4]) __attribute__((always_inline)) {
        const int cs = (s & 1) + 4 * (s >> 1);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const unsigned flip = (unsigned)(((cs ^ (2 * i)) & 7) << 4), add = (unsigned)(i * 32 * FPITCH + parity * 2 * W_IMG);
            af[i] = *LDS_PTR(v8h, lds + ((lane_a ^ flip) + add));
            bf[i] = *LDS_PTR(v8h, lds + ((lane_b ^ flip) + add));
        }
    };
    // One stage: the products of the stage in half `parity`, in four K sub-steps.  On entry fa[0],
    // fb[0] hold the fragments of sub-step 0; the fragments of a sub-step are read during the one
    // before it.  STORE: meanwhile (xa, xb), the bytes of the next stage, go into the other half
    // during the first three sub-steps, in eight pieces, so that the widening and the LDS writes
    // are issued between the matrix instructions and not after them.  The stage's barrier stands
    // before the last sub-step: by then this wave has read all its fragments of this half and
    // written its share of the other half, and after it the fragments of the next stage's sub-step
    // 0 are read from the other half during the last sub-step's products (behind the last stage
    // they are read for nothing).
    // Since every wave's reads of a half precede the barrier of that stage, the writes into it, which
    // belong to the stage after, follow that barrier.
    v8h fa[2][4], fb[2][4];
    auto stage = [&](auto store_tag, int parity, const u32x4 (&xa)[WNV], const u32x4 (&xb)[WNV]) __attribute__((always_inline)) {
        constexpr bool STORE = decltype(store_tag)::value;
        constexpr int STEPS = FK / 16;
        uint8_t* other = lds + (parity ^ 1) * 2 * W_IMG;
        // sub-step S with the pieces FIRST .. LAST - 1 of the store
        auto substep = [&](auto s_c, auto first_c, auto last_c) __attribute__((always_inline)) {
            constexpr int S = decltype(s_c)::value, FIRST = decltype(first_c)::value, LAST = decltype(last_c)::value;
            constexpr int PIECES = STORE ? LAST - FIRST : 0;
            if (S == STEPS - 1) __syncthreads();
            if (S + 1 < STEPS) read_frags(parity, S + 1, fa[(S + 1) & 1], fb[(S + 1) & 1]);
            else read_frags(parity ^ 1, 0, fa[0], fb[0]);
#pragma unroll
            for (int nb = 0; nb < 4; ++nb)
#pragma unroll
                for (int mb = 0; mb < 4; ++mb)
                    acc[nb][mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fb[S & 1][nb], fa[S & 1][mb], acc[nb][mb], 0, 0, 0);
            if (STORE) {
#pragma unroll
                for (int q = FIRST; q < LAST; ++q) {
                    store_wide_piece<FMT_A, A_KC>(other, xa, tid, q);
                    store_wide_piece<FMT_B, B_KC>(other + W_IMG, xb, tid, q);
                }
            }
            // Order asked of the scheduler: after every matrix instruction a few of the sub-step's other
            // instructions (fragment reads, widening, LDS writes, loads), of whatever kind is ready.
            // (Asked for kind by kind, the order fell apart wherever an instruction of the kind asked
            // for was not ready, and most of a sub-step's vector work ended up behind one matrix
            // instruction.)
            constexpr int OTHERS = PIECES == 3 ? 4 : PIECES == 2 ? 3 : 2;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002 | 0x020 | 0x100 | 0x200, OTHERS, 0);
            }
            __builtin_amdgcn_sched_barrier(0);        // nothing drifts into another sub-step (register pressure)
        };
        using std::integral_constant;
        substep(integral_constant<int, 0>{}, integral_constant<int, 0>{}, integral_constant<int, 3>{});
        substep(integral_constant<int, 1>{}, integral_constant<int, 3>{}, integral_constant<int, 6>{});
        substep(integral_constant<int, 2>{}, integral_constant<int, 6>{}, integral_constant<int, 8>{});
        substep(integral_constant<int, 3>{}, integral_constant<int, 8>{}, integral_constant<int, 8>{});
    };

    u32x4 a0[WNV], b0[WNV], a1[WNV], b1[WNV];         // register set 0: even stages, set 1: odd stages
    fetch(a0, b0, 0);
    if (stages > 1) fetch(a1, b1, 1);
#pragma unroll
    for (int q = 0; q < 2 * WNV; ++q) {
        store_wide_piece<FMT_A, A_KC>(lds, a0, tid, q);
        store_wide_piece<FMT_B, B_KC>(lds + W_IMG, b0, tid, q);
    }
    __syncthreads();
    read_frags(0, 0, fa[0], fb[0]);
    // Two stages per trip; an odd last stage follows the loop.  (With the loop left from the middle
    // of a trip, or with a choice between two forms of a stage inside it, the compiler spilled a
    // thousand registers per lane.)  Every condition is the same for the whole workgroup.
    int64_t st = 0;
    // trips whose two fetches need no tests: straight-line code (with branches in the loop the
    // accumulators changed register class, 256 moves, in every stage)
    const int64_t inside = (m0 + WT <= M && n0 + WT <= N) ? K / FK : 0;
    for (; st + 3 < inside; st += 2) {
        fetch_inside(a0, b0, st + 2);
        stage(std::true_type{}, 0, a1, b1);
        fetch_inside(a1, b1, st + 3);
        stage(std::true_type{}, 1, a0, b0);
    }
    // the other trips: edge tiles, and the end of K
    for (; st + 2 <= stages; st += 2) {
        if (st + 2 < stages) fetch(a0, b0, st + 2);
        stage(std::true_type{}, 0, a1, b1);
        if (st + 3 < stages) fetch(a1, b1, st + 3);
        stage(std::true_type{}, 1, a0, b0);           // after the last stage: old bytes into a half nobody reads again
    }
    if (st < stages) stage(std::false_type{}, 0, a0, b0);

    store_outputs<4>(acc, C, M, N, m0 + wm * 128, n0 + wn * 128, r, h, ep);
}

template <int FA, int FB, bool A_KC, bool B_KC>
int launch_one(const GemmArgs& g, bool wide)
{
    if (!wide) {
        hipLaunchKernelGGL((gemm_mfma_any_kernel<FA, FB, A_KC, B_KC>), dim3((unsigned)tile_count(g, FT)), dim3(256), 0, g.stream,
                           g.A, g.B, g.C, g.M, g.N, g.K, g.ep);
        return check_launch("gemm (matrix-core kernel for any shape)");
    }
    // the wide form needs more dynamic LDS than the default limit: raised once per device
    static std::atomic<unsigned long long> attr_set{0ull};
    auto kern = gemm_mfma_any_wide_kernel<FA, FB, A_KC, B_KC>;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return fail(FP8_ERR_DEVICE, "hipGetDevice failed");
    const unsigned long long bit = 1ull << (dev & 63);
    if (dev >= 64 || !(attr_set.load(std::memory_order_relaxed) & bit)) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, W_LDS);
        if (e != hipSuccess)
            return fail(FP8_ERR_DEVICE, "hipFuncSetAttribute(LDS=%d): %s", W_LDS, hipGetErrorString(e));
        if (dev < 64) attr_set.fetch_or(bit, std::memory_order_relaxed);
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)tile_count(g, WT)), dim3(256), W_LDS, g.stream, g.A, g.B, g.C, g.M, g.N, g.K, g.ep);
    return check_launch("gemm (matrix-core kernel for any shape, wide form)");
}

template <int FA, int FB>
int launch_layout(const GemmArgs& g, bool wide)
{
    // A stored M x K is K-contiguous; B stored N x K (transB) is K-contiguous
    if (!g.transA) return g.transB ? launch_one<FA, FB, true, true>(g, wide) : launch_one<FA, FB, true, false>(g, wide);
    return g.transB ? launch_one<FA, FB, false, true>(g, wide) : launch_one<FA, FB, false, false>(g, wide);
}

}  // namespace

bool mfma_any_takes(const GemmArgs& g)
{
    return g.M > 0 && g.N > 0 && g.K > 0 && tile_count(g, FT) <= 0x7fffffffll;
}

// The wide form where its 256 x 256 tiles fill the rounds of one workgroup per compute unit to
// 80 % at least and K is long enough for the two-stage pipeline to pay; FP8_KNOB_TILE_N forces
// either form (128 / 256).
bool mfma_any_wide(const GemmArgs& g)
{
    const int forced = knob(FP8_KNOB_TILE_N);
    const int64_t tiles = tile_count(g, WT), units = 256;
    const int64_t rounds = (tiles + units - 1) / units;
    // 32-bit offsets within a tile's stage: 255 rows of K bytes, or 63 K-rows of M / N bytes
    if (g.K >= (1 << 24) || g.M >= (1 << 26) || g.N >= (1 << 26)) return false;
    if (forced) return forced == 256;
    return g.K >= 8 * FK && 5 * tiles >= 4 * rounds * units;
}

int launch_mfma_any(const GemmArgs& g)
{
    const bool wide = mfma_any_wide(g);
    if (g.fmtA == FP8_E4M3)
        return g.fmtB == FP8_E4M3 ? launch_layout<FP8_E4M3, FP8_E4M3>(g, wide) : launch_layout<FP8_E4M3, FP8_E5M2>(g, wide);
    return g.fmtB == FP8_E4M3 ? launch_layout<FP8_E5M2, FP8_E4M3>(g, wide) : launch_layout<FP8_E5M2, FP8_E5M2>(g, wide);
}

}  // namespace fp8mm
