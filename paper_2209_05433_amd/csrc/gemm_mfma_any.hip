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
// 32 KB of LDS and about 150 registers per lane: several workgroups share a compute unit and hide
// each other's barriers and load latencies; nothing here is pipelined by hand.
#include "gemm_common.hpp"

#include <type_traits>

namespace fp8mm {
namespace {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

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

    // ---- epilogue: c = acc / (sA sB) element by element, as in the generic kernel -----------------
    const float sA_host = ep.sA, sB_host = ep.sB;     // by value: a choice between two memory locations would cost scratch
    const bool uniform = !ep.a_per_row && !ep.b_per_col;
    const float r_uniform = uniform ? (float)(1.0 / ((double)scale_value(ep.sA_dev, sA_host) * (double)scale_value(ep.sB_dev, sB_host))) : 0.0f;
    const float sD = (ep.out_kind >= OUT_E4M3) ? scale_value(ep.sD_dev, 1.0f) : 1.0f;
    unsigned amax_bits = 0;
#pragma unroll
    for (int mb = 0; mb < 2; ++mb) {
        const int64_t gm = m0 + wm * 64 + mb * 32 + r;
        if (gm >= M) continue;
        const double a = ep.a_per_row ? (double)ep.sA_dev[gm] : (double)scale_value(ep.sA_dev, sA_host);
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int64_t gn = n0 + wn * 64 + nb * 32 + 8 * (e >> 2) + 4 * h + (e & 3);
                if (gn >= N) continue;
                float rcp = r_uniform;
                if (!uniform) {
                    const double b = ep.b_per_col ? (double)ep.sB_dev[gn] : (double)scale_value(ep.sB_dev, sB_host);
                    rcp = (float)(1.0 / (a * b));
                }
                const float c = acc[nb][mb][e] * rcp;
                amax_bits = max(amax_bits, as_u32(c) & 0x7fffffffu);
                const int64_t o = gm * N + gn;
                switch (ep.out_kind) {
                    case OUT_F32: ((float*)C)[o] = c; break;
                    case OUT_BF16: ((unsigned short*)C)[o] = (unsigned short)bf16_bits_any(c); break;
                    case OUT_E4M3: ((uint8_t*)C)[o] = (uint8_t)encode_bits<FP8_E4M3>(c * sD); break;
                    default: ((uint8_t*)C)[o] = (uint8_t)encode_bits<FP8_E5M2>(c * sD); break;
                }
            }
    }
    if (ep.amax_out) wave_amax_commit(amax_bits, ep.amax_out);
}

template <int FA, int FB, bool A_KC, bool B_KC>
int launch_one(const GemmArgs& g, unsigned tiles)
{
    hipLaunchKernelGGL((gemm_mfma_any_kernel<FA, FB, A_KC, B_KC>), dim3(tiles), dim3(256), 0, g.stream, g.A, g.B, g.C,
                       g.M, g.N, g.K, g.ep);
    return check_launch("gemm (matrix-core kernel for any shape)");
}

template <int FA, int FB>
int launch_layout(const GemmArgs& g, unsigned tiles)
{
    // A stored M x K is K-contiguous; B stored N x K (transB) is K-contiguous
    if (!g.transA) return g.transB ? launch_one<FA, FB, true, true>(g, tiles) : launch_one<FA, FB, true, false>(g, tiles);
    return g.transB ? launch_one<FA, FB, false, true>(g, tiles) : launch_one<FA, FB, false, false>(g, tiles);
}

int64_t tile_count(const GemmArgs& g) { return ((g.M + FT - 1) / FT) * ((g.N + FT - 1) / FT); }

}  // namespace

bool mfma_any_takes(const GemmArgs& g)
{
    return g.M > 0 && g.N > 0 && g.K > 0 && tile_count(g) <= 0x7fffffffll;
}

int launch_mfma_any(const GemmArgs& g)
{
    const unsigned tiles = (unsigned)tile_count(g);
    if (g.fmtA == FP8_E4M3)
        return g.fmtB == FP8_E4M3 ? launch_layout<FP8_E4M3, FP8_E4M3>(g, tiles) : launch_layout<FP8_E4M3, FP8_E5M2>(g, tiles);
    return g.fmtB == FP8_E4M3 ? launch_layout<FP8_E5M2, FP8_E4M3>(g, tiles) : launch_layout<FP8_E5M2, FP8_E5M2>(g, tiles);
}

}  // namespace fp8mm
