// Tiled FP8 x FP8 GEMM with fp32 accumulation and the fused epilogue, for gfx950 (MI355X).
//
//   c[M x N] = (op(A)[M x K] x op(B)[K x N]) / (sA sB),   D = cast_out(c)
//
// A and B hold E4M3 / E5M2 bytes (arXiv 2209.05433, Table 1), each in either storage order; the
// products are accumulated in fp32 by the matrix cores and the reciprocals of the scaling factors
// are applied once per output (Section 2); the result is written as fp32, bf16 or FP8.
//
// Conditions (checked by the dispatcher): K a multiple of 16; 16-byte aligned A and B; N a multiple
// of 16 if B is stored K x N, M a multiple of 16 if A is stored K x M.  K is walked in pairs of
// stages (128 bytes); where K is not a multiple of 128 the last pair is filled up with zero bytes.  M and N need not be
// multiples of the tile: loads of rows / columns beyond the edge are redirected to existing ones,
// their outputs are not stored.  Where the rows of C (or a per-column factor vector) do not start
// on 16-byte boundaries the epilogue stores element by element (EpilogueArgs::ragged_n).
//
//   - one workgroup of 4 waves per 256 x 256 output tile, each wave owns 128 x 128 of it as
//     4 x 4 blocks of v_mfma_f32_32x32x64_f8f6f4 (K = 64 per instruction, operand formats
//     selected per operand, so the E5M2 x E4M3 mix costs nothing extra); a 256 x 128 variant
//     (each wave 128 x 64) serves problems with too few wide tiles to fill the chip;
//   - K is walked in stages of 64.  An operand that is contiguous along M / N in memory (B stored
//     K x N, A stored K x M) comes as one 64 x 256 slab (16 KB) per stage in a ring of four; an
//     operand that is contiguous along K (A stored M x K, B stored N x K) as one 256 x 128 slab
//     (32 KB) per pair of stages in a ring of three (two for B if both are of this kind): 160 KB of
//     LDS in all.  Slabs are filled by direct global->LDS loads issued two to four stages ahead of
//     use.  K-contiguous rows are fetched 128 bytes at a time
//     because the vector L1 keeps at most 64 requests to the L2 in flight and asks for whole
//     128-byte lines: 64-byte row pieces double its requests;
//   - the MFMA wants, per lane, 32 consecutive-K bytes of one row of op(A) / one column of op(B).
//     From a K-contiguous slab these are plain 16-byte LDS reads; from the other kind they come
//     through the transposing LDS read ds_read_b64_tr_b8, which hands each lane 8 K-consecutive
//     bytes of one column out of an 8 x 16 byte block.  No transposed copy of an operand is made;
//   - slabs are stored with an XOR swizzle of the 16-byte chunk index so that the fragment reads
//     spread over the LDS banks; the swizzle is applied on the global side of the direct loads
//     (LDS placement of a direct load is fixed: lane i writes 16 bytes at base + 16 i);
//   - the instruction computes D[i][j] with operand 0 supplying i.  B fragments are operand 0,
//     so every lane ends up with 4 consecutive N outputs of one row of C; the epilogue turns
//     32 x 128 blocks around through LDS and stores whole 128-byte lines;
//   - workgroup ids are spread round-robin over the 8 XCDs by the hardware; the id -> tile map
//     gives every XCD one contiguous run of a column-sweeping order in bands of 8 tile rows,
//     so the 32 tiles an XCD works on at a time share 8 row slabs of A and 4 column slabs of
//     B in its L2;
//   - the products are formed either by the FP8 instruction above (ACC_FP8) or, after an exact
//     widening of the bytes to fp16 in registers, by v_mfma_f32_32x32x16_f16 (ACC_F16, the
//     default): see the note at the ACC_* constants for why both exist.
//
// This file is compiled once per (storage orders, accumulation mode): -DFP8MM_LAYOUT, -DFP8MM_ACC.
#include "gemm_common.hpp"

#include <atomic>
#include <type_traits>

namespace fp8mm {
namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v2f __attribute__((ext_vector_type(2)));
typedef __bf16 v2bf __attribute__((ext_vector_type(2)));

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))

// ------------------------------------------------------------------------------------------
// Fast kernel
// ------------------------------------------------------------------------------------------
constexpr int BM = 256, BK = 64;
// The tile is 256 rows of op(A) by 64 NB columns of op(B), NB = 4 or 2 (template parameter): two
// waves side by side along N, each NB blocks of 32 columns wide.  The narrow tile is for problems
// whose 256 x 256 tiles would leave much of the last round of workgroups empty.
// An operand tile of EXT rows / columns (256, or 128 for the narrow B) is staged in one of two ways,
// depending on how the operand lies in memory:
//   K-contiguous  (A row-major M x K; B given as N x K): one EXT x 128 slab per PAIR of stages,
//                 fragments by 16-byte LDS reads;
//   MN-contiguous (B row-major K x N; A given as K x M): one 64 x EXT slab per stage, ring of
//                 four, fragments by the transposing 8-byte LDS read.
constexpr int MC_SLOTS = 4;
constexpr int FAST_LDS = 160 * 1024;         // all of the LDS of a compute unit
constexpr int FAST_THREADS = 256;
constexpr int GROUP_M = 8;                   // tile rows per band of the tile order
constexpr int NUM_XCD = 8;

// Chunk swizzles.  K-contiguous slab: rows of 128 B = 8 chunks; MN-contiguous slab: rows of
// EXT bytes = 16 or 8 chunks (the swizzle value is reduced to the chunk count).  Measured on gfx950: with these a 16-byte fragment read costs 5 clocks per
// wave instruction (the conflict-free rate, 64 banks of 4 bytes) and a transposing 8-byte read
// 7.3 clocks.
__device__ __forceinline__ int swz_kc(int row) { return (row >> 1) & 7; }
// MN-contiguous slab: mc_pos = position in its K-row of the chunk whose index in memory is c; mc_mem
// = the memory chunk that sits at position p (the inverse map, used on the global side of the direct
// loads, whose LDS placement is fixed).  The XOR with the K-row spreads the 8 K-rows that one 16-lane
// group of a transposing read touches over 8 chunk positions.  In a 256-byte row (16 chunks, all 64
// banks) the odd memory chunks also change halves: the two 16-lane groups that are served
// together read neighbouring chunks (columns 0-15 and 16-31 of a block), which then lie in
// different halves of the banks instead of sharing 32 of them.
template <int CH>
__device__ __forceinline__ int mc_pos(int c, int krow)
{
    const int p = c ^ (krow & 7 & (CH - 1));
    return CH == 16 ? p ^ ((c & 1) << 3) : p;
}
template <int CH>
__device__ __forceinline__ int mc_mem(int p, int krow)
{
    const int c = p ^ (krow & 7 & (CH - 1));               // right but for bit 3, which does not enter bit 0
    return CH == 16 ? c ^ ((c & 1) << 3) : c;
}

// s_waitcnt with only the vector-memory counter constrained (gfx9 encoding:
// vmcnt = bits 3:0 and 15:14, expcnt = 6:4, lgkmcnt = 11:8).
template <int VM>
__device__ __forceinline__ void wait_vmcnt()
{
    __builtin_amdgcn_s_waitcnt((VM & 15) | ((VM >> 4) << 14) | (7 << 4) | (15 << 8));
}

struct TileMap { int tm, tn; };

// Workgroup id -> output tile.  Ids go round-robin over the XCDs; XCD x gets ids x, x+8, ...
// which are mapped to one contiguous run [start(x), start(x) + count(x)) of the order below.
// Order: bands of GROUP_M tile rows; inside a band go down the rows first, then to the next
// tile column.
__device__ __forceinline__ TileMap map_tile(int bid, int tiles_m, int tiles_n, int group_m)
{
    const int total = tiles_m * tiles_n;
    const int x = bid % NUM_XCD, idx = bid / NUM_XCD;
    const int base = total / NUM_XCD, rem = total % NUM_XCD;
    const int p = x * base + (x < rem ? x : rem) + idx;
    const int band_tiles = group_m * tiles_n;
    const int band = p / band_tiles;
    const int q = p - band * band_tiles;
    const int rows = min(group_m, tiles_m - band * group_m);
    TileMap t;
    t.tm = band * group_m + q % rows;
    t.tn = q / rows;
    return t;
}

// One operand of the tile as the kernel sees it.  r = row of A / column of B inside the EXT-wide
// tile, k = position along K:
//   KC: element (r, k) at tile + r * ld + k;   MC: element (r, k) at tile + k * ld + r.
struct Operand {
    const uint8_t* tile;     // first byte of the tile's rows (KC) or columns (MC)
    unsigned ld;             // leading dimension in bytes
    unsigned off[8];         // per-lane offsets of this wave's direct loads (EXT/32 used by KC, EXT/64 by MC)
    unsigned region;         // LDS byte offset of the operand's ring
    unsigned rd;             // per-lane LDS offset of its first fragment read (region included)
    // persistent form: where the next slab to be loaded starts (the loads run ahead of the products,
    // into the next tile), how many slabs of its tile have been loaded, and the byte offset from
    // `tile` of the rows / columns of the tile after the one that is being loaded
    const uint8_t* ldp;
    int ld_rel;
    size_t nxt;
};

template <bool KC, int EXT>
__device__ __forceinline__ void operand_setup(Operand& op, const uint8_t* base, unsigned ld, int r0, int valid,
                                              unsigned region, int w, int l, int wsel)
{
    // `valid` (1..EXT) rows / columns of the tile exist; loads of the others are redirected to an
    // existing one (their products only reach outputs that are never stored).
    op.ld = ld;
    op.region = region;
    const int h = l >> 5;
#pragma unroll
    for (int t = 0; t < 8; ++t) op.off[t] = 0;
    if (KC) {
        constexpr int LW = EXT / 32;                  // loads per wave per slab; each fills 8 rows (1 KB)
        op.tile = base + (size_t)r0 * ld;
#pragma unroll
        for (int t = 0; t < LW; ++t) {
            const int row = (w * LW + t) * 8 + (l >> 3);
            op.off[t] = (unsigned)min(row, valid - 1) * ld + (((l & 7) ^ swz_kc(row)) * 16);
        }
        // lane = (r = l % 32, h = l / 32) reads K bytes 32h .. 32h+31 of row r of its stage:
        // chunks 4 par + 2h and + 1 of the 128-byte row (par = stage parity)
        const int row = wsel * (EXT / 2) + (l & 31);
        op.rd = region + row * 128 + (((2 * h) ^ swz_kc(row)) * 16);
    } else {
        constexpr int CH = EXT / 16;                  // 16-byte chunks per K-row
        constexpr int KR = 1024 / EXT;                // K-rows filled by one load instruction (1 KB)
        constexpr int LW = 64 / KR / 4;               // loads per wave per slab
        op.tile = base + r0;
#pragma unroll
        for (int t = 0; t < LW; ++t) {
            const int krow = (w * LW + t) * KR + l / CH;
            const int chunk = mc_mem<CH>(l % CH, krow);                // 16 columns; `valid` is a multiple of 16 here
            op.off[t] = (unsigned)krow * ld + min(chunk, (valid - 1) >> 4) * 16;
        }
        // lane = (r = l % 32, h): column r, K bytes 32h .. 32h+31, gathered by four transposing
        // reads of 8 K-rows x 16 columns per 16-lane group; lanes 2q and 2q+1 address K-row q
        const int t16 = l & 15, gq = (l >> 4) & 1;
        const int krow = 32 * h + (t16 >> 1);
        op.rd = region + krow * EXT + mc_pos<CH>(wsel * (CH / 2) + gq, krow) * 16 + (t16 & 1) * 8;
    }
}

// Direct loads are written as inline assembly: the compiler then keeps no account of them and
// inserts no waits of its own; completion is tracked by explicit vmcnt waits.  LDS placement:
// M0 holds the wave-uniform base, lane i writes 16 bytes at M0 + 16 i.  M0 is an input operand of
// the statement (physical-register constraint): the compiler loads it and knows it is in use.  The
// s_nop is the wait state the hardware wants between a scalar write of M0 and its use here.
__device__ __forceinline__ void direct_load(const uint8_t* base, unsigned off, unsigned lds_addr)
{
    asm volatile("s_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(off), "s"(base), "{m0}"(lds_addr) : "memory");
}

// Sixteen zero bytes in device memory, never written: where K is not a multiple of 128 the chunks of
// the last stage pair that lie beyond K are fetched from here, so that every lane of every direct
// load still issues (the wait counts stay those of the schedule) and the products of the padding
// are 0 x 0.
__device__ __attribute__((aligned(16))) uint8_t g_zero_chunk[16];

// The same load with a full address per lane: the lane's chunk if it lies inside K, else the zeros.
__device__ __forceinline__ void direct_load_or_zero(const uint8_t* base, unsigned off, bool valid, unsigned lds_addr)
{
    const uint8_t* p = valid ? base + off : g_zero_chunk;
    asm volatile("s_nop 0\n\tglobal_load_lds_dwordx4 %0, off" :: "v"(p), "{m0}"(lds_addr) : "memory");
}

// One read-part of the fragment reads of stage kt for one operand: 16 bytes per lane of block blk
// (half 0 or 1 of the lane's 32 bytes), as one 16-byte read (KC) or two transposing reads (MC).
template <bool KC, int EXT>
__device__ __forceinline__ void read_part(const uint8_t* smem, const Operand& op, int kt, int kc_slot, int blk, int half,
                                          v8i* f)
{
    if (KC) {
        const unsigned addr = (op.rd ^ (unsigned)((kt & 1) * 64 + half * 16)) + kc_slot * (EXT * 128) + blk * 32 * 128;
        const v4i a = *LDS_PTR(v4i, smem + addr);
        f[blk][4 * half + 0] = a.x; f[blk][4 * half + 1] = a.y; f[blk][4 * half + 2] = a.z; f[blk][4 * half + 3] = a.w;
    } else {
        const unsigned base = (unsigned)(kt & (MC_SLOTS - 1)) * (64 * EXT) + (op.rd ^ (unsigned)(blk * 32));
#pragma unroll
        for (int s = 2 * half; s < 2 * half + 2; ++s) {
            const v2i p = __builtin_amdgcn_ds_read_tr8_b64_v2i32(LDS_PTR(v2i, smem + base + s * 8 * EXT));
            f[blk][2 * s] = p.x; f[blk][2 * s + 1] = p.y;
        }
    }
}

// The epilogue of one wave: its 128 x 32 NB sub-tile of accumulators -> memory.
//   c = acc * ra(row) [* cb(column)]: the reciprocal scales, applied once per output;
//   amax of |c| (if asked for); conversion to the output kind; whole-line stores.
// A lane holds 4 consecutive N of one C row per accumulator quad; written straight out that would
// be small pieces scattered over 32 rows per instruction.  Instead the wave turns each 32 x 32 NB
// block around through its own piece of the (now idle) LDS and stores it with 16 bytes per lane
// along N: whole 128-byte lines (64-byte halves for FP8 outputs of the narrow tile).  Every output kind is
// converted before the turn (FP8: multiplied by the output scale and rounded four at a time by the
// routine of the cast kernels), so the turn moves 4, 2 or 1 bytes per output.
template <int OUT, bool BVEC, int NB>
__device__ __forceinline__ void epilogue(v16f (&acc)[NB][4], uint8_t* smem, const EpilogueArgs& ep, void* C, int M, int N,
                                         int wave_m0, int wave_n0, int w, int l)
{
    constexpr bool FP8OUT = OUT == OUT_E4M3 || OUT == OUT_E5M2;
    constexpr int ESZ = OUT == OUT_F32 ? 4 : OUT == OUT_BF16 ? 2 : 1;     // bytes per output in memory
    constexpr int LSZ = ESZ;                                              // bytes per output in LDS
    constexpr int WN = 32 * NB;                                           // columns of the wave's sub-tile
    constexpr int ROWB = WN * LSZ + 16;                                   // padded LDS row of the wave's block
    constexpr int ROWS_PER_ST = 1024 / (WN * ESZ);                        // C rows covered by one store instruction
    const int h = l >> 5;

    // reciprocal scales: per row in ra (with the per-tensor sB folded in), per column in cb
    // (the by-value factors are copied out of the argument block first: a choice between two
    // memory locations would force the block into scratch memory)
    const float sA_host = ep.sA, sB_host = ep.sB;
    float ra[4];
    {
        const double b = BVEC ? 1.0 : (double)scale_value(ep.sB_dev, sB_host);
#pragma unroll
        for (int mb = 0; mb < 4; ++mb) {
            const float a = ep.a_per_row ? ep.sA_dev[min(wave_m0 + mb * 32 + (l & 31), M - 1)] : scale_value(ep.sA_dev, sA_host);
            ra[mb] = (float)(1.0 / ((double)a * b));
        }
    }
    v4f cb[BVEC ? NB : 1][BVEC ? 4 : 1];
    if (BVEC) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int col = wave_n0 + nb * 32 + 8 * q + 4 * h;
                v4f s;
                if (ep.ragged_n) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) s[i] = ep.sB_dev[min(col + i, N - 1)];
                } else {
                    s = *(const v4f*)(ep.sB_dev + min(col, N - 4));
                }
                cb[BVEC ? nb : 0][BVEC ? q : 0] = (v4f){1.0f / s.x, 1.0f / s.y, 1.0f / s.z, 1.0f / s.w};
            }
    }
    const float sD = FP8OUT ? scale_value(ep.sD_dev, 1.0f) : 1.0f;
    unsigned amax_bits = 0;

    uint8_t* blk = smem + w * (32 * ROWB);
    uint8_t* c_wave = (uint8_t*)C + ((size_t)wave_m0 * N + wave_n0) * ESZ;
    const int st_row = l / (64 / ROWS_PER_ST), st_col = (l % (64 / ROWS_PER_ST)) * 16;   // byte column in memory
#pragma unroll
    for (int mb = 0; mb < 4; ++mb) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float c0 = acc[nb][mb][4 * q + 0] * ra[mb], c1 = acc[nb][mb][4 * q + 1] * ra[mb];
                float c2 = acc[nb][mb][4 * q + 2] * ra[mb], c3 = acc[nb][mb][4 * q + 3] * ra[mb];
                if (BVEC) {
                    const v4f s = cb[BVEC ? nb : 0][BVEC ? q : 0];
                    c0 *= s.x; c1 *= s.y; c2 *= s.z; c3 *= s.w;
                }
                if (ep.amax_out) {
                    // outputs beyond the edges of C hold products of redirected loads: not counted
                    // (unless N is ragged, the four columns are inside or outside together)
                    const int col = wave_n0 + nb * 32 + 8 * q + 4 * h;
                    const bool row_in = wave_m0 + mb * 32 + (l & 31) < M;
                    const unsigned k0 = row_in && col < N ? 0x7fffffffu : 0u, k1 = row_in && col + 1 < N ? 0x7fffffffu : 0u;
                    const unsigned k2 = row_in && col + 2 < N ? 0x7fffffffu : 0u, k3 = row_in && col + 3 < N ? 0x7fffffffu : 0u;
                    const unsigned m01 = max(as_u32(c0) & k0, as_u32(c1) & k1);
                    const unsigned m23 = max(as_u32(c2) & k2, as_u32(c3) & k3);
                    amax_bits = max(amax_bits, max(m01, m23));
                }
                uint8_t* dst = blk + (l & 31) * ROWB + (nb * 32 + 8 * q + 4 * h) * LSZ;
                if (OUT == OUT_F32) {
                    *LDS_PTR(v4f, dst) = (v4f){c0, c1, c2, c3};
                } else if (OUT == OUT_BF16) {
                    v2i o;
                    o.x = (int)__builtin_bit_cast(unsigned, __builtin_convertvector((v2f){c0, c1}, v2bf));
                    o.y = (int)__builtin_bit_cast(unsigned, __builtin_convertvector((v2f){c2, c3}, v2bf));
                    *LDS_PTR(v2i, dst) = o;
                } else {
                    *LDS_PTR(unsigned, dst) = encode4<OUT == OUT_E4M3 ? FP8_E4M3 : FP8_E5M2>(c0 * sD, c1 * sD, c2 * sD, c3 * sD);
                }
            }
#pragma unroll
        for (int i = 0; i < 32 / ROWS_PER_ST; ++i) {
            const int row = i * ROWS_PER_ST + st_row;
            uint8_t* out = c_wave + (size_t)(mb * 32 + row) * N * ESZ + st_col;
            if (wave_m0 + mb * 32 + row >= M || wave_n0 + st_col / ESZ >= N) continue;   // beyond the edges of C
            const u32x4 o = *LDS_PTR(u32x4, blk + row * ROWB + st_col);
            if (!ep.ragged_n) {
                *(u32x4*)out = o;                        // (non-temporal stores measured the same, 8 shapes)
            } else {                                    // rows of C start anywhere: element by element
                const int left = N - (wave_n0 + st_col / ESZ);          // columns from the lane's first one to the edge
#pragma unroll
                for (int e = 0; e < 16 / ESZ; ++e) {
                    if (e < left) {
                        if (ESZ == 4) ((unsigned*)out)[e] = o[e];
                        else if (ESZ == 2) ((unsigned short*)out)[e] = (unsigned short)(o[e >> 1] >> (16 * (e & 1)));
                        else out[e] = (uint8_t)(o[e >> 2] >> (8 * (e & 3)));
                    }
                }
            }
        }
    }
    if (ep.amax_out) wave_amax_commit(amax_bits, ep.amax_out);
}

// A_KC / B_KC: how the operand lies in memory (see Operand); NB: width of the tile in blocks of 32
// columns per wave.  LDS: an MN-contiguous operand takes a ring of four stage slabs; a K-contiguous
// one a ring of three stage-pair slabs, or of two for B when both operands are K-contiguous.
//
// PERSIST: the persistent form for problems of several rounds of small tiles.  The grid is one
// workgroup per compute unit; a workgroup takes the tiles blockIdx.x, blockIdx.x + gridDim.x, ... and
// walks them as ONE long K loop: the stages of the next tile follow the last stage of the current
// one in the ring, so the direct loads of a tile's first stages are issued (and its first
// fragments read) while the previous tile is still being multiplied, and a tile ends with nothing
// but its stores.  Since all of the LDS then holds operands of the next tile, the outputs leave
// straight from the registers (8 or 16 bytes per lane, 32 rows per instruction) instead of being
// turned around through LDS: more, smaller writes, which do not matter where the output is small.
// The stores are vector-memory instructions like the direct loads and complete in order with
// them: the waits of the three steps after a tile end leave room for them.  Conditions (checked by
// the dispatcher): no edge tiles, K a multiple of 128 and at least 512, per-tensor factors, fp32 or
// bf16 output with rows on 16-byte boundaries, no output maximum, no K slices.
//
// The body works on tile number `bid_in` of a region of the output that starts at column n_begin and
// is tiles_n tiles wide (the whole output for the plain kernel; see gemm_mixed_kernel).
template <int FMT_A, int FMT_B, int ACC, bool A_KC, bool B_KC, int NB, bool PERSIST>
__device__ __forceinline__ void gemm_tile_body(
    const uint8_t* __restrict__ A, const uint8_t* __restrict__ B, void* __restrict__ C,
    int M, int N, int K, const EpilogueArgs& ep, int group_m, int splits, int pairs_per_split,
    int bid_in, int n_begin, int tiles_n)
{
    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
    constexpr int BN = 64 * NB;                             // tile width
    constexpr int P = 2 * NB;                               // parts a stage is cut into
    constexpr int A_RING = 3;                               // stage pairs in A's ring (if A_KC)
    constexpr int B_RING = A_KC ? 2 : 3;                    // stage pairs in B's ring (if B_KC)
    constexpr bool HAS_MC = !A_KC || !B_KC;
    // direct loads per wave: per pair slab (K-contiguous) / per stage slab (MN-contiguous)
    constexpr int A_KC_LOADS = 8, A_MC_LOADS = 4, B_KC_LOADS = 2 * NB, B_MC_LOADS = NB;
    // LDS map: the operand with the smaller ring (MN-contiguous, or B when both are K-contiguous) first.
    constexpr unsigned A_REGION = A_KC ? 65536u : 0u;
    constexpr unsigned B_REGION = A_KC ? 0u : 65536u;

    const int tid = threadIdx.x;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6), l = tid & 63;
    const int wm = w >> 1, wn = w & 1;
    // K is walked in pairs of stages (128 bytes); a last pair that reaches beyond K is filled up
    // with zeros.  With splits > 1 the workgroup computes one slice of K (pairs_per_split pairs,
    // the last slice what is left) of its tile and writes the fp32 sums, without the scales, into
    // slice `split` of C, which is then a workspace of `splits` M x N matrices.
    int bid = bid_in, split = 0;
    if (!PERSIST && splits > 1) { split = bid % splits; bid /= splits; }
    const int tiles_m = (M + BM - 1) / BM;
    const TileMap tile = map_tile(bid, tiles_m, tiles_n, group_m);
    int m0 = tile.tm * BM, n0 = n_begin + tile.tn * BN;     // the tile whose products are being accumulated
    const int pair0 = split * pairs_per_split;
    const int KT_TILE = 2 * min(pairs_per_split, (K + 2 * BK - 1) / (2 * BK) - pair0);     // stages of one tile
    // PERSIST: `units` tiles in a row; every stage and pair index below is then a global one
    const int units = PERSIST ? (tiles_m * tiles_n - bid + (int)gridDim.x - 1) / (int)gridDim.x : 1;
    const int KT = units * KT_TILE;
    const int kend = K - pair0 * 2 * BK;                    // bytes of K from the start of the slice to the end of K
    const bool ktail = !PERSIST && kend < KT * BK;          // the slice ends in a partly filled pair
    const unsigned lds0 = (unsigned)(uintptr_t)LDS_PTR(void, smem);
    C = (uint8_t*)C + (size_t)split * (size_t)M * (size_t)N * 4;

    Operand opA, opB;
    operand_setup<A_KC, BM>(opA, A + (size_t)pair0 * 2 * BK * (A_KC ? 1 : (size_t)M), A_KC ? (unsigned)K : (unsigned)M,
                            PERSIST ? 0 : m0, PERSIST ? BM : min(BM, M - m0), A_REGION, w, l, wm);
    operand_setup<B_KC, BN>(opB, B + (size_t)pair0 * 2 * BK * (B_KC ? 1 : (size_t)N), B_KC ? (unsigned)K : (unsigned)N,
                            PERSIST ? 0 : n0, PERSIST ? BN : min(BN, N - n0), B_REGION, w, l, wn);
    // persistent form: where the rows / columns of a tile start, relative to the operand's first byte
    auto a_start = [&](int tm0) { return A_KC ? (size_t)tm0 * (size_t)K : (size_t)tm0; };
    auto b_start = [&](int tn0) { return B_KC ? (size_t)tn0 * (size_t)K : (size_t)tn0; };
    int unit = 0;                                           // index of the current tile in this workgroup's list
    int nm0 = m0, nn0 = n0;                                 // the tile after the current one
    if (PERSIST && units > 1) {
        const TileMap t2 = map_tile(bid + (int)gridDim.x, tiles_m, tiles_n, group_m);
        nm0 = t2.tm * BM; nn0 = t2.tn * BN;
    }
    opA.ldp = opA.tile + (PERSIST ? a_start(m0) : 0); opA.ld_rel = 0; opA.nxt = PERSIST ? a_start(nm0) : 0;
    opB.ldp = opB.tile + (PERSIST ? b_start(n0) : 0); opB.ld_rel = 0; opB.nxt = PERSIST ? b_start(nn0) : 0;

    // ---- the schedule of direct loads, as a function of the step index s (the prologue plays
    // the steps -5 .. -1).  Step s issues, in this order:
    //   for a K-contiguous operand, if s is odd: the slab of stage pair (s+1)/2 + ring - 1 into
    //                the slot that stage s frees, spread over the first half of the parts;
    //   for an MN-contiguous operand the slab of stage s + 4, spread over the second half.
    // (Splitting the pair slab over the odd and the even step, for the same number of loads in
    // every step, measured 2 % slower in the FP8 mode.)
    // If both operands are K-contiguous, B's ring holds two pairs only and its loads have less
    // than two steps to arrive; they must not queue behind A's.  Then the odd steps issue B alone
    // and the even step s issues A's pair s/2 + 2, spread over all parts, into the slot of the pair
    // that ended a step ago (three steps of lead are left).
    auto kc_pair_of = [](int s, int ring) { return (s + 1) / 2 + ring - 1; };     // s odd (may be negative)
    auto pair_valid = [&](int p) { return p >= 0 && 2 * p < KT; };
    auto stage_valid = [&](int st) { return st >= 0 && st < KT; };
    auto count_step = [&](int s) {
        int n = 0;
        if (A_KC && B_KC)
            return (s & 1) ? (pair_valid(kc_pair_of(s, B_RING)) ? B_KC_LOADS : 0) : (pair_valid(s / 2 + A_RING - 1) ? A_KC_LOADS : 0);
        if (A_KC && (s & 1) && pair_valid(kc_pair_of(s, A_RING))) n += A_KC_LOADS;
        if (B_KC && (s & 1) && pair_valid(kc_pair_of(s, B_RING))) n += B_KC_LOADS;
        if (!A_KC && stage_valid(s + 4)) n += A_MC_LOADS;
        if (!B_KC && stage_valid(s + 4)) n += B_MC_LOADS;
        return n;
    };
    // Loads complete in order.  Stage t is complete once the last load issued for it is: that is
    // the last load of step t - 4 if an operand is MN-contiguous, else of the step that issued
    // B's pair t/2.  `upto` = last step whose loads have been issued when the wait is placed.
    // When a step waits for the stage after its own and every step of the window issues its full
    // set, the count depends on the parity of the step alone and is a compile-time constant: with
    // an MN-contiguous operand the window is one odd and one even step; with two K-contiguous
    // operands it is A's even step and B's odd step before an even step, A's even step before an odd one.
    constexpr int STEADY_EVEN = HAS_MC ? (A_KC ? A_KC_LOADS : 2 * A_MC_LOADS) + (B_KC ? B_KC_LOADS : 2 * B_MC_LOADS)
                                       : A_KC_LOADS + B_KC_LOADS;
    constexpr int STEADY_ODD = HAS_MC ? STEADY_EVEN : A_KC_LOADS;
    // extra: younger instructions that are not direct loads (the stores of a tile end, persistent form)
    auto wait_stage = [&](int t, int upto, int extra = 0) {
        const int s_need = HAS_MC ? t - 4 : 2 * (t / 2) - 2 * B_RING + 1;
        int allowed = extra;
        for (int s = s_need + 1; s <= upto; ++s) allowed += count_step(s);
        switch (allowed >> 1) {                   // every count is even
            case 0: wait_vmcnt<0>(); break;   case 1: wait_vmcnt<2>(); break;   case 2: wait_vmcnt<4>(); break;
            case 3: wait_vmcnt<6>(); break;   case 4: wait_vmcnt<8>(); break;   case 5: wait_vmcnt<10>(); break;
            case 6: wait_vmcnt<12>(); break;  case 7: wait_vmcnt<14>(); break;  case 8: wait_vmcnt<16>(); break;
            case 9: wait_vmcnt<18>(); break;  case 10: wait_vmcnt<20>(); break; case 11: wait_vmcnt<22>(); break;
            case 12: wait_vmcnt<24>(); break; case 13: wait_vmcnt<26>(); break; case 14: wait_vmcnt<28>(); break;
            case 15: wait_vmcnt<30>(); break; case 16: wait_vmcnt<32>(); break; case 17: wait_vmcnt<34>(); break;
            case 18: wait_vmcnt<36>(); break; case 19: wait_vmcnt<38>(); break; case 20: wait_vmcnt<40>(); break;
            case 21: wait_vmcnt<42>(); break; case 22: wait_vmcnt<44>(); break; case 23: wait_vmcnt<46>(); break;
            case 24: wait_vmcnt<48>(); break; case 25: wait_vmcnt<50>(); break; case 26: wait_vmcnt<52>(); break;
            case 27: wait_vmcnt<54>(); break; case 28: wait_vmcnt<56>(); break; case 29: wait_vmcnt<58>(); break;
            case 30: wait_vmcnt<60>(); break;
            default: if (allowed > 60) wait_vmcnt<62>(); else wait_vmcnt<0>(); break;   // the counter holds 63 at most
        }
    };
    // load t of this wave for a pair slab (loads-per-wave lw: the slab takes 4 lw KB) / a stage slab
    // TAIL (compile-time, never in the steady-state steps): the slice may end in a partly filled
    // pair; then the lane's chunk is tested against the end of K (see direct_load_or_zero).
    auto issue_kc = [&](auto tail_tag, const Operand& op, int lw, int pair, int slot, int t) {
        const unsigned lds = lds0 + op.region + slot * (lw * 4096) + w * (lw * 1024) + t * 1024;
        if (PERSIST) {
            direct_load(op.ldp, op.off[t], lds);             // the running pointer (see advance_loads)
        } else if (decltype(tail_tag)::value && ktail) {
            // row of the slab = (w lw + t) 8 + l / 8, chunk = (l % 8) ^ swz_kc(row)
            const int chunk = (l & 7) ^ (((w * lw + t) * 4 + (l >> 4)) & 7);
            direct_load_or_zero(op.tile + (size_t)pair * 2 * BK, op.off[t], pair * 2 * BK + chunk * 16 < kend, lds);
        } else {
            direct_load(op.tile + (size_t)pair * 2 * BK, op.off[t], lds);
        }
    };
    auto issue_mc = [&](auto tail_tag, const Operand& op, int lw, int st, int t) {
        const unsigned lds = lds0 + op.region + (st & (MC_SLOTS - 1)) * (lw * 4096) + w * (lw * 1024) + t * 1024;
        if (PERSIST) {
            direct_load(op.ldp, op.off[t], lds);
        } else if (decltype(tail_tag)::value && ktail) {
            // K-row of the slab = (w lw + t) KR + l / CH with KR = 16 / lw rows per load, CH = 4 lw chunks per row
            const int krow = (w * lw + t) * (16 / lw) + l / (4 * lw);
            direct_load_or_zero(op.tile + (size_t)st * BK * op.ld, op.off[t], st * BK + krow < kend, lds);
        } else {
            direct_load(op.tile + (size_t)st * BK * op.ld, op.off[t], lds);
        }
    };
    // the loads of step s that fall into part j; sa, sb = ring slots the K-contiguous slabs of
    // this step go to (the slots of the pair that stage s ends; for A in an even step when both
    // operands are K-contiguous: of the pair before the one stage s begins)
    // FULL (compile-time): the caller guarantees that every load of the step exists, and no test is
    // made.  The tests are branches, and a branch ends the region within which the compiler may
    // move the conversions of one part under the MFMAs of the part before.
    auto issue_part = [&](auto full_tag, int s, bool odd, int j, int sa, int sb) {
        constexpr bool FULL = decltype(full_tag)::value;
        constexpr int H = P / 2;
        const std::integral_constant<bool, !FULL> tail;
        if (A_KC && B_KC) {
            if (odd) {
                const int p = kc_pair_of(s, B_RING);
                if (j < H && (FULL || pair_valid(p))) {
#pragma unroll
                    for (int t = j * (B_KC_LOADS / H); t < (j + 1) * (B_KC_LOADS / H); ++t) issue_kc(tail, opB, B_KC_LOADS, p, sb, t);
                }
            } else {
                const int p = s / 2 + A_RING - 1;
                if (FULL || pair_valid(p)) {
#pragma unroll
                    for (int t = j * (A_KC_LOADS / P); t < (j + 1) * (A_KC_LOADS / P); ++t) issue_kc(tail, opA, A_KC_LOADS, p, sa, t);
                }
            }
        } else if (j < H) {
            if (odd) {
                if (A_KC) {
                    const int p = kc_pair_of(s, A_RING);
                    if (FULL || pair_valid(p)) {
#pragma unroll
                        for (int t = j * (A_KC_LOADS / H); t < (j + 1) * (A_KC_LOADS / H); ++t) issue_kc(tail, opA, A_KC_LOADS, p, sa, t);
                    }
                }
                if (B_KC) {
                    const int p = kc_pair_of(s, B_RING);
                    if (FULL || pair_valid(p)) {
#pragma unroll
                        for (int t = j * (B_KC_LOADS / H); t < (j + 1) * (B_KC_LOADS / H); ++t) issue_kc(tail, opB, B_KC_LOADS, p, sb, t);
                    }
                }
            }
        } else if (FULL || stage_valid(s + 4)) {
            const int jj = j - H;
            if (!A_KC) {
#pragma unroll
                for (int t = jj * (A_MC_LOADS / H); t < (jj + 1) * (A_MC_LOADS / H); ++t) issue_mc(tail, opA, A_MC_LOADS, s + 4, t);
            }
            if (!B_KC) {
#pragma unroll
                for (int t = jj * (B_MC_LOADS / H); t < (jj + 1) * (B_MC_LOADS / H); ++t) issue_mc(tail, opB, B_MC_LOADS, s + 4, t);
            }
        }
    };

    // Persistent form: after the loads of step s have been issued, the running pointers of the operands
    // that loaded a slab in it move on by one slab (a pair of stages = 128 bytes along K for a
    // K-contiguous operand, a stage = 64 K-rows for the other kind); after the last slab of a tile
    // they jump to the first slab of the next tile.  The conditions are those of issue_part.
    auto advance = [&](Operand& op, size_t inc, int slabs_per_tile) {
        op.ldp += inc;
        if (++op.ld_rel == slabs_per_tile) { op.ld_rel = 0; op.ldp = op.tile + op.nxt; }
    };
    auto advance_loads = [&](auto full_tag, int s, bool odd) {
        constexpr bool FULL = decltype(full_tag)::value;    // every load of the step exists: no tests
        if (A_KC) {
            if (B_KC ? !odd : odd) {
                const int p = B_KC ? s / 2 + A_RING - 1 : kc_pair_of(s, A_RING);
                if (FULL || pair_valid(p)) advance(opA, 2 * BK, KT_TILE / 2);
            }
        } else if (FULL || stage_valid(s + 4)) {
            advance(opA, (size_t)BK * opA.ld, KT_TILE);
        }
        if (B_KC) {
            if (odd && (FULL || pair_valid(kc_pair_of(s, B_RING)))) advance(opB, 2 * BK, KT_TILE / 2);
        } else if (FULL || stage_valid(s + 4)) {
            advance(opB, (size_t)BK * opB.ld, KT_TILE);
        }
    };

    v16f acc[NB][4];
#pragma unroll
    for (int i = 0; i < NB; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    // The block products of a stage, in P parts.
    //   ACC_FP8: one v_mfma_f32_32x32x64_f8f6f4 per block (K = 64); part j = B block j/2 against
    //            the A blocks 2(j%2) and 2(j%2)+1.
    //   ACC_F16: the FP8 bytes are widened exactly to fp16 in registers and each block takes four
    //            v_mfma_f32_32x32x16_f16 (K = 16, 8 of the lane's 32 bytes each); a part is two B
    //            blocks of one K sub-step against the four A blocks.  The operands of a part are
    //            converted during the part before it (for part 0: during the last part of the
    //            stage before, from that stage's freshly read fragments): the conversions are then
    //            independent of the MFMAs they are issued between and run in their shadow.  A
    //            conversion costs 8 cycles of the vector ALU (measured), an MFMA 32 of the matrix
    //            pipe: 24 conversions fit under the 8 MFMAs of a part, but only if none of those
    //            MFMAs waits for one of them.
    constexpr int PPS = NB / 2;                   // parts per K sub-step (ACC_F16)
    v8h a16[2][4], b16[2][2];                     // [sub-step parity][A block], [part parity][B block of the part]
    auto compute_fp8 = [&](int j, v8i (&af)[4], v8i (&bf)[NB]) {
        const int nb = j >> 1;
#pragma unroll
        for (int mb = 2 * (j & 1); mb < 2 * (j & 1) + 2; ++mb)
            acc[nb][mb] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                bf[nb], af[mb], acc[nb][mb], FMT_B, FMT_A, 0, 0, 0, 0);
    };
    // operands of part j of a stage whose fragments are (af, bf)
    auto convert_f16 = [&](int j, v8i (&af)[4], v8i (&bf)[NB]) {
        const int s = j / PPS, nb0 = 2 * (j % PPS);
#pragma unroll
        for (int i = 0; i < 2; ++i) b16[j & 1][i] = widen8<FMT_B>(bf[nb0 + i][2 * s], bf[nb0 + i][2 * s + 1]);
        if (j % PPS == 0) {
#pragma unroll
            for (int mb = 0; mb < 4; ++mb) a16[s & 1][mb] = widen8<FMT_A>(af[mb][2 * s], af[mb][2 * s + 1]);
        }
    };
    auto compute_f16 = [&](int j) {
        const int s = j / PPS, nb0 = 2 * (j % PPS);
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int mb = 0; mb < 4; ++mb)
                acc[nb0 + i][mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(b16[j & 1][i], a16[s & 1][mb], acc[nb0 + i][mb], 0, 0, 0);
    };
    // fragment reads of the next stage that go out in one part: 8 / P read-parts of A, one of B;
    // the first halves of all blocks first (the first conversions of the next stage need them)
    constexpr int A_RP = 8 / P;
    constexpr int READS_PER_PART = A_RP * (A_KC ? 1 : 2) + (B_KC ? 1 : 2);
    auto sched_part = [&]() {
        if (ACC == ACC_FP8) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                        // MFMA
            __builtin_amdgcn_sched_group_barrier(0x100, (READS_PER_PART + 1) / 2, 0); // LDS reads
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, READS_PER_PART / 2, 0);
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                    // MFMA
                if (i < READS_PER_PART) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, 3, 0);                    // widening for the next part
            }
            __builtin_amdgcn_sched_barrier(0);        // nothing drifts into another part (register pressure)
        }
    };
    auto read_both = [&](int kt, int j, int sa, int sb, v8i (&af)[4], v8i (&bf)[NB]) {
#pragma unroll
        for (int r = 0; r < A_RP; ++r) {
            const int ra = j * A_RP + r;
            read_part<A_KC, BM>(smem, opA, kt, sa, ra & 3, ra >> 2, af);
        }
        read_part<B_KC, BN>(smem, opB, kt, sb, j % NB, j / NB, bf);
    };

    // One K stage kt (not the last).  The frags of stage kt are in (af, bf); their LDS reads were
    // issued a stage ago.  First stage kt+1 is made visible.  Then, in P parts, the direct loads of
    // step kt are issued (into the slots that stage kt, whose frags are in registers, has freed),
    // a share of the MFMAs of stage kt runs, and the fragment reads of stage kt+1 go out into
    // (af_n, bf_n).  Spreading matters: the four waves run in step, and a wave that issues its
    // loads in one burst waits for the address unit before it reaches its first MFMA.
    // (sa, sb) = ring slots of the pair of stage kt, (sa_n, sb_n) = of the pair of stage kt+1.
    // after_tag (compile-time; persistent form): the stores of a tile end were issued within the last
    // three steps, after the loads this step waits for
    constexpr int TILE_STORES = 16 * NB;          // store instructions per wave at a tile end
    auto k_step = [&](auto full_tag, int kt, bool odd, int sa, int sb, int sa_n, int sb_n, v8i (&af)[4], v8i (&bf)[NB],
                      v8i (&af_n)[4], v8i (&bf_n)[NB], auto after_tag) {
        constexpr bool FULL = decltype(full_tag)::value;
        constexpr bool after_stores = decltype(after_tag)::value;
        // slot that A's loads of this step go to
        const int sa_ld = (A_KC && B_KC && !odd) ? (sa == 0 ? A_RING - 1 : sa - 1) : sa;
        const int sb_ld = sb;
        if (FULL || kt + 8 < KT) {
            if (PERSIST && after_stores) {
                if (odd) wait_vmcnt<(STEADY_ODD + TILE_STORES < 62 ? STEADY_ODD + TILE_STORES : 62)>();
                else wait_vmcnt<(STEADY_EVEN + TILE_STORES < 62 ? STEADY_EVEN + TILE_STORES : 62)>();
            } else {
                if (odd) wait_vmcnt<STEADY_ODD>(); else wait_vmcnt<STEADY_EVEN>();
            }
        } else {
            wait_stage(kt + 1, kt - 1, PERSIST && after_stores ? TILE_STORES : 0);
        }
        __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0): this wave's LDS reads of stage kt are done
        __builtin_amdgcn_s_barrier();         // stage kt+1 is complete; nobody reads the slots of stage kt any more
#pragma unroll
        for (int j = 0; j < P; ++j) {
            issue_part(full_tag, kt, odd, j, sa_ld, sb_ld);
            read_both(kt + 1, j, sa_n, sb_n, af_n, bf_n);
            if (ACC == ACC_FP8) {
                compute_fp8(j, af, bf);
            } else {
                compute_f16(j);
                if (j + 1 < P) convert_f16(j + 1, af, bf); else convert_f16(0, af_n, bf_n);
            }
            sched_part();
        }
        if (PERSIST) advance_loads(full_tag, kt, odd);
    };

    // Prologue: steps -5 .. -1 of the same schedule, then stage 0 visible and its frags read.
    // KT is even and >= 2 (a stage beyond K holds zeros).
    v8i af0[4], bf0[NB], af1[4], bf1[NB];
    const std::integral_constant<bool, true> full;
    const std::integral_constant<bool, false> checked;
    for (int s = -5; s < 0; ++s) {
        // a pair issued by a step s < 0 has an index below the ring size: slot = pair
        const int sa = !A_KC ? 0 : (s & 1) ? (s + 1) / 2 + A_RING - 1 : s / 2 + A_RING - 1;
        const int sb = !B_KC ? 0 : (s & 1) ? (s + 1) / 2 + B_RING - 1 : s / 2 + B_RING - 1;
#pragma unroll
        for (int j = 0; j < P; ++j) issue_part(checked, s, s & 1, j, sa, sb);
        if (PERSIST) advance_loads(checked, s, s & 1);
    }
    wait_stage(0, -1);
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int j = 0; j < P; ++j) read_both(0, j, 0, 0, af0, bf0);
    if (ACC == ACC_F16) convert_f16(0, af0, bf0);
    int sa = 0, sb = 0;                       // ring slots of the current stage pair
    int kt = 0;

    // ---- persistent form: the end of a tile -----------------------------------------------------
    // c = acc / (sA sB) straight from the registers: a lane holds 4 consecutive N of one row of C per
    // accumulator quad; then the accumulators are cleared and the bookkeeping moves on to the next
    // tile (whose first stages are in the ring already and whose first fragments are in registers).
    const float ra_tile = PERSIST ? (float)(1.0 / ((double)scale_value(ep.sA_dev, ep.sA) * (double)scale_value(ep.sB_dev, ep.sB))) : 0.0f;
    int next_end = KT_TILE;                   // global index of the first stage of the next tile
    auto tile_end = [&](bool more) {
        const int le = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
        const size_t row = (size_t)(m0 + wm * 128 + (le & 31));
        const int col = n0 + wn * (32 * NB) + 4 * (le >> 5);
        if (ep.out_kind == OUT_BF16) {
            unsigned short* c0 = (unsigned short*)C + row * (size_t)N + col;
#pragma unroll
            for (int mb = 0; mb < 4; ++mb)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const v16f& a = acc[nb][mb];
                        v2i o;
                        o.x = (int)__builtin_bit_cast(unsigned, __builtin_convertvector((v2f){a[4 * q] * ra_tile, a[4 * q + 1] * ra_tile}, v2bf));
                        o.y = (int)__builtin_bit_cast(unsigned, __builtin_convertvector((v2f){a[4 * q + 2] * ra_tile, a[4 * q + 3] * ra_tile}, v2bf));
                        *(v2i*)(c0 + (size_t)(mb * 32) * N + nb * 32 + 8 * q) = o;
                    }
        } else {
            float* c0 = (float*)C + row * (size_t)N + col;
#pragma unroll
            for (int mb = 0; mb < 4; ++mb)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const v16f& a = acc[nb][mb];
                        *(v4f*)(c0 + (size_t)(mb * 32) * N + nb * 32 + 8 * q) =
                            (v4f){a[4 * q] * ra_tile, a[4 * q + 1] * ra_tile, a[4 * q + 2] * ra_tile, a[4 * q + 3] * ra_tile};
                    }
        }
        if (!more) return;
#pragma unroll
        for (int i = 0; i < NB; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
        ++unit;
        m0 = nm0; n0 = nn0;
        if (unit + 1 < units) {
            const TileMap t2 = map_tile(bid + (unit + 1) * (int)gridDim.x, tiles_m, tiles_n, group_m);
            nm0 = t2.tm * BM; nn0 = t2.tn * BN;
            opA.nxt = a_start(nm0); opB.nxt = b_start(nn0);
        }
        next_end += KT_TILE;
    };
    const std::integral_constant<bool, true> yes;
    const std::integral_constant<bool, false> no;

    // One round of the outer loop per tile (a single one unless PERSIST).  The tile end sits between
    // the inner loops, not inside them: inside, the accumulators would have to change register
    // class (the stores read them as vector registers, the matrix instructions keep them in the
    // accumulation registers) on every trip.
    for (;;) {
        const int tile_stop = next_end < KT ? next_end : KT - 2;     // the last pair of the last tile is peeled below
        // steps whose loads all exist (the last stage a step s touches is s + 6) and whose waits are
        // the steady ones: no tests inside
        for (; kt + 10 < KT && kt < tile_stop; kt += 2) {
            const int sa_n = A_KC ? (sa == A_RING - 1 ? 0 : sa + 1) : 0;
            const int sb_n = B_KC ? (sb == B_RING - 1 ? 0 : sb + 1) : 0;
            k_step(full, kt, false, sa, sb, sa, sb, af0, bf0, af1, bf1, no);
            k_step(full, kt + 1, true, sa, sb, sa_n, sb_n, af1, bf1, af0, bf0, no);
            sa = sa_n; sb = sb_n;
        }
        for (; kt < tile_stop; kt += 2) {
            const int sa_n = A_KC ? (sa == A_RING - 1 ? 0 : sa + 1) : 0;
            const int sb_n = B_KC ? (sb == B_RING - 1 ? 0 : sb + 1) : 0;
            k_step(checked, kt, false, sa, sb, sa, sb, af0, bf0, af1, bf1, no);
            k_step(checked, kt + 1, true, sa, sb, sa_n, sb_n, af1, bf1, af0, bf0, no);
            sa = sa_n; sb = sb_n;
        }
        if (!PERSIST || next_end >= KT) break;
        tile_end(true);
        // The first three steps of the next tile wait for loads that are older than these stores:
        // two pairs of steps (a tile has at least four) with the stores counted in, in the tested form.
        {
            const int sa_n = A_KC ? (sa == A_RING - 1 ? 0 : sa + 1) : 0;
            const int sb_n = B_KC ? (sb == B_RING - 1 ? 0 : sb + 1) : 0;
            k_step(checked, kt, false, sa, sb, sa, sb, af0, bf0, af1, bf1, yes);
            k_step(checked, kt + 1, true, sa, sb, sa_n, sb_n, af1, bf1, af0, bf0, yes);
            sa = sa_n; sb = sb_n; kt += 2;
        }
        {
            const int sa_n = A_KC ? (sa == A_RING - 1 ? 0 : sa + 1) : 0;
            const int sb_n = B_KC ? (sb == B_RING - 1 ? 0 : sb + 1) : 0;
            k_step(checked, kt, false, sa, sb, sa, sb, af0, bf0, af1, bf1, yes);
            k_step(checked, kt + 1, true, sa, sb, sa_n, sb_n, af1, bf1, af0, bf0, no);
            sa = sa_n; sb = sb_n; kt += 2;
        }
    }
    k_step(checked, KT - 2, false, sa, sb, sa, sb, af0, bf0, af1, bf1, no);
#pragma unroll
    for (int j = 0; j < P; ++j) {
        if (ACC == ACC_FP8) {
            compute_fp8(j, af1, bf1);
        } else {
            compute_f16(j);
            if (j + 1 < P) convert_f16(j + 1, af1, bf1);
        }
    }
    if (PERSIST) {
        tile_end(false);
        return;
    }

    // ---- epilogue (wave-uniform choice of the output kind and of the scale granularity) --------
    __builtin_amdgcn_s_waitcnt(0xC07F);
    __builtin_amdgcn_s_barrier();                           // every wave is done with the operand slabs
    const int wave_m0 = m0 + wm * 128, wave_n0 = n0 + wn * (32 * NB);
    // The lane index is taken afresh from the execution mask count: values derived from the one
    // computed before the K loop would have to stay in registers (or be spilled) all through it.
    const int le = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
    if (ep.b_per_col) {
        switch (ep.out_kind) {
            case OUT_F32: epilogue<OUT_F32, true, NB>(acc, smem, ep, C, M, N, wave_m0, wave_n0, w, le); break;
            case OUT_BF16: epilogue<OUT_BF16, true, NB>(acc, smem, ep, C, M, N, wave_m0, wave_n0, w, le); break;
            case OUT_E4M3: epilogue<OUT_E4M3, true, NB>(acc, smem, ep, C, M, N, wave_m0, wave_n0, w, le); break;
            default: epilogue<OUT_E5M2, true, NB>(acc, smem, ep, C, M, N, wave_m0, wave_n0, w, le); break;
        }
    } else {
        switch (ep.out_kind) {
            case OUT_F32: epilogue<OUT_F32, false, NB>(acc, smem, ep, C, M, N, wave_m0, wave_n0, w, le); break;
            case OUT_BF16: epilogue<OUT_BF16, false, NB>(acc, smem, ep, C, M, N, wave_m0, wave_n0, w, le); break;
            case OUT_E4M3: epilogue<OUT_E4M3, false, NB>(acc, smem, ep, C, M, N, wave_m0, wave_n0, w, le); break;
            default: epilogue<OUT_E5M2, false, NB>(acc, smem, ep, C, M, N, wave_m0, wave_n0, w, le); break;
        }
    }
}

template <int FMT_A, int FMT_B, int ACC, bool A_KC, bool B_KC, int NB, bool PERSIST>
__global__ __launch_bounds__(FAST_THREADS, 1) void gemm_fast_kernel(
    const uint8_t* __restrict__ A, const uint8_t* __restrict__ B, void* __restrict__ C,
    int M, int N, int K, EpilogueArgs ep, int group_m, int splits, int pairs_per_split)
{
    gemm_tile_body<FMT_A, FMT_B, ACC, A_KC, B_KC, NB, PERSIST>(A, B, C, M, N, K, ep, group_m, splits, pairs_per_split,
                                                              (int)blockIdx.x, 0, (N + 64 * NB - 1) / (64 * NB));
}

// Both tile widths in one launch: the first wide_cols * 256 columns of the output in 256 x 256 tiles
// (workgroups 0 .. tiles_m * wide_cols - 1, dispatched first), the remaining columns in 256 x 128
// tiles.  For problems whose tiles of one width leave much of the last round of workgroups empty
// (4096 x 6144: 384 wide tiles = 1.5 rounds, 768 narrow ones = 3 rounds at 0.6 of the wide tile's
// time each; 256 wide + 256 narrow = one round of each); the narrow tiles also fill the compute
// units that the last wide tiles leave idle.  The choice of wide_cols is the dispatcher's.
template <int FMT_A, int FMT_B, int ACC, bool A_KC, bool B_KC>
__global__ __launch_bounds__(FAST_THREADS, 1) void gemm_mixed_kernel(
    const uint8_t* __restrict__ A, const uint8_t* __restrict__ B, void* __restrict__ C,
    int M, int N, int K, EpilogueArgs ep, int group_m, int pairs, int wide_cols)
{
    const int wide_tiles = ((M + BM - 1) / BM) * wide_cols;
    if ((int)blockIdx.x < wide_tiles)
        gemm_tile_body<FMT_A, FMT_B, ACC, A_KC, B_KC, 4, false>(A, B, C, M, N, K, ep, group_m, 1, pairs, (int)blockIdx.x, 0, wide_cols);
    else
        gemm_tile_body<FMT_A, FMT_B, ACC, A_KC, B_KC, 2, false>(A, B, C, M, N, K, ep, group_m, 1, pairs, (int)blockIdx.x - wide_tiles,
                                                                wide_cols * 256, (N - wide_cols * 256 + 127) / 128);
}

// ---- launch ------------------------------------------------------------------------------
// The knob FP8_KNOB_GROUP_M sets the number of tile rows per band of the tile order (0: GROUP_M).
int group_m_setting()
{
    const int v = knob(FP8_KNOB_GROUP_M);
    return v > 0 ? v : GROUP_M;
}

// Compute units of the current device (the persistent form runs one workgroup on each).
int compute_units()
{
    static std::atomic<int> cached[64];
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0) return 256;
    if (dev < 64 && (n = cached[dev].load(std::memory_order_relaxed)) > 0) return n;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
    if (dev < 64) cached[dev].store(n, std::memory_order_relaxed);
    return n;
}

template <int FA, int FB, int ACC, bool A_KC, bool B_KC, int NB, bool PERSIST = false>
int launch_fast(const GemmArgs& g)
{
    // the kernel needs more dynamic LDS than the default limit: raised once per device
    static std::atomic<unsigned long long> attr_set{0ull};
    auto kern = gemm_fast_kernel<FA, FB, ACC, A_KC, B_KC, NB, PERSIST>;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return fail(FP8_ERR_DEVICE, "hipGetDevice failed");
    const unsigned long long bit = 1ull << (dev & 63);
    if (dev >= 64 || !(attr_set.load(std::memory_order_relaxed) & bit)) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, FAST_LDS);
        if (e != hipSuccess)
            return fail(FP8_ERR_DEVICE, "hipFuncSetAttribute(LDS=%d): %s", FAST_LDS, hipGetErrorString(e));
        if (dev < 64) attr_set.fetch_or(bit, std::memory_order_relaxed);
    }
    constexpr int BN = 64 * NB;
    const int tiles = (int)(((g.M + BM - 1) / BM) * ((g.N + BN - 1) / BN));
    const int pairs = (int)((g.K + 2 * BK - 1) / (2 * BK));
    const int splits = !PERSIST && g.splits > 1 ? g.splits : 1;
    const int grid = PERSIST ? min(tiles, compute_units()) : tiles * splits;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(FAST_THREADS), FAST_LDS, g.stream, g.A, g.B, g.C,
                       (int)g.M, (int)g.N, (int)g.K, g.ep, group_m_setting(), splits,
                       splits > 1 ? g.pairs_per_split : pairs);
    return check_launch(PERSIST ? "gemm (tiled kernel, persistent form)" : "gemm (tiled kernel)");
}

template <int FA, int FB, int ACC, bool A_KC, bool B_KC>
int launch_mixed(const GemmArgs& g)
{
    static std::atomic<unsigned long long> attr_set{0ull};
    auto kern = gemm_mixed_kernel<FA, FB, ACC, A_KC, B_KC>;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return fail(FP8_ERR_DEVICE, "hipGetDevice failed");
    const unsigned long long bit = 1ull << (dev & 63);
    if (dev >= 64 || !(attr_set.load(std::memory_order_relaxed) & bit)) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, FAST_LDS);
        if (e != hipSuccess)
            return fail(FP8_ERR_DEVICE, "hipFuncSetAttribute(LDS=%d): %s", FAST_LDS, hipGetErrorString(e));
        if (dev < 64) attr_set.fetch_or(bit, std::memory_order_relaxed);
    }
    const int64_t tiles_m = (g.M + BM - 1) / BM;
    const int64_t grid = tiles_m * g.wide_cols + tiles_m * ((g.N - (int64_t)g.wide_cols * 256 + 127) / 128);
    const int pairs = (int)((g.K + 2 * BK - 1) / (2 * BK));
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(FAST_THREADS), FAST_LDS, g.stream, g.A, g.B, g.C,
                       (int)g.M, (int)g.N, (int)g.K, g.ep, group_m_setting(), pairs, g.wide_cols);
    return check_launch("gemm (tiled kernel, both tile widths)");
}

}  // namespace

#if !defined(FP8MM_LAYOUT) || !defined(FP8MM_ACC)
#error "compile with -DFP8MM_LAYOUT=0..3 (2 * transA + transB) and -DFP8MM_ACC=0|1"
#endif

template <int NB>
static int launch_formats(const GemmArgs& g)
{
    constexpr bool A_KC = (FP8MM_LAYOUT & 2) == 0;   // A row-major M x K is K-contiguous
    constexpr bool B_KC = (FP8MM_LAYOUT & 1) != 0;   // B stored N x K is K-contiguous
    constexpr int ACC = FP8MM_ACC;
    if (NB == 2 && g.persist) {                      // the persistent form exists for the narrow tile
        if (g.fmtA == FP8_E4M3)
            return g.fmtB == FP8_E4M3 ? launch_fast<FP8_E4M3, FP8_E4M3, ACC, A_KC, B_KC, 2, true>(g)
                                      : launch_fast<FP8_E4M3, FP8_E5M2, ACC, A_KC, B_KC, 2, true>(g);
        return g.fmtB == FP8_E4M3 ? launch_fast<FP8_E5M2, FP8_E4M3, ACC, A_KC, B_KC, 2, true>(g)
                                  : launch_fast<FP8_E5M2, FP8_E5M2, ACC, A_KC, B_KC, 2, true>(g);
    }
    if (g.fmtA == FP8_E4M3)
        return g.fmtB == FP8_E4M3 ? launch_fast<FP8_E4M3, FP8_E4M3, ACC, A_KC, B_KC, NB>(g)
                                  : launch_fast<FP8_E4M3, FP8_E5M2, ACC, A_KC, B_KC, NB>(g);
    return g.fmtB == FP8_E4M3 ? launch_fast<FP8_E5M2, FP8_E4M3, ACC, A_KC, B_KC, NB>(g)
                              : launch_fast<FP8_E5M2, FP8_E5M2, ACC, A_KC, B_KC, NB>(g);
}

static int launch_mixed_formats(const GemmArgs& g)
{
    constexpr bool A_KC = (FP8MM_LAYOUT & 2) == 0, B_KC = (FP8MM_LAYOUT & 1) != 0;
    constexpr int ACC = FP8MM_ACC;
    if (g.fmtA == FP8_E4M3)
        return g.fmtB == FP8_E4M3 ? launch_mixed<FP8_E4M3, FP8_E4M3, ACC, A_KC, B_KC>(g) : launch_mixed<FP8_E4M3, FP8_E5M2, ACC, A_KC, B_KC>(g);
    return g.fmtB == FP8_E4M3 ? launch_mixed<FP8_E5M2, FP8_E4M3, ACC, A_KC, B_KC>(g) : launch_mixed<FP8_E5M2, FP8_E5M2, ACC, A_KC, B_KC>(g);
}

int FP8MM_TILED_NAME(FP8MM_LAYOUT, FP8MM_ACC)(const GemmArgs& g)
{
    if (g.wide_cols > 0) return launch_mixed_formats(g);
    return g.tile_n == 128 ? launch_formats<2>(g) : launch_formats<4>(g);
}

}  // namespace fp8mm
