// fp32 -> FP8 rounding on the device (arXiv 2209.05433, Section 2 and Table 1): round to the
// nearest FP8 value, ties to the even code; finite overflow saturates to the largest finite
// value (or, in the strict mode, becomes NaN / inf); NaN -> NaN, inf -> NaN (E4M3) or inf (E5M2).
// Used by the cast kernels and by the FP8-output epilogue of the GEMM.
#pragma once

#include "common.hpp"

namespace fp8mm {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float as_f32(unsigned u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ unsigned as_u32(float f) { return __builtin_bit_cast(unsigned, f); }

// Rounding by integer arithmetic on the bits of y.
//   normal results   : re-bias the exponent, add half of the dropped field (+ the tie bit),
//                      shift the dropped mantissa bits out; a mantissa carry bumps the
//                      exponent as it should.
//   subnormal results: adding 2^(emin - mbits + 23) in fp32 leaves the multiple of the
//                      subnormal step, rounded to nearest even by the adder, in the low bits.
//   SAT = false is the strict conversion of Section 2: rounding that lands beyond the largest
//   finite value gives NaN (E4M3) or inf (E5M2) instead of saturating.
template <int FMT, bool SAT = true>
__device__ __forceinline__ unsigned encode_bits(float y)
{
    constexpr int MB = FMT == FP8_E4M3 ? 3 : 2;                 // mantissa bits
    constexpr int BIAS = FMT == FP8_E4M3 ? 7 : 15;
    constexpr unsigned DROP = 23 - MB;                          // dropped fp32 mantissa bits
    constexpr unsigned REBIAS = (unsigned)(127 - BIAS) << 23;
    constexpr unsigned MIN_NORMAL = (unsigned)(127 + 1 - BIAS) << 23;
    constexpr unsigned MAGIC = (unsigned)(127 + 1 - BIAS - MB + 23) << 23;
    constexpr unsigned MAX_BITS = FMT == FP8_E4M3 ? 0x43E00000u : 0x47600000u;   // 448, 57344
    constexpr unsigned MAX_CODE = FMT == FP8_E4M3 ? 0x7Eu : 0x7Bu;
    constexpr unsigned INF_CODE = FMT == FP8_E4M3 ? 0x7Fu : 0x7Cu;

    const unsigned u = as_u32(y);
    const unsigned a = u & 0x7fffffffu;
    const unsigned sign = (u >> 24) & 0x80u;

    unsigned r = a - REBIAS;
    r = (r + ((1u << (DROP - 1)) - 1u) + ((r >> DROP) & 1u)) >> DROP;
    const unsigned sub = as_u32(as_f32(a) + as_f32(MAGIC)) - MAGIC;

    unsigned code = a < MIN_NORMAL ? sub : r;
    if (SAT) code = a >= MAX_BITS ? MAX_CODE : code;
    else code = code > INF_CODE ? INF_CODE : code;          // rounded past the grid: NaN / inf
    code = a >= 0x7f800000u ? INF_CODE : code;
    code = a > 0x7f800000u ? 0x7Fu : code;
    return sign | code;
}

// Two values through the hardware converter.  The converter rounds to nearest even and
// produces subnormals; the saturation rule is applied in front of it with a median-of-three
// clamp.  NaN and inf inputs are not handled here (the caller routes them to encode_bits).
template <int FMT, bool HI>
__device__ __forceinline__ unsigned cvt_pair(float a, float b, unsigned old)
{
    constexpr float FMAX = FMT == FP8_E4M3 ? 448.0f : 57344.0f;
    a = __builtin_amdgcn_fmed3f(a, FMAX, -FMAX);
    b = __builtin_amdgcn_fmed3f(b, FMAX, -FMAX);
    if (FMT == FP8_E4M3) return (unsigned)__builtin_amdgcn_cvt_pk_fp8_f32(a, b, (int)old, HI);
    return (unsigned)__builtin_amdgcn_cvt_pk_bf8_f32(a, b, (int)old, HI);
}

__device__ __forceinline__ bool is_special(float y)      // NaN or +-inf
{
    return __builtin_amdgcn_class(y, 0x207);
}

// Four scaled values -> one dword of FP8 bytes (element 0 in the low byte), integer path.
template <int FMT, bool SAT = true>
__device__ __forceinline__ unsigned encode4_bits(float y0, float y1, float y2, float y3)
{
    return encode_bits<FMT, SAT>(y0) | (encode_bits<FMT, SAT>(y1) << 8) | (encode_bits<FMT, SAT>(y2) << 16) |
           (encode_bits<FMT, SAT>(y3) << 24);
}

// Four scaled values -> 4 FP8 bytes (saturating): the converter instructions, with NaN / inf quadruples
// routed to the integer path.
template <int FMT>
__device__ __forceinline__ unsigned encode4(float y0, float y1, float y2, float y3)
{
    if (is_special(y0) | is_special(y1) | is_special(y2) | is_special(y3)) return encode4_bits<FMT>(y0, y1, y2, y3);
    const unsigned w = cvt_pair<FMT, false>(y0, y1, 0u);
    return cvt_pair<FMT, true>(y2, y3, w);
}

// Sixteen scaled values -> four dwords.  Converter path: one test for NaN/inf over all sixteen
// (a single, almost never taken branch per item), then eight packed conversions.
template <int FMT, int PATH>
__device__ __forceinline__ u32x4 encode16(const float (&y)[16])
{
    u32x4 o;
    if (PATH == kCastBitsStrict) {
#pragma unroll
        for (int d = 0; d < 4; ++d) o[d] = encode4_bits<FMT, false>(y[4 * d], y[4 * d + 1], y[4 * d + 2], y[4 * d + 3]);
        return o;
    }
    bool fast = PATH == kCastCvt;
    if (PATH == kCastCvt) {
        bool special = false;
#pragma unroll
        for (int i = 0; i < 16; ++i) special |= is_special(y[i]);
        fast = !special;
    }
    if (fast) {
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const unsigned w = cvt_pair<FMT, false>(y[4 * d], y[4 * d + 1], 0u);
            o[d] = cvt_pair<FMT, true>(y[4 * d + 2], y[4 * d + 3], w);
        }
    } else {
#pragma unroll
        for (int d = 0; d < 4; ++d) o[d] = encode4_bits<FMT>(y[4 * d], y[4 * d + 1], y[4 * d + 2], y[4 * d + 3]);
    }
    return o;
}

}  // namespace fp8mm
