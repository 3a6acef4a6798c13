// Exact FP8 -> fp32 decode on the device, written from the field definitions of Table 1
// (arXiv 2209.05433): E4M3 = S.EEEE.MMM, bias 7, S.1111.111 is NaN, no infinities;
// E5M2 = S.EEEEE.MM, bias 15 = the upper byte of an IEEE half.
#pragma once

#include "common.hpp"

namespace fp8mm {

template <int FMT>
__device__ __forceinline__ float decode_fp8(unsigned b)
{
    if (FMT == FP8_E5M2) {
        return (float)__builtin_bit_cast(_Float16, (unsigned short)(b << 8));
    }
    const unsigned sign = (b & 0x80u) << 24;
    const unsigned e = (b >> 3) & 15u, m = b & 7u;
    unsigned mag;
    if (e == 15u && m == 7u) mag = 0x7fc00000u;
    else if (e == 0u) mag = __builtin_bit_cast(unsigned, (float)m * 0.001953125f);   // m * 2^-9
    else mag = ((e + 120u) << 23) | (m << 20);                                       // 2^(e-7) * (1 + m/8)
    return __builtin_bit_cast(float, mag | sign);
}

}  // namespace fp8mm
