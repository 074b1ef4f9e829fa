// fp32 -> FP8 (OCP E4M3) conversion used by the quantisation kernel and by the
// FP8 GEMM's epilogue.
#pragma once

#include "common.h"

namespace moe {

// nearest E4M3 code (OCP: bias 7, largest finite 448, no infinities), ties to
// even, magnitudes above 448 saturate, NaN stays NaN
__device__ __forceinline__ uint32_t f32_to_e4m3(float x) {
    const uint32_t u = __float_as_uint(x);
    const uint32_t sign = (u >> 24) & 0x80u;
    uint32_t a = u & 0x7fffffffu;
    uint32_t code;
    if (a > 0x7f800000u) {
        code = 0x7fu;                              // NaN
    } else if (a > 0x43e00000u) {
        code = 0x7eu;                              // above 448: saturate
    } else if (a < 0x3c800000u) {
        code = (uint32_t)(int)rintf(__uint_as_float(a) * 512.0f);   // below 2^-6: multiples of 2^-9
    } else {
        a += 0x7ffffu + ((a >> 20) & 1u);          // round the mantissa to 3 bits, ties to even
        code = (a >> 20) - ((127u - 7u) << 3);     // rebias; a carry out of the mantissa bumps the exponent
    }
    return sign | code;
}

}  // namespace moe
