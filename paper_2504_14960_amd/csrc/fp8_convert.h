// fp32 -> FP8 (OCP E4M3) conversion used by the quantisation kernel and by the
// FP8 GEMM's epilogue.
#pragma once

#include "common.h"

namespace moe {

// Two fp32 values to their nearest E4M3 codes (OCP: bias 7, largest finite 448,
// no infinities), ties to even; magnitudes above 448, infinities included,
// saturate to 448; NaN stays NaN.  Returns code(a) | code(b) << 8.
//
// The hardware conversion rounds exactly this way for every finite input up to
// the saturation point but turns larger magnitudes into NaN, so the inputs are
// clamped first; the clamp maps NaN to 448, which is put right afterwards.
__device__ __forceinline__ uint32_t f32x2_to_e4m3(float a, float b) {
    const float ca = __builtin_amdgcn_fmed3f(a, -448.f, 448.f);
    const float cb = __builtin_amdgcn_fmed3f(b, -448.f, 448.f);
    uint32_t r = (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(ca, cb, 0, false) & 0xffffu;
    if (a != a) r = (r & 0xff00u) | 0x7fu | ((__float_as_uint(a) >> 24) & 0x80u);
    if (b != b) r = (r & 0x00ffu) | 0x7f00u | ((__float_as_uint(b) >> 16) & 0x8000u);
    return r;
}

// four values to four codes, lowest byte first
__device__ __forceinline__ uint32_t f32x4_to_e4m3(float a, float b, float c, float d) {
    return f32x2_to_e4m3(a, b) | (f32x2_to_e4m3(c, d) << 16);
}

__device__ __forceinline__ uint32_t f32_to_e4m3(float x) { return f32x2_to_e4m3(x, x) & 0xffu; }

}  // namespace moe
