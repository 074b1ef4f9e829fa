// Per-tensor FP8 quantisation for the FP8 expert FFN (Section 4.5, FP8 with
// delayed scaling): dst = e4m3(src * scale), and max |src| is folded into
// *amax for the scales of later steps.  One pass, HBM-bound.
#include "fp8_convert.h"

namespace moe {

namespace {

// Each lane converts VEC consecutive values per step (one 16-byte load), U steps
// in flight; consecutive lanes take consecutive vectors, so loads and stores of a
// wave are contiguous.
template <bool BF16>
__global__ __launch_bounds__(256) void fp8_quantize_kernel(const void* __restrict__ src, size_t n, float scale,
                                                           uint8_t* __restrict__ dst, float* __restrict__ amax) {
    constexpr int VEC = BF16 ? 8 : 4;
    constexpr int U = 4;
    const size_t nvec = n / VEC;
    const size_t stride = (size_t)gridDim.x * 256;
    float m = 0.f;
    for (size_t i0 = (size_t)blockIdx.x * 256 + threadIdx.x; i0 < nvec; i0 += stride * U) {
        u32x4 in[U];
#pragma unroll
        for (int k = 0; k < U; ++k) {
            const size_t i = i0 + (size_t)k * stride;
            in[k] = u32x4{0u, 0u, 0u, 0u};
            if (i < nvec) in[k] = *reinterpret_cast<const u32x4*>(static_cast<const uint8_t*>(src) + i * 16);
        }
#pragma unroll
        for (int k = 0; k < U; ++k) {
            const size_t i = i0 + (size_t)k * stride;
            if (i >= nvec) continue;
            float v[VEC];
            if (BF16) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    v[2 * j] = __uint_as_float(in[k][j] << 16);
                    v[2 * j + 1] = __uint_as_float(in[k][j] & 0xffff0000u);
                }
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) v[j] = __uint_as_float(in[k][j]);
            }
            uint32_t w[VEC / 4];
#pragma unroll
            for (int q = 0; q < VEC / 4; ++q) {
#pragma unroll
                for (int j = 0; j < 4; ++j) m = fmaxf(m, fabsf(v[4 * q + j]));   // fmaxf drops a NaN operand
                w[q] = f32x4_to_e4m3(v[4 * q] * scale, v[4 * q + 1] * scale, v[4 * q + 2] * scale,
                                     v[4 * q + 3] * scale);
            }
            if (BF16) {
                u32x2 o;
                o[0] = w[0];
                o[1] = w[VEC / 4 - 1];
                *reinterpret_cast<u32x2*>(dst + i * VEC) = o;
            } else {
                *reinterpret_cast<uint32_t*>(dst + i * VEC) = w[0];
            }
        }
    }
    // tail (n not a multiple of VEC): the first few threads of block 0
    if (blockIdx.x == 0 && threadIdx.x < (n % VEC)) {
        const size_t i = nvec * VEC + threadIdx.x;
        const float x = BF16 ? __uint_as_float((uint32_t) static_cast<const uint16_t*>(src)[i] << 16)
                             : static_cast<const float*>(src)[i];
        m = fmaxf(m, fabsf(x));
        dst[i] = (uint8_t)f32_to_e4m3(x * scale);
    }
    if (amax) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
        // Non-negative floats order like their bit patterns.  *amax only grows, so a wave whose
        // maximum does not exceed the value it reads can skip the atomic: thousands of atomics
        // on one address would otherwise serialise and dominate the kernel.
        if ((threadIdx.x & 63) == 0 && m > __builtin_nontemporal_load(amax))
            atomicMax(reinterpret_cast<int*>(amax), __float_as_int(m));
    }
}

}  // namespace

void launch_fp8_quantize(const void* src, moe_dtype_t dt, size_t n, float scale, void* dst, float* amax,
                         hipStream_t s) {
    if (n == 0) return;
    const size_t vec = (dt == MOE_BF16) ? 8 : 4;
    size_t blocks = (n / vec + 4 * 256 - 1) / (4 * 256);   // 4 vectors per thread and pass
    if (blocks < 1) blocks = 1;
    if (blocks > 256 * 8) blocks = 256 * 8;
    if (dt == MOE_BF16)
        hipLaunchKernelGGL(fp8_quantize_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, s, src, n, scale,
                           static_cast<uint8_t*>(dst), amax);
    else
        hipLaunchKernelGGL(fp8_quantize_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, s, src, n, scale,
                           static_cast<uint8_t*>(dst), amax);
}

}  // namespace moe
