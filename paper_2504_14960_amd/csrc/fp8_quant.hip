// Per-tensor FP8 quantisation for the FP8 expert FFN (Section 4.5, FP8 with
// delayed scaling): dst = e4m3(src * scale), and max |src| is folded into
// *amax for the scales of later steps.  One pass, HBM-bound: 16 values per lane
// per iteration (32 or 64 bytes in, 16 bytes out).
#include "fp8_convert.h"

namespace moe {

namespace {

template <bool BF16>
__global__ __launch_bounds__(256) void fp8_quantize_kernel(const void* __restrict__ src, size_t n, float scale,
                                                           uint8_t* __restrict__ dst, float* __restrict__ amax) {
    const size_t nvec = n / 16;
    float m = 0.f;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < nvec; i += (size_t)gridDim.x * 256) {
        float v[16];
        if (BF16) {
            const u32x4* p = reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(src) + i * 16);
            const u32x4 a = p[0], b = p[1];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                v[2 * j] = __uint_as_float(a[j] << 16);
                v[2 * j + 1] = __uint_as_float(a[j] & 0xffff0000u);
                v[8 + 2 * j] = __uint_as_float(b[j] << 16);
                v[8 + 2 * j + 1] = __uint_as_float(b[j] & 0xffff0000u);
            }
        } else {
            const u32x4* p = reinterpret_cast<const u32x4*>(static_cast<const float*>(src) + i * 16);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const u32x4 a = p[q];
#pragma unroll
                for (int j = 0; j < 4; ++j) v[4 * q + j] = __uint_as_float(a[j]);
            }
        }
        u32x4 o;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            uint32_t w = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float x = v[4 * q + j];
                m = fmaxf(m, fabsf(x));   // fmaxf drops a NaN operand
                w |= f32_to_e4m3(x * scale) << (8 * j);
            }
            o[q] = w;
        }
        *reinterpret_cast<u32x4*>(dst + i * 16) = o;
    }
    // tail (n not a multiple of 16): the first few threads of block 0
    if (blockIdx.x == 0 && threadIdx.x < (n & 15)) {
        const size_t i = nvec * 16 + threadIdx.x;
        const float x = BF16 ? __uint_as_float((uint32_t) static_cast<const uint16_t*>(src)[i] << 16)
                             : static_cast<const float*>(src)[i];
        m = fmaxf(m, fabsf(x));
        dst[i] = (uint8_t)f32_to_e4m3(x * scale);
    }
    if (amax) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
        // non-negative floats order like their bit patterns
        if ((threadIdx.x & 63) == 0 && m > 0.f) atomicMax(reinterpret_cast<int*>(amax), __float_as_int(m));
    }
}

}  // namespace

void launch_fp8_quantize(const void* src, moe_dtype_t dt, size_t n, float scale, void* dst, float* amax,
                         hipStream_t s) {
    if (n == 0) return;
    size_t blocks = (n / 16 + 255) / 256;
    if (blocks < 1) blocks = 1;
    if (blocks > 256 * 16) blocks = 256 * 16;
    if (dt == MOE_BF16)
        hipLaunchKernelGGL(fp8_quantize_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, s, src, n, scale,
                           static_cast<uint8_t*>(dst), amax);
    else
        hipLaunchKernelGGL(fp8_quantize_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, s, src, n, scale,
                           static_cast<uint8_t*>(dst), amax);
}

}  // namespace moe
