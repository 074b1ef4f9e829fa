// a4. Un-permute + gate-weighted combine: the paper's "Token Restore" (Section
// 3.1.2) fused with the weighted sum of Eq. 1 (Section 3.1.1).
//
// One wave per token.  Lane k fetches the token's k-th row index and gate; the
// wave then walks the row in 16-byte-per-lane slices, gathers that slice from
// each kept expert row, accumulates gate * value in fp32 in ascending k and
// rounds once.  Dropped assignments (row < 0) contribute nothing.
#include "common.h"

namespace moe {

namespace {

template <bool BF16>
__global__ __launch_bounds__(256) void combine_kernel(const uint8_t* __restrict__ y_perm,
                                                      const int32_t* __restrict__ row_of_assign,
                                                      const float* __restrict__ gate,
                                                      const uint8_t* __restrict__ addend,
                                                      uint8_t* __restrict__ y, int T, int K,
                                                      int row_bytes, int r_max) {
    constexpr int NV = BF16 ? 8 : 4;  // values per 16-byte slice
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int t = blockIdx.x * 4 + wave; t < T; t += gridDim.x * 4) {
        int my_row = -1;
        float my_gate = 0.f;
        if (lane < K) {
            my_row = row_of_assign[(size_t)t * K + lane];
            my_gate = gate[(size_t)t * K + lane];
        }
        if ((unsigned)my_row >= (unsigned)r_max) my_row = -1;
        const uint64_t kept = __ballot(my_row >= 0);
        for (int o0 = 0; o0 < row_bytes; o0 += 2048) {  // uniform trip count: shuffles inside
            float acc[2][NV];
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < NV; ++j) acc[i][j] = 0.f;
            const int o = o0 + lane * 16;
            uint64_t m = kept;
            while (m) {
                const int k = __ffsll((unsigned long long)m) - 1;
                m &= m - 1;
                const int row = __shfl(my_row, k, 64);
                const float g = __shfl(my_gate, k, 64);
                const uint8_t* src = y_perm + (size_t)row * row_bytes + o;
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    if (o + i * 1024 < row_bytes) {
                        const u32x4 v = *reinterpret_cast<const u32x4*>(src + i * 1024);
                        if (BF16) {
#pragma unroll
                            for (int j = 0; j < 4; ++j) {
                                acc[i][2 * j] = fmaf(g, __uint_as_float(v[j] << 16), acc[i][2 * j]);
                                acc[i][2 * j + 1] = fmaf(g, __uint_as_float(v[j] & 0xffff0000u), acc[i][2 * j + 1]);
                            }
                        } else {
#pragma unroll
                            for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(g, __uint_as_float(v[j]), acc[i][j]);
                        }
                    }
                }
            }
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                if (o + i * 1024 < row_bytes) {
                    const size_t at = (size_t)t * row_bytes + o + i * 1024;
                    if (addend) {
                        const u32x4 v = *reinterpret_cast<const u32x4*>(addend + at);
                        if (BF16) {
#pragma unroll
                            for (int j = 0; j < 4; ++j) {
                                acc[i][2 * j] += __uint_as_float(v[j] << 16);
                                acc[i][2 * j + 1] += __uint_as_float(v[j] & 0xffff0000u);
                            }
                        } else {
#pragma unroll
                            for (int j = 0; j < 4; ++j) acc[i][j] += __uint_as_float(v[j]);
                        }
                    }
                    u32x4 out;
                    if (BF16) {
#pragma unroll
                        for (int j = 0; j < 4; ++j) out[j] = pack2_bf16(acc[i][2 * j], acc[i][2 * j + 1]);
                    } else {
#pragma unroll
                        for (int j = 0; j < 4; ++j) out[j] = __float_as_uint(acc[i][j]);
                    }
                    *reinterpret_cast<u32x4*>(y + at) = out;
                }
            }
        }
    }
}

}  // namespace

void launch_combine(const void* y_perm, const int32_t* row_of_assign, const float* gate,
                    const void* addend, int T, int H, int K, int r_max, moe_dtype_t dt, void* y,
                    hipStream_t s) {
    int grid = (T + 3) / 4;
    if (grid > 256 * 16) grid = 256 * 16;
    const int row_bytes = H * (dt == MOE_BF16 ? 2 : 4);
    if (dt == MOE_BF16)
        hipLaunchKernelGGL((combine_kernel<true>), dim3(grid), dim3(256), 0, s,
                           static_cast<const uint8_t*>(y_perm), row_of_assign, gate,
                           static_cast<const uint8_t*>(addend), static_cast<uint8_t*>(y), T, K,
                           row_bytes, r_max);
    else
        hipLaunchKernelGGL((combine_kernel<false>), dim3(grid), dim3(256), 0, s,
                           static_cast<const uint8_t*>(y_perm), row_of_assign, gate,
                           static_cast<const uint8_t*>(addend), static_cast<uint8_t*>(y), T, K,
                           row_bytes, r_max);
}

}  // namespace moe
