// a4. Un-permute + gate-weighted combine: the paper's "Token Restore" (Section
// 3.1.2) fused with the weighted sum of Eq. 1 (Section 3.1.1); further down its
// backward.  Without gates the same kernels are the backward of the permute
// (a sum of the kept rows of every token).
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
            my_gate = gate ? gate[(size_t)t * K + lane] : 1.f;   // no gates: plain sum of the kept rows
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

// Fast path for K <= KMAX (2, 4 or 8): all row indices and gates of a token are
// made wave-uniform first, then every 16-byte slice of all K rows is requested
// before the first FMA, so up to 8 loads per lane are in flight.  Whether an
// assignment was dropped is wave-uniform, so skipping it costs a scalar branch
// only; the sum still runs in ascending k.
template <bool BF16, int KMAX>
__global__ __launch_bounds__(256) void combine_small_k_kernel(
    const uint8_t* __restrict__ y_perm, const int32_t* __restrict__ row_of_assign,
    const float* __restrict__ gate, const uint8_t* __restrict__ addend, uint8_t* __restrict__ y, int T,
    int K, int row_bytes, int r_max) {
    constexpr int NV = BF16 ? 8 : 4;
    constexpr int CP = KMAX == 8 ? 2 : 8 / KMAX;  // 1 KiB slices per pass (8 to 16 loads per lane in flight)
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int t = blockIdx.x * 4 + wave; t < T; t += gridDim.x * 4) {
        int my_row = -1;
        float my_gate = 0.f;
        if (lane < K) {
            my_row = row_of_assign[(size_t)t * K + lane];
            my_gate = gate ? gate[(size_t)t * K + lane] : 1.f;   // no gates: plain sum of the kept rows
        }
        if ((unsigned)my_row >= (unsigned)r_max) my_row = -1;
        int rows[KMAX];
        float gates[KMAX];
        bool keep[KMAX];
#pragma unroll
        for (int k = 0; k < KMAX; ++k) {
            const int r = __builtin_amdgcn_readlane(my_row, k);
            keep[k] = r >= 0;
            rows[k] = keep[k] ? r : 0;
            gates[k] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, my_gate), k));
        }
        for (int o0 = 0; o0 < row_bytes; o0 += CP * 1024) {
            u32x4 v[KMAX][CP];
#pragma unroll
            for (int k = 0; k < KMAX; ++k) {
                const uint8_t* src = y_perm + (size_t)rows[k] * row_bytes;
#pragma unroll
                for (int i = 0; i < CP; ++i) {
                    const int o = o0 + i * 1024 + lane * 16;
                    v[k][i] = u32x4{0u, 0u, 0u, 0u};
                    if (keep[k] && o < row_bytes) v[k][i] = *reinterpret_cast<const u32x4*>(src + o);
                }
            }
#pragma unroll
            for (int i = 0; i < CP; ++i) {
                const int o = o0 + i * 1024 + lane * 16;
                if (o >= row_bytes) continue;
                float acc[NV];
#pragma unroll
                for (int j = 0; j < NV; ++j) acc[j] = 0.f;
#pragma unroll
                for (int k = 0; k < KMAX; ++k) {
                    if (!keep[k]) continue;  // wave-uniform
                    const float g = gates[k];
                    if (BF16) {
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            acc[2 * j] = fmaf(g, __uint_as_float(v[k][i][j] << 16), acc[2 * j]);
                            acc[2 * j + 1] = fmaf(g, __uint_as_float(v[k][i][j] & 0xffff0000u), acc[2 * j + 1]);
                        }
                    } else {
#pragma unroll
                        for (int j = 0; j < 4; ++j) acc[j] = fmaf(g, __uint_as_float(v[k][i][j]), acc[j]);
                    }
                }
                const size_t at = (size_t)t * row_bytes + o;
                if (addend) {
                    const u32x4 av = *reinterpret_cast<const u32x4*>(addend + at);
                    if (BF16) {
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            acc[2 * j] += __uint_as_float(av[j] << 16);
                            acc[2 * j + 1] += __uint_as_float(av[j] & 0xffff0000u);
                        }
                    } else {
#pragma unroll
                        for (int j = 0; j < 4; ++j) acc[j] += __uint_as_float(av[j]);
                    }
                }
                u32x4 out;
                if (BF16) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) out[j] = pack2_bf16(acc[2 * j], acc[2 * j + 1]);
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j) out[j] = __float_as_uint(acc[j]);
                }
                *reinterpret_cast<u32x4*>(y + at) = out;
            }
        }
    }
}

// Backward of the combine (Section 3.3: the backward mirrors the forward).  One
// wave per token: the token's dy row is read once in 16-byte lanes; for each kept
// assignment the scaled row gate * dy goes to dy_perm[row] (every kept row has
// exactly one source) and the dot product <dy, y_perm[row]> is accumulated in fp32
// and reduced over the wave in a fixed order.  Dropped assignments get dgate = 0.
template <bool BF16>
__global__ __launch_bounds__(256) void combine_backward_kernel(
    const uint8_t* __restrict__ dy, const uint8_t* __restrict__ y_perm, const int32_t* __restrict__ row_of_assign,
    const float* __restrict__ gate, uint8_t* __restrict__ dy_perm, float* __restrict__ dgate, int T, int K,
    int row_bytes, int r_max) {
    constexpr int NV = BF16 ? 8 : 4;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int t = blockIdx.x * 4 + wave; t < T; t += gridDim.x * 4) {
        int my_row = -1;
        float my_gate = 0.f;
        if (lane < K) {
            my_row = row_of_assign[(size_t)t * K + lane];
            my_gate = gate[(size_t)t * K + lane];
        }
        if ((unsigned)my_row >= (unsigned)r_max) my_row = -1;
        float my_dot = 0.f;  // lane k ends up holding dgate[t,k]
        for (int k = 0; k < K; ++k) {  // uniform trip count: shuffles inside
            const int row = __shfl(my_row, k, 64);
            if (row < 0) continue;     // wave-uniform
            const float g = __shfl(my_gate, k, 64);
            const uint8_t* src = dy + (size_t)t * row_bytes;
            const uint8_t* yp = y_perm + (size_t)row * row_bytes;
            uint8_t* dst = dy_perm + (size_t)row * row_bytes;
            float dot = 0.f;
            for (int o = lane * 16; o < row_bytes; o += 1024) {
                const u32x4 v = *reinterpret_cast<const u32x4*>(src + o);
                const u32x4 w = *reinterpret_cast<const u32x4*>(yp + o);
                float a[NV], b[NV];
                if (BF16) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        a[2 * j] = __uint_as_float(v[j] << 16);
                        a[2 * j + 1] = __uint_as_float(v[j] & 0xffff0000u);
                        b[2 * j] = __uint_as_float(w[j] << 16);
                        b[2 * j + 1] = __uint_as_float(w[j] & 0xffff0000u);
                    }
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        a[j] = __uint_as_float(v[j]);
                        b[j] = __uint_as_float(w[j]);
                    }
                }
                u32x4 out;
#pragma unroll
                for (int j = 0; j < NV; ++j) dot = fmaf(a[j], b[j], dot);
                if (BF16) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) out[j] = pack2_bf16(g * a[2 * j], g * a[2 * j + 1]);
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j) out[j] = __float_as_uint(g * a[j]);
                }
                *reinterpret_cast<u32x4*>(dst + o) = out;
            }
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) dot += __shfl_xor(dot, off, 64);
            if (lane == k) my_dot = dot;
        }
        if (lane < K) dgate[(size_t)t * K + lane] = my_dot;
    }
}

// Fast path of the backward for K <= KMAX (2, 4 or 8), same idea as the forward's:
// rows and gates wave-uniform, the dy slices of a pass read once, every kept
// y_perm slice requested before the first FMA.
template <bool BF16, int KMAX>
__global__ __launch_bounds__(256) void combine_backward_small_k_kernel(
    const uint8_t* __restrict__ dy, const uint8_t* __restrict__ y_perm, const int32_t* __restrict__ row_of_assign,
    const float* __restrict__ gate, uint8_t* __restrict__ dy_perm, float* __restrict__ dgate, int T, int K,
    int row_bytes, int r_max) {
    constexpr int NV = BF16 ? 8 : 4;
    constexpr int CP = KMAX == 8 ? 2 : 8 / KMAX;  // 1 KiB slices per pass (8 to 16 loads per lane in flight)
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int t = blockIdx.x * 4 + wave; t < T; t += gridDim.x * 4) {
        int my_row = -1;
        float my_gate = 0.f;
        if (lane < K) {
            my_row = row_of_assign[(size_t)t * K + lane];
            my_gate = gate[(size_t)t * K + lane];
        }
        if ((unsigned)my_row >= (unsigned)r_max) my_row = -1;
        int rows[KMAX];
        float gates[KMAX], dot[KMAX];
        bool keep[KMAX];
#pragma unroll
        for (int k = 0; k < KMAX; ++k) {
            const int r = __builtin_amdgcn_readlane(my_row, k);
            keep[k] = r >= 0;
            rows[k] = keep[k] ? r : 0;
            gates[k] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, my_gate), k));
            dot[k] = 0.f;
        }
        const uint8_t* src = dy + (size_t)t * row_bytes;
        for (int o0 = 0; o0 < row_bytes; o0 += CP * 1024) {
            u32x4 v[CP], w[KMAX][CP];
#pragma unroll
            for (int i = 0; i < CP; ++i) {
                const int o = o0 + i * 1024 + lane * 16;
                v[i] = u32x4{0u, 0u, 0u, 0u};
                if (o < row_bytes) v[i] = *reinterpret_cast<const u32x4*>(src + o);
            }
#pragma unroll
            for (int k = 0; k < KMAX; ++k)
#pragma unroll
                for (int i = 0; i < CP; ++i) {
                    const int o = o0 + i * 1024 + lane * 16;
                    w[k][i] = u32x4{0u, 0u, 0u, 0u};
                    if (keep[k] && o < row_bytes)
                        w[k][i] = *reinterpret_cast<const u32x4*>(y_perm + (size_t)rows[k] * row_bytes + o);
                }
#pragma unroll
            for (int i = 0; i < CP; ++i) {
                const int o = o0 + i * 1024 + lane * 16;
                if (o >= row_bytes) continue;
                float a[NV];
                if (BF16) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        a[2 * j] = __uint_as_float(v[i][j] << 16);
                        a[2 * j + 1] = __uint_as_float(v[i][j] & 0xffff0000u);
                    }
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j) a[j] = __uint_as_float(v[i][j]);
                }
#pragma unroll
                for (int k = 0; k < KMAX; ++k) {
                    if (!keep[k]) continue;  // wave-uniform
                    u32x4 out;
                    if (BF16) {
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            dot[k] = fmaf(a[2 * j], __uint_as_float(w[k][i][j] << 16), dot[k]);
                            dot[k] = fmaf(a[2 * j + 1], __uint_as_float(w[k][i][j] & 0xffff0000u), dot[k]);
                            out[j] = pack2_bf16(gates[k] * a[2 * j], gates[k] * a[2 * j + 1]);
                        }
                    } else {
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            dot[k] = fmaf(a[j], __uint_as_float(w[k][i][j]), dot[k]);
                            out[j] = __float_as_uint(gates[k] * a[j]);
                        }
                    }
                    *reinterpret_cast<u32x4*>(dy_perm + (size_t)rows[k] * row_bytes + o) = out;
                }
            }
        }
        float my_dot = 0.f;
#pragma unroll
        for (int k = 0; k < KMAX; ++k) {
            float d = dot[k];
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) d += __shfl_xor(d, off, 64);
            if (lane == k) my_dot = keep[k] ? d : 0.f;
        }
        if (lane < K) dgate[(size_t)t * K + lane] = my_dot;
    }
}

template <bool BF16>
void launch_combine_backward_t(const void* dy, const void* y_perm, const int32_t* row_of_assign, const float* gate,
                               int T, int H, int K, int r_max, void* dy_perm, float* dgate, hipStream_t s) {
    int grid = (T + 3) / 4;
    if (grid > 256 * 16) grid = 256 * 16;
    const int row_bytes = H * (BF16 ? 2 : 4);
    const uint8_t* a = static_cast<const uint8_t*>(dy);
    const uint8_t* b = static_cast<const uint8_t*>(y_perm);
    uint8_t* c = static_cast<uint8_t*>(dy_perm);
    if (K <= 2)
        hipLaunchKernelGGL((combine_backward_small_k_kernel<BF16, 2>), dim3(grid), dim3(256), 0, s, a, b, row_of_assign, gate, c, dgate, T, K, row_bytes, r_max);
    else if (K <= 4)
        hipLaunchKernelGGL((combine_backward_small_k_kernel<BF16, 4>), dim3(grid), dim3(256), 0, s, a, b, row_of_assign, gate, c, dgate, T, K, row_bytes, r_max);
    else if (K <= 8)
        hipLaunchKernelGGL((combine_backward_small_k_kernel<BF16, 8>), dim3(grid), dim3(256), 0, s, a, b, row_of_assign, gate, c, dgate, T, K, row_bytes, r_max);
    else
        hipLaunchKernelGGL((combine_backward_kernel<BF16>), dim3(grid), dim3(256), 0, s, a, b, row_of_assign, gate, c, dgate, T, K, row_bytes, r_max);
}

template <bool BF16>
void launch_combine_t(const void* y_perm, const int32_t* row_of_assign, const float* gate,
                      const void* addend, int T, int H, int K, int r_max, void* y, hipStream_t s) {
    int grid = (T + 3) / 4;
    if (grid > 256 * 16) grid = 256 * 16;
    const int row_bytes = H * (BF16 ? 2 : 4);
    const uint8_t* yp = static_cast<const uint8_t*>(y_perm);
    const uint8_t* ad = static_cast<const uint8_t*>(addend);
    uint8_t* out = static_cast<uint8_t*>(y);
    if (K <= 2)
        hipLaunchKernelGGL((combine_small_k_kernel<BF16, 2>), dim3(grid), dim3(256), 0, s, yp, row_of_assign, gate, ad, out, T, K, row_bytes, r_max);
    else if (K <= 4)
        hipLaunchKernelGGL((combine_small_k_kernel<BF16, 4>), dim3(grid), dim3(256), 0, s, yp, row_of_assign, gate, ad, out, T, K, row_bytes, r_max);
    else if (K <= 8)
        hipLaunchKernelGGL((combine_small_k_kernel<BF16, 8>), dim3(grid), dim3(256), 0, s, yp, row_of_assign, gate, ad, out, T, K, row_bytes, r_max);
    else
        hipLaunchKernelGGL((combine_kernel<BF16>), dim3(grid), dim3(256), 0, s, yp, row_of_assign, gate, ad, out, T, K, row_bytes, r_max);
}

}  // namespace

void launch_combine_backward(const void* dy, const void* y_perm, const int32_t* row_of_assign, const float* gate,
                             int T, int H, int K, int r_max, moe_dtype_t dt, void* dy_perm, float* dgate,
                             hipStream_t s) {
    if (dt == MOE_BF16)
        launch_combine_backward_t<true>(dy, y_perm, row_of_assign, gate, T, H, K, r_max, dy_perm, dgate, s);
    else
        launch_combine_backward_t<false>(dy, y_perm, row_of_assign, gate, T, H, K, r_max, dy_perm, dgate, s);
}

void launch_combine(const void* y_perm, const int32_t* row_of_assign, const float* gate,
                    const void* addend, int T, int H, int K, int r_max, moe_dtype_t dt, void* y,
                    hipStream_t s) {
    if (dt == MOE_BF16)
        launch_combine_t<true>(y_perm, row_of_assign, gate, addend, T, H, K, r_max, y, s);
    else
        launch_combine_t<false>(y_perm, row_of_assign, gate, addend, T, H, K, r_max, y, s);
}

}  // namespace moe
