// Backward of the router (Eq. 2 + Eq. 3 by the chain rule; Section 3.3: the
// backward workflow mirrors the forward one).
//
//   router_dlogits_kernel   dgate [T,K] -> dlogits [T,E] through the (optional)
//                           renormalisation and the softmax Jacobian; one lane
//                           per token, a few passes over its E fp32 logits
//   router_dx_kernel        dx[t,:]  = sum_e dlogits[t,e] W_g[e,:]   (16 tokens x
//                           2048 columns per workgroup, W_g rows read once per
//                           workgroup, dlogits tile in LDS)
//   router_dw_partial / router_dw_reduce
//                           dW_g[e,:] = sum_t dlogits[t,e] x[t,:]: every
//                           workgroup sums a slab of tokens into registers (a
//                           thread owns 4 columns x 32 experts; the dlogits tile
//                           is read from LDS four experts at a time) and writes
//                           an fp32 partial; the partials are added in a fixed
//                           order (deterministic, no float atomics).  The same
//                           pass leaves per-slab column sums of dlogits, which
//                           router_dbias_reduce adds up to dbias.
//   router_dbias_kernel     dbias[e] = sum_t dlogits[t,e] when dW_g is not asked for
#include "common.h"

namespace moe {

namespace {

__global__ __launch_bounds__(64) void router_dlogits_kernel(const float* __restrict__ logits,
                                                             const int32_t* __restrict__ idx,
                                                             const float* __restrict__ dgate, int T, int E, int K,
                                                             int renorm, float* __restrict__ dlogits) {
    const int t = blockIdx.x * 64 + threadIdx.x;
    if (t >= T) return;
    const float* l = logits + (size_t)t * E;
    const int32_t* ix = idx + (size_t)t * K;
    const float* dg = dgate + (size_t)t * K;
    float* dl = dlogits + (size_t)t * E;
    float m = -INFINITY;
    for (int e = 0; e < E; ++e) m = fmaxf(m, l[e]);
    float z = 0.f;
    for (int e = 0; e < E; ++e) z += expf(l[e] - m);
    const float rz = 1.f / z;
    float S = 0.f, a = 0.f;
    for (int k = 0; k < K; ++k) {
        const int e = ix[k];
        if ((unsigned)e < (unsigned)E) S += expf(l[e] - m) * rz;
    }
    if (renorm)
        for (int k = 0; k < K; ++k) {
            const int e = ix[k];
            if ((unsigned)e < (unsigned)E) a += dg[k] * (expf(l[e] - m) * rz / S);
        }
    float sum_qp = 0.f;
    for (int k = 0; k < K; ++k) {
        const int e = ix[k];
        if ((unsigned)e >= (unsigned)E) continue;
        const float q = renorm ? (dg[k] - a) / S : dg[k];
        sum_qp += q * (expf(l[e] - m) * rz);
    }
    for (int e = 0; e < E; ++e) dl[e] = -(expf(l[e] - m) * rz) * sum_qp;
    for (int k = 0; k < K; ++k) {
        const int e = ix[k];
        if ((unsigned)e >= (unsigned)E) continue;
        const float q = renorm ? (dg[k] - a) / S : dg[k];
        dl[e] += q * (expf(l[e] - m) * rz);
    }
}

template <bool BF16>
__device__ __forceinline__ void load8(const void* p, size_t elem, float (&v)[8]) {
    if (BF16) {
        const u32x4 r = *reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(p) + elem);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            v[2 * j] = __uint_as_float(r[j] << 16);
            v[2 * j + 1] = __uint_as_float(r[j] & 0xffff0000u);
        }
    } else {
        const f32x4 a = *reinterpret_cast<const f32x4*>(static_cast<const float*>(p) + elem);
        const f32x4 b = *reinterpret_cast<const f32x4*>(static_cast<const float*>(p) + elem + 4);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            v[j] = a[j];
            v[4 + j] = b[j];
        }
    }
}

constexpr int DX_TOK = 16;    // tokens per workgroup of router_dx_kernel
constexpr int DW_CHUNK = 64;  // tokens of the dlogits tile held in LDS at a time
constexpr int DW_EB = 32;     // experts per register block of router_dw_partial_kernel
constexpr int DW_COLS = 4;    // columns per thread of router_dw_partial_kernel
// tokens per slab of router_dw_partial_kernel: a function of T only, so the summation order is reproducible
__host__ __device__ inline int dw_slab(int T) { return T >= 32768 ? 256 : 128; }

// dx[t, c..c+7] = sum_e dl[t,e] W[e, c..c+7]; H a multiple of 8
template <bool BF16>
__global__ __launch_bounds__(256) void router_dx_kernel(const float* __restrict__ dlogits, const void* __restrict__ w,
                                                        int T, int H, int E, void* __restrict__ dx) {
    __shared__ float dl[DX_TOK][kMaxExperts];
    const int t0 = blockIdx.y * DX_TOK;
    const int c = (blockIdx.x * 256 + threadIdx.x) * 8;
    for (int i = threadIdx.x; i < DX_TOK * E; i += 256) {
        const int lt = i / E, e = i - lt * E;
        dl[lt][e] = (t0 + lt < T) ? dlogits[(size_t)(t0 + lt) * E + e] : 0.f;
    }
    __syncthreads();
    if (c >= H) return;
    float acc[DX_TOK][8];
#pragma unroll
    for (int lt = 0; lt < DX_TOK; ++lt)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[lt][j] = 0.f;
    for (int e = 0; e < E; ++e) {
        float wv[8];
        load8<BF16>(w, (size_t)e * H + c, wv);
#pragma unroll
        for (int lt = 0; lt < DX_TOK; ++lt) {
            const float d = dl[lt][e];
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[lt][j] = fmaf(d, wv[j], acc[lt][j]);
        }
    }
#pragma unroll
    for (int lt = 0; lt < DX_TOK; ++lt) {
        if (t0 + lt >= T) break;
        const size_t at = (size_t)(t0 + lt) * H + c;
        if (BF16) {
            u32x4 o;
#pragma unroll
            for (int j = 0; j < 4; ++j) o[j] = pack2_bf16(acc[lt][2 * j], acc[lt][2 * j + 1]);
            *reinterpret_cast<u32x4*>(static_cast<uint16_t*>(dx) + at) = o;
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) static_cast<float*>(dx)[at + j] = acc[lt][j];
        }
    }
}

// partial[s][e][c] = sum over the tokens of slab s of dl[t,e] x[t,c]; thread = DW_COLS columns x DW_EB experts.
// pbias[s][e] = sum over the tokens of slab s of dl[t,e] (written by the workgroups of the first column block).
template <bool BF16>
__global__ __launch_bounds__(256) void router_dw_partial_kernel(const float* __restrict__ dlogits,
                                                                const void* __restrict__ x, int T, int H, int E,
                                                                int slab, float* __restrict__ partial,
                                                                float* __restrict__ pbias) {
    __shared__ __attribute__((aligned(16))) float dl[DW_CHUNK][DW_EB];
    const int s = blockIdx.y, t0 = s * slab;
    const int c = (blockIdx.x * 256 + threadIdx.x) * DW_COLS;   // H is a multiple of 8
    const int nt = min(slab, T - t0);
    for (int e0 = 0; e0 < E; e0 += DW_EB) {
        const int ne = min(DW_EB, E - e0);
        float acc[DW_EB][DW_COLS];
#pragma unroll
        for (int le = 0; le < DW_EB; ++le)
#pragma unroll
            for (int j = 0; j < DW_COLS; ++j) acc[le][j] = 0.f;
        float bsum = 0.f;
        for (int k0 = 0; k0 < nt; k0 += DW_CHUNK) {
            const int nk = min(DW_CHUNK, nt - k0);
            __syncthreads();
            for (int i = threadIdx.x; i < DW_CHUNK * DW_EB; i += 256) {
                const int lt = i / DW_EB, le = i - lt * DW_EB;
                dl[lt][le] = (lt < nk && le < ne) ? dlogits[(size_t)(t0 + k0 + lt) * E + e0 + le] : 0.f;
            }
            __syncthreads();
            if (blockIdx.x == 0 && threadIdx.x < DW_EB)
                for (int lt = 0; lt < nk; ++lt) bsum += dl[lt][threadIdx.x];   // ascending token order
            if (c < H) {
#pragma unroll 4
                for (int lt = 0; lt < nk; ++lt) {
                    float xv[DW_COLS];
                    const size_t at = (size_t)(t0 + k0 + lt) * H + c;
                    if (BF16) {
                        const u32x2 r = *reinterpret_cast<const u32x2*>(static_cast<const uint16_t*>(x) + at);
                        xv[0] = __uint_as_float(r[0] << 16);
                        xv[1] = __uint_as_float(r[0] & 0xffff0000u);
                        xv[2] = __uint_as_float(r[1] << 16);
                        xv[3] = __uint_as_float(r[1] & 0xffff0000u);
                    } else {
                        const f32x4 r = *reinterpret_cast<const f32x4*>(static_cast<const float*>(x) + at);
#pragma unroll
                        for (int j = 0; j < DW_COLS; ++j) xv[j] = r[j];
                    }
#pragma unroll
                    for (int q = 0; q < DW_EB / 4; ++q) {
                        const f32x4 d = *reinterpret_cast<const f32x4*>(&dl[lt][4 * q]);
#pragma unroll
                        for (int u = 0; u < 4; ++u)
#pragma unroll
                            for (int j = 0; j < DW_COLS; ++j) acc[4 * q + u][j] = fmaf(d[u], xv[j], acc[4 * q + u][j]);
                    }
                }
            }
        }
        if (c < H) {
#pragma unroll
            for (int le = 0; le < DW_EB; ++le)
                if (le < ne) {
                    f32x4 o;
#pragma unroll
                    for (int j = 0; j < DW_COLS; ++j) o[j] = acc[le][j];
                    *reinterpret_cast<f32x4*>(partial + ((size_t)s * E + e0 + le) * H + c) = o;
                }
        }
        if (blockIdx.x == 0 && threadIdx.x < ne) pbias[(size_t)s * E + e0 + threadIdx.x] = bsum;
    }
}

// dw[i..i+3] = sum_s partial[s][i..i+3] in ascending s; n a multiple of 4
__global__ __launch_bounds__(256) void router_dw_reduce_kernel(const float* __restrict__ partial, int S, size_t n,
                                                               float* __restrict__ dw) {
    const size_t i = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (i >= n) return;
    f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int s = 0; s < S; ++s) {
        const f32x4 v = *reinterpret_cast<const f32x4*>(partial + (size_t)s * n + i);
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[j] += v[j];
    }
    *reinterpret_cast<f32x4*>(dw + i) = acc;
}

// dbias[e] = sum_s pbias[s][e] in ascending s
__global__ __launch_bounds__(256) void router_dbias_reduce_kernel(const float* __restrict__ pbias, int S, int E,
                                                                  float* __restrict__ dbias) {
    const int e = threadIdx.x;
    if (e >= E) return;
    float acc = 0.f;
    for (int s = 0; s < S; ++s) acc += pbias[(size_t)s * E + e];
    dbias[e] = acc;
}

// dbias[e] = sum_t dl[t,e]: one workgroup per expert, strided partial sums folded in a fixed tree
__global__ __launch_bounds__(256) void router_dbias_kernel(const float* __restrict__ dlogits, int T, int E,
                                                           float* __restrict__ dbias) {
    __shared__ float red[256];
    const int e = blockIdx.x;
    float acc = 0.f;
    for (int t = threadIdx.x; t < T; t += 256) acc += dlogits[(size_t)t * E + e];
    red[threadIdx.x] = acc;
    __syncthreads();
    for (int d = 128; d > 0; d >>= 1) {
        if (threadIdx.x < d) red[threadIdx.x] += red[threadIdx.x + d];
        __syncthreads();
    }
    if (threadIdx.x == 0) dbias[e] = red[0];
}

}  // namespace

size_t router_backward_workspace_bytes(int T, int H, int E) {
    const int slab = dw_slab(T);
    const size_t S = ((size_t)(T > 0 ? T : 1) + slab - 1) / slab;
    return S * (size_t)E * H * sizeof(float) + S * (size_t)E * sizeof(float);
}

void launch_router_backward(const void* x, const void* w, const float* logits, const int32_t* idx, const float* dgate,
                            int T, int H, int E, int K, int renorm, moe_dtype_t dt, float* dlogits, void* dx,
                            float* dw, float* dbias, void* ws, hipStream_t s) {
    hipLaunchKernelGGL(router_dlogits_kernel, dim3((T + 63) / 64), dim3(64), 0, s, logits, idx, dgate, T, E, K,
                       renorm, dlogits);
    const bool bf16 = dt == MOE_BF16;
    if (dx) {
        const dim3 grid((H / 8 + 255) / 256, (T + DX_TOK - 1) / DX_TOK);
        if (bf16)
            hipLaunchKernelGGL(router_dx_kernel<true>, grid, dim3(256), 0, s, dlogits, w, T, H, E, dx);
        else
            hipLaunchKernelGGL(router_dx_kernel<false>, grid, dim3(256), 0, s, dlogits, w, T, H, E, dx);
    }
    if (dw) {
        const int slab = dw_slab(T);
        const int S = (T + slab - 1) / slab;
        const dim3 grid((H / DW_COLS + 255) / 256, S);
        float* partial = static_cast<float*>(ws);
        float* pbias = partial + (size_t)S * E * H;
        if (bf16)
            hipLaunchKernelGGL(router_dw_partial_kernel<true>, grid, dim3(256), 0, s, dlogits, x, T, H, E, slab,
                               partial, pbias);
        else
            hipLaunchKernelGGL(router_dw_partial_kernel<false>, grid, dim3(256), 0, s, dlogits, x, T, H, E, slab,
                               partial, pbias);
        const size_t n = (size_t)E * H;
        hipLaunchKernelGGL(router_dw_reduce_kernel, dim3((unsigned)((n / 4 + 255) / 256)), dim3(256), 0, s, partial, S,
                           n, dw);
        if (dbias) hipLaunchKernelGGL(router_dbias_reduce_kernel, dim3(1), dim3(256), 0, s, pbias, S, E, dbias);
    } else if (dbias) {
        hipLaunchKernelGGL(router_dbias_kernel, dim3(E), dim3(256), 0, s, dlogits, T, E, dbias);
    }
}

}  // namespace moe
