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
//                           workgroup sums a slab of tokens into registers and
//                           writes an fp32 partial; the partials are added in a
//                           fixed order (deterministic, no float atomics)
//   router_dbias_kernel     dbias[e] = sum_t dlogits[t,e]
#include "common.h"

namespace moe {

namespace {

__global__ __launch_bounds__(256) void router_dlogits_kernel(const float* __restrict__ logits,
                                                             const int32_t* __restrict__ idx,
                                                             const float* __restrict__ dgate, int T, int E, int K,
                                                             int renorm, float* __restrict__ dlogits) {
    const int t = blockIdx.x * 256 + threadIdx.x;
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
constexpr int DW_TOK = 128;   // tokens per workgroup (slab) of router_dw_partial_kernel
constexpr int DW_EB = 32;     // experts per register block of router_dw_partial_kernel

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

// partial[s][e][c] = sum over the tokens of slab s of dl[t,e] x[t,c]; thread = one column
template <bool BF16>
__global__ __launch_bounds__(256) void router_dw_partial_kernel(const float* __restrict__ dlogits,
                                                                const void* __restrict__ x, int T, int H, int E,
                                                                float* __restrict__ partial) {
    __shared__ float dl[DW_TOK][DW_EB + 1];
    const int s = blockIdx.y, t0 = s * DW_TOK;
    const int c = blockIdx.x * 256 + threadIdx.x;
    const int nt = min(DW_TOK, T - t0);
    for (int e0 = 0; e0 < E; e0 += DW_EB) {
        const int ne = min(DW_EB, E - e0);
        __syncthreads();
        for (int i = threadIdx.x; i < DW_TOK * DW_EB; i += 256) {
            const int lt = i / DW_EB, le = i - lt * DW_EB;
            dl[lt][le] = (lt < nt && le < ne) ? dlogits[(size_t)(t0 + lt) * E + e0 + le] : 0.f;
        }
        __syncthreads();
        if (c >= H) continue;
        float acc[DW_EB];
#pragma unroll
        for (int le = 0; le < DW_EB; ++le) acc[le] = 0.f;
        for (int lt = 0; lt < nt; ++lt) {
            const float xv = BF16 ? __uint_as_float((uint32_t) static_cast<const uint16_t*>(x)[(size_t)(t0 + lt) * H + c] << 16)
                                  : static_cast<const float*>(x)[(size_t)(t0 + lt) * H + c];
#pragma unroll
            for (int le = 0; le < DW_EB; ++le) acc[le] = fmaf(dl[lt][le], xv, acc[le]);
        }
        for (int le = 0; le < ne; ++le) partial[((size_t)s * E + e0 + le) * H + c] = acc[le];
    }
}

// dw[i] = sum_s partial[s][i] in ascending s
__global__ __launch_bounds__(256) void router_dw_reduce_kernel(const float* __restrict__ partial, int S, size_t n,
                                                               float* __restrict__ dw) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    float acc = 0.f;
    for (int s = 0; s < S; ++s) acc += partial[(size_t)s * n + i];
    dw[i] = acc;
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
    const size_t S = ((size_t)T + DW_TOK - 1) / DW_TOK;
    return (S > 0 ? S : 1) * (size_t)E * H * sizeof(float);
}

void launch_router_backward(const void* x, const void* w, const float* logits, const int32_t* idx, const float* dgate,
                            int T, int H, int E, int K, int renorm, moe_dtype_t dt, float* dlogits, void* dx,
                            float* dw, float* dbias, void* ws, hipStream_t s) {
    hipLaunchKernelGGL(router_dlogits_kernel, dim3((T + 255) / 256), dim3(256), 0, s, logits, idx, dgate, T, E, K,
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
        const int S = (T + DW_TOK - 1) / DW_TOK;
        const dim3 grid((H + 255) / 256, S);
        float* partial = static_cast<float*>(ws);
        if (bf16)
            hipLaunchKernelGGL(router_dw_partial_kernel<true>, grid, dim3(256), 0, s, dlogits, x, T, H, E, partial);
        else
            hipLaunchKernelGGL(router_dw_partial_kernel<false>, grid, dim3(256), 0, s, dlogits, x, T, H, E, partial);
        const size_t n = (size_t)E * H;
        hipLaunchKernelGGL(router_dw_reduce_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, partial, S, n, dw);
    }
    if (dbias) hipLaunchKernelGGL(router_dbias_kernel, dim3(E), dim3(256), 0, s, dlogits, T, E, dbias);
}

}  // namespace moe
