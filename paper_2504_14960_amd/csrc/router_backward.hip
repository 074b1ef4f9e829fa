// Backward of the router (Eq. 2 + Eq. 3 by the chain rule; Section 3.3: the
// backward workflow mirrors the forward one).
//
//   router_dlogits_kernel   dgate [T,K] -> dlogits [T,E] through the (optional)
//                           renormalisation and the softmax Jacobian; one lane
//                           per token, a few passes over its E fp32 logits
//   router_dx_kernel        dx[t,:]  = sum_e dlogits[t,e] W_g[e,:]   (32 tokens x
//                           512 columns per workgroup on the fp32 matrix
//                           instruction, dlogits tile in LDS)
//   router_dw_partial / router_dw_reduce
//                           dW_g[e,:] = sum_t dlogits[t,e] x[t,:]: every
//                           workgroup sums a slab of tokens in the accumulators
//                           of the fp32 matrix instruction and writes an fp32
//                           partial; the partials are added in a fixed
//                           order (deterministic, no float atomics).  The same
//                           pass leaves per-slab column sums of dlogits, which
//                           router_dbias_reduce adds up to dbias.
//   router_dbias_kernel     dbias[e] = sum_t dlogits[t,e] when dW_g is not asked for
#include <type_traits>

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

// Both products of the router's backward run on the fp32 matrix instruction
// (32x32x2: lane l feeds A[l % 32][l / 32] and B[l / 32][l % 32], one value each,
// and holds D[8q + 4(l / 32) + u][l % 32] in element 4q + u).  With a k extent of
// two and one value per lane, both operands are read in their natural row-major
// layout; products and sums are fp32 as in the vector form.  A lane loads FOUR
// consecutive columns at once and uses them in four MFMAs, so the four
// accumulators of a lane are four consecutive output columns.
__device__ __forceinline__ f32x16 mfma_f32(float a, float b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

// Four consecutive elements as they sit in memory (bf16: 8 bytes, fp32: 16 bytes); converted only where they are
// used, so that a batch of loads can stay in flight.  Callers pass in-range addresses and mask the values later.
template <bool BF16>
struct Raw4 {
    typedef typename std::conditional<BF16, u32x2, f32x4>::type type;
};
template <bool BF16>
__device__ __forceinline__ typename Raw4<BF16>::type load_raw4(const void* p, size_t elem) {
    if constexpr (BF16)
        return *reinterpret_cast<const u32x2*>(static_cast<const uint16_t*>(p) + elem);
    else
        return *reinterpret_cast<const f32x4*>(static_cast<const float*>(p) + elem);
}
template <bool BF16>
__device__ __forceinline__ void cvt4(const typename Raw4<BF16>::type& r, bool ok, float (&v)[4]) {
    if constexpr (BF16) {
        v[0] = __uint_as_float(r[0] << 16);
        v[1] = __uint_as_float(r[0] & 0xffff0000u);
        v[2] = __uint_as_float(r[1] << 16);
        v[3] = __uint_as_float(r[1] & 0xffff0000u);
    } else {
        v[0] = r[0]; v[1] = r[1]; v[2] = r[2]; v[3] = r[3];
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] = ok ? v[j] : 0.f;
}

constexpr int DX_TOK = 32;    // tokens per workgroup of router_dx_kernel (one MFMA row block)
// tokens per slab of router_dw_partial_kernel: a function of T only, so the summation order is reproducible
inline int dw_slab(int T) { return T >= 32768 ? 256 : 128; }
constexpr int RB_WCOLS = 128; // columns per wave (4 per lane) of the router backward's MFMA kernels

// dx[t, c] = sum_e dl[t,e] W[e,c].  Workgroup = 32 tokens x 512 columns (4 waves of 128 columns); the dlogits tile
// sits in LDS (rows padded by one float: conflict-free column reads).  H a multiple of 8.
template <bool BF16>
__global__ __launch_bounds__(256) void router_dx_kernel(const float* __restrict__ dlogits, const void* __restrict__ w,
                                                        int T, int H, int E, void* __restrict__ dx) {
    __shared__ float dl[DX_TOK][kMaxExperts + 1];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int t0 = blockIdx.y * DX_TOK;
    for (int i = threadIdx.x; i < DX_TOK * E; i += 256) {
        const int lt = i / E, e = i - lt * E;
        dl[lt][e] = (t0 + lt < T) ? dlogits[(size_t)(t0 + lt) * E + e] : 0.f;
    }
    __syncthreads();
    const int row = lane & 31, half = lane >> 5;
    const int c = (blockIdx.x * 4 + wave) * RB_WCOLS + 4 * row;
    const bool c_ok = c < H;
    f32x16 acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;
    // operands of U steps (2 experts each) are requested before the MFMAs of the previous U steps are issued;
    // out-of-range lanes read a valid address (expert E - 1, column 0) and their values are zeroed at use
    constexpr int U = 8;
    typedef typename Raw4<BF16>::type raw_t;
    const int c_safe = c_ok ? c : 0;
    float a_cur[U], a_nxt[U];
    raw_t w_cur[U], w_nxt[U];
    auto fetch = [&](int e_first, float (&a)[U], raw_t (&wr)[U]) {
#pragma unroll
        for (int i = 0; i < U; ++i) {
            const int e = min(e_first + 2 * i + half, E - 1);
            a[i] = dl[row][e];
            wr[i] = load_raw4<BF16>(w, (size_t)e * H + c_safe);
        }
    };
    fetch(0, a_cur, w_cur);
    for (int e0 = 0; e0 < E; e0 += 2 * U) {
        const bool more = e0 + 2 * U < E;   // wave-uniform
        if (more) fetch(e0 + 2 * U, a_nxt, w_nxt);
#pragma unroll
        for (int i = 0; i < U; ++i) {
            const bool ok = e0 + 2 * i + half < E;
            float wv[4];
            cvt4<BF16>(w_cur[i], ok && c_ok, wv);
            const float a = ok ? a_cur[i] : 0.f;
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[j] = mfma_f32(a, wv[j], acc[j]);
        }
        if (!more) break;
#pragma unroll
        for (int i = 0; i < U; ++i) {
            a_cur[i] = a_nxt[i];
            w_cur[i] = w_nxt[i];
        }
    }
    if (!c_ok) return;
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int t = t0 + 8 * q + 4 * half + u;
            if (t >= T) continue;
            const size_t at = (size_t)t * H + c;
            const int v = 4 * q + u;
            if (BF16) {
                u32x2 o;
                o[0] = pack2_bf16(acc[0][v], acc[1][v]);
                o[1] = pack2_bf16(acc[2][v], acc[3][v]);
                *reinterpret_cast<u32x2*>(static_cast<uint16_t*>(dx) + at) = o;
            } else {
                *reinterpret_cast<f32x4*>(static_cast<float*>(dx) + at) = f32x4{acc[0][v], acc[1][v], acc[2][v], acc[3][v]};
            }
        }
}

// partial[s][e][c] = sum over the tokens of slab s of dl[t,e] x[t,c]; pbias[s][e] = sum over the slab of dl[t,e]
// (written by the first wave of the first column block).  Workgroup = one slab x 512 columns (4 waves of 128
// columns); a wave keeps two 32-expert blocks in its accumulators and passes over its tokens once per 64 experts.
// Token pairs (2p, 2p + 1) are the two k values of one MFMA: the sum over a slab runs in that fixed order.
template <bool BF16>
__global__ __launch_bounds__(256) void router_dw_partial_kernel(const float* __restrict__ dlogits,
                                                                const void* __restrict__ x, int T, int H, int E,
                                                                int slab, float* __restrict__ partial,
                                                                float* __restrict__ pbias) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int s = blockIdx.y, t0 = s * slab;
    const int nt = min(slab, T - t0);
    const int row = lane & 31, half = lane >> 5;
    const int c = (blockIdx.x * 4 + wave) * RB_WCOLS + 4 * row;
    const bool c_ok = c < H;
    const bool bias_wave = blockIdx.x == 0 && wave == 0;
    for (int eb = 0; eb < E; eb += 64) {
        const bool two = eb + 32 < E;   // wave-uniform: a second block of experts in this pass
        const bool e0_ok = eb + row < E, e1_ok = eb + 32 + row < E;
        f32x16 acc[2][4];
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[b][j][v] = 0.f;
        float bs0 = 0.f, bs1 = 0.f;
        // operands of U token pairs are requested before the MFMAs of the previous U pairs are issued; out-of-range
        // lanes read a valid address (last token of the slab, column 0, expert E - 1), zeroed at use
        constexpr int U = 4;
        typedef typename Raw4<BF16>::type raw_t;
        const int c_safe = c_ok ? c : 0;
        const int e0_safe = min(eb + row, E - 1), e1_safe = min(eb + 32 + row, E - 1);
        raw_t x_cur[U], x_nxt[U];
        float a0_cur[U], a1_cur[U], a0_nxt[U], a1_nxt[U];
        auto fetch = [&](int p_first, raw_t (&xr)[U], float (&a0)[U], float (&a1)[U]) {
#pragma unroll
            for (int i = 0; i < U; ++i) {
                const size_t t = (size_t)(t0 + min(p_first + 2 * i + half, nt - 1));
                xr[i] = load_raw4<BF16>(x, t * H + c_safe);
                a0[i] = dlogits[t * E + e0_safe];
                a1[i] = dlogits[t * E + e1_safe];
            }
        };
        fetch(0, x_cur, a0_cur, a1_cur);
        for (int p = 0; p < nt; p += 2 * U) {
            const bool more = p + 2 * U < nt;   // wave-uniform
            if (more) fetch(p + 2 * U, x_nxt, a0_nxt, a1_nxt);
#pragma unroll
            for (int i = 0; i < U; ++i) {
                const bool t_ok = p + 2 * i + half < nt;
                float xv[4];
                cvt4<BF16>(x_cur[i], t_ok && c_ok, xv);
                const float a0 = (t_ok && e0_ok) ? a0_cur[i] : 0.f;
                const float a1 = (t_ok && e1_ok) ? a1_cur[i] : 0.f;
                bs0 += a0;
                bs1 += a1;
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[0][j] = mfma_f32(a0, xv[j], acc[0][j]);
                if (two) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[1][j] = mfma_f32(a1, xv[j], acc[1][j]);
                }
            }
            if (!more) break;
#pragma unroll
            for (int i = 0; i < U; ++i) {
                x_cur[i] = x_nxt[i];
                a0_cur[i] = a0_nxt[i];
                a1_cur[i] = a1_nxt[i];
            }
        }
        if (c_ok) {
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int q = 0; q < 4; ++q)
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int e = eb + 32 * b + 8 * q + 4 * half + u;
                        const int v = 4 * q + u;
                        if (e < E)
                            *reinterpret_cast<f32x4*>(partial + ((size_t)s * E + e) * H + c) =
                                f32x4{acc[b][0][v], acc[b][1][v], acc[b][2][v], acc[b][3][v]};
                    }
        }
        if (bias_wave) {   // even tokens in lanes 0..31, odd tokens in lanes 32..63
            bs0 += __shfl_xor(bs0, 32, 64);
            bs1 += __shfl_xor(bs1, 32, 64);
            if (half == 0) {
                if (e0_ok) pbias[(size_t)s * E + eb + row] = bs0;
                if (e1_ok) pbias[(size_t)s * E + eb + 32 + row] = bs1;
            }
        }
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

// dbias[e] = sum_s pbias[s][e]: one workgroup per expert, strided partial sums folded in a fixed tree
__global__ __launch_bounds__(256) void router_dbias_reduce_kernel(const float* __restrict__ pbias, int S, int E,
                                                                  float* __restrict__ dbias) {
    __shared__ float red[256];
    const int e = blockIdx.x;
    float acc = 0.f;
    for (int s = threadIdx.x; s < S; s += 256) acc += pbias[(size_t)s * E + e];
    red[threadIdx.x] = acc;
    __syncthreads();
    for (int d = 128; d > 0; d >>= 1) {
        if (threadIdx.x < d) red[threadIdx.x] += red[threadIdx.x + d];
        __syncthreads();
    }
    if (threadIdx.x == 0) dbias[e] = red[0];
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
        const dim3 grid((H + 4 * RB_WCOLS - 1) / (4 * RB_WCOLS), (T + DX_TOK - 1) / DX_TOK);
        if (bf16)
            hipLaunchKernelGGL(router_dx_kernel<true>, grid, dim3(256), 0, s, dlogits, w, T, H, E, dx);
        else
            hipLaunchKernelGGL(router_dx_kernel<false>, grid, dim3(256), 0, s, dlogits, w, T, H, E, dx);
    }
    if (dw) {
        const int slab = dw_slab(T);
        const int S = (T + slab - 1) / slab;
        const dim3 grid((H + 4 * RB_WCOLS - 1) / (4 * RB_WCOLS), S);
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
        if (dbias) hipLaunchKernelGGL(router_dbias_reduce_kernel, dim3(E), dim3(256), 0, s, pbias, S, E, dbias);
    } else if (dbias) {
        hipLaunchKernelGGL(router_dbias_kernel, dim3(E), dim3(256), 0, s, dlogits, T, E, dbias);
    }
}

}  // namespace moe
