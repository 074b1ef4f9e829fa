// a1. Router: logits = x W_g^T (+ bias), softmax over experts, top-K gating
// (Eq. 2 and Eq. 3, Section 3.1.1; router paragraph of Section 3.3).
//
// bf16 path: one workgroup owns 16*MB tokens and all experts.  Its four waves
// split the hidden dimension; each wave streams its slices of the token rows
// with fully coalesced 16-byte loads, parks them in a wave-private LDS region
// and re-reads them in MFMA operand order (16x16x32 bf16, fp32 accumulate).
// The router weight is small and stays in L2; its fragments are read straight
// from global memory.  Partial sums are folded in a fixed wave order, so the
// logits are bit-reproducible.  Selection is done by groups of lanes, one
// group per token, with butterfly reductions on (value desc, index asc) keys.
#include "common.h"

namespace moe {

namespace {

__device__ __forceinline__ bool ranks_before(float a, int ia, float b, int ib) {
    return (a > b) || (a == b && ia < ib);
}

// One token per group of G lanes (G a power of two, <= 64); lane `lig` of the
// group holds the logits of experts lig + j*G, j < VPL.  Lane k of the group
// writes slot k.
template <int VPL>
__device__ __forceinline__ void select_topk(const float (&vin)[VPL], int lig, int G, int E, int K,
                                            int renorm, bool valid, int32_t* idx_out,
                                            float* gate_out) {
    float v[VPL];
    float m = -INFINITY;
#pragma unroll
    for (int j = 0; j < VPL; ++j) {
        const int e = lig + j * G;
        float x = vin[j];
        x = (x != x) ? -INFINITY : x;  // NaN ranks last
        v[j] = (e < E) ? x : -INFINITY;
        m = fmaxf(m, v[j]);
    }
    for (int off = G >> 1; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, G));
    float z = 0.f;
#pragma unroll
    for (int j = 0; j < VPL; ++j) {
        const int e = lig + j * G;
        if (e < E) z += expf(v[j] - m);
    }
    for (int off = G >> 1; off > 0; off >>= 1) z += __shfl_xor(z, off, G);

    uint32_t taken = 0;
    float my_gate = 0.f, gsum = 0.f;
    int my_idx = 0;
    for (int k = 0; k < K; ++k) {
        float bv = -INFINITY;
        int be = 0x7fffffff;
#pragma unroll
        for (int j = 0; j < VPL; ++j) {
            const int e = lig + j * G;
            if (e < E && !((taken >> j) & 1u) && ranks_before(v[j], e, bv, be)) {
                bv = v[j];
                be = e;
            }
        }
        for (int off = G >> 1; off > 0; off >>= 1) {
            const float ov = __shfl_xor(bv, off, G);
            const int oe = __shfl_xor(be, off, G);
            if (ranks_before(ov, oe, bv, be)) {
                bv = ov;
                be = oe;
            }
        }
        if (be < E && (be & (G - 1)) == lig) taken |= 1u << (be / G);
        const float p = expf(bv - m) / z;
        gsum += p;
        if (lig == k) {
            my_gate = p;
            my_idx = be;
        }
    }
    if (renorm) my_gate /= gsum;
    if (valid && lig < K) {
        idx_out[lig] = my_idx;
        gate_out[lig] = my_gate;
    }
}

__host__ __device__ inline int group_lanes(int E) {
    int g = 1;
    while (g < E && g < 64) g <<= 1;
    return g;
}

// Selection for `ntok` tokens whose logits sit in `rows` (row stride `ld`, LDS
// or global), spread over the 4 waves of the workgroup.
template <int VPL>
__device__ __forceinline__ void select_block(const float* rows, int ld, int ntok, int t0, int T,
                                             int E, int K, int renorm, int32_t* topk_idx,
                                             float* topk_gate) {
    const int G = group_lanes(E);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nwaves = blockDim.x >> 6;
    const int per_wave = 64 / G;
    const int lig = lane & (G - 1), grp = lane / G;
    for (int base = wave * per_wave; base < ntok; base += nwaves * per_wave) {
        const int lt = base + grp;
        const bool valid = lt < ntok && (t0 + lt) < T;
        float v[VPL];
#pragma unroll
        for (int j = 0; j < VPL; ++j) {
            const int e = lig + j * G;
            v[j] = (valid && e < E) ? rows[(size_t)lt * ld + e] : -INFINITY;
        }
        const size_t o = (size_t)(t0 + (valid ? lt : 0)) * K;
        select_topk<VPL>(v, lig, G, E, K, renorm, valid, topk_idx + o, topk_gate + o);
    }
}

__device__ __forceinline__ void select_dispatch(const float* rows, int ld, int ntok, int t0, int T,
                                                int E, int K, int renorm, int32_t* topk_idx,
                                                float* topk_gate) {
    if (E <= 64)
        select_block<1>(rows, ld, ntok, t0, T, E, K, renorm, topk_idx, topk_gate);
    else if (E <= 128)
        select_block<2>(rows, ld, ntok, t0, T, E, K, renorm, topk_idx, topk_gate);
    else
        select_block<4>(rows, ld, ntok, t0, T, E, K, renorm, topk_idx, topk_gate);
}

// Selection with L lanes per token (K <= KSEL <= 8, L in {1, 2, 4, 8}).  Lane
// `sub` of a token walks its block of ceil(E/L) consecutive logits (with an odd
// row stride the lanes of a wave then hit distinct LDS banks), keeping its KSEL
// best in a sorted register list (insertion by compare-and-swap on the key
// (value desc, index asc), so equal logits keep the lower index first).  The L
// lists are then merged pairwise across lanes: the element-wise better of my
// list and the partner's reversed list is a bitonic sequence holding the KSEL
// best of both, and log2(KSEL) compare-exchange stages sort it; both partners
// end with the same list.  A second walk gives the softmax denominator.
// L = 1 needs no cross-lane traffic at all; L = 8 gives 8192 tokens of a
// 64-expert layer 1024 waves of work instead of 128.
// `rows` must be LDS (row stride `ld`, odd => conflict-free).
template <int KSEL, int L>
__device__ __forceinline__ void select_lanes(const float* rows, int ld, int ntok, int t0, int T, int E,
                                             int K, int renorm, int32_t* topk_idx, float* topk_gate) {
    const int sub = threadIdx.x % L;
    const int tpb = blockDim.x / L;  // tokens per pass of the workgroup
    for (int base = 0; base < ntok; base += tpb) {
        const int lt = base + threadIdx.x / L;
        const bool valid = lt < ntok && t0 + lt < T;  // same for the L lanes of a token
        const float* r = rows + (size_t)(valid ? lt : 0) * ld;
        float lv[KSEL];
        int le[KSEL];
#pragma unroll
        for (int j = 0; j < KSEL; ++j) {
            lv[j] = -INFINITY;
            le[j] = 0x7fffffff;
        }
        const int e_begin = sub * ((E + L - 1) / L), e_end = min(E, e_begin + (E + L - 1) / L);
        for (int e = e_begin; e < e_end; ++e) {
            float cv = r[e];
            cv = (cv != cv) ? -INFINITY : cv;  // NaN ranks last
            int ce = e;
#pragma unroll
            for (int j = 0; j < KSEL; ++j) {
                const bool b = ranks_before(cv, ce, lv[j], le[j]);
                const float tv = b ? lv[j] : cv;
                const int te = b ? le[j] : ce;
                lv[j] = b ? cv : lv[j];
                le[j] = b ? ce : le[j];
                cv = tv;
                ce = te;
            }
        }
#pragma unroll
        for (int off = 1; off < L; off <<= 1) {
            float pv[KSEL];
            int pe[KSEL];
#pragma unroll
            for (int j = 0; j < KSEL; ++j) {
                pv[j] = __shfl_xor(lv[j], off, 64);
                pe[j] = __shfl_xor(le[j], off, 64);
            }
#pragma unroll
            for (int j = 0; j < KSEL; ++j) {
                const bool b = ranks_before(pv[KSEL - 1 - j], pe[KSEL - 1 - j], lv[j], le[j]);
                lv[j] = b ? pv[KSEL - 1 - j] : lv[j];
                le[j] = b ? pe[KSEL - 1 - j] : le[j];
            }
#pragma unroll
            for (int d = KSEL / 2; d > 0; d >>= 1)
#pragma unroll
                for (int j = 0; j < KSEL; ++j)
                    if ((j & d) == 0) {
                        const bool b = ranks_before(lv[j + d], le[j + d], lv[j], le[j]);
                        const float tv = lv[j];
                        const int te = le[j];
                        lv[j] = b ? lv[j + d] : tv;
                        le[j] = b ? le[j + d] : te;
                        lv[j + d] = b ? tv : lv[j + d];
                        le[j + d] = b ? te : le[j + d];
                    }
        }
        const float m = lv[0];
        float z = 0.f;
        for (int e = e_begin; e < e_end; ++e) {
            float v = r[e];
            v = (v != v) ? -INFINITY : v;
            z += expf(v - m);
        }
#pragma unroll
        for (int off = 1; off < L; off <<= 1) z += __shfl_xor(z, off, 64);
        float gsum = 0.f;
#pragma unroll
        for (int k = 0; k < KSEL; ++k)
            if (k < K) gsum += expf(lv[k] - m) / z;
        // lane `sub` writes the slots sub, sub + L, ...
#pragma unroll
        for (int k = 0; k < KSEL; ++k)
            if (k < K && (k % L) == sub && valid) {
                const size_t o = (size_t)(t0 + lt) * K;
                const float p = expf(lv[k] - m) / z;
                topk_idx[o + k] = le[k];
                topk_gate[o + k] = renorm ? p / gsum : p;
            }
    }
}

// lanes per token of the register-list selection: about 8 logits per lane
__host__ __device__ inline int lanes_per_token(int E) { return E >= 64 ? 8 : E >= 32 ? 4 : E >= 16 ? 2 : 1; }

template <int KSEL>
__device__ __forceinline__ void select_lanes_for(const float* rows, int ld, int ntok, int t0, int T, int E,
                                                 int K, int renorm, int32_t* topk_idx, float* topk_gate) {
    switch (lanes_per_token(E)) {
        case 8: select_lanes<KSEL, 8>(rows, ld, ntok, t0, T, E, K, renorm, topk_idx, topk_gate); break;
        case 4: select_lanes<KSEL, 4>(rows, ld, ntok, t0, T, E, K, renorm, topk_idx, topk_gate); break;
        case 2: select_lanes<KSEL, 2>(rows, ld, ntok, t0, T, E, K, renorm, topk_idx, topk_gate); break;
        default: select_lanes<KSEL, 1>(rows, ld, ntok, t0, T, E, K, renorm, topk_idx, topk_gate); break;
    }
}

// K <= 8: register lists; larger K: one lane group per token.
__device__ __forceinline__ void select_tokens(const float* rows, int ld, int ntok, int t0, int T, int E,
                                              int K, int renorm, int32_t* topk_idx, float* topk_gate) {
    if (K <= 2)
        select_lanes_for<2>(rows, ld, ntok, t0, T, E, K, renorm, topk_idx, topk_gate);
    else if (K <= 4)
        select_lanes_for<4>(rows, ld, ntok, t0, T, E, K, renorm, topk_idx, topk_gate);
    else if (K <= 8)
        select_lanes_for<8>(rows, ld, ntok, t0, T, E, K, renorm, topk_idx, topk_gate);
    else
        select_dispatch(rows, ld, ntok, t0, T, E, K, renorm, topk_idx, topk_gate);
}

// ------------------------------------------------------------------ bf16 / MFMA
template <int MB, int NB>
__global__ __launch_bounds__(256) void router_bf16_kernel(
    const bf16_t* __restrict__ x, const bf16_t* __restrict__ w, const float* __restrict__ bias,
    float* __restrict__ logits, int T, int H, int E, int K, int renorm,
    int32_t* __restrict__ topk_idx, float* __restrict__ topk_gate) {
    constexpr int TOK = 16 * MB;      // tokens per workgroup
    // MFMA k-steps per slice: 8 token loads in flight per lane where the weight
    // fragments of a slice (KSTEPS * NB of them, kept in registers) allow it
    constexpr int KSTEPS = (8 / MB < ((16 / NB) > 1 ? (16 / NB) : 1)) ? 8 / MB : ((16 / NB) > 1 ? (16 / NB) : 1);
    constexpr int KC = 32 * KSTEPS;   // hidden elements per slice
    constexpr int LPR = KC / 8;       // lanes covering one row slice
    constexpr int KCP = KC + 8;       // padded LDS row (elements)
    constexpr int RPI = 64 / LPR;     // rows per load instruction
    constexpr int NLD = TOK / RPI;    // token loads per lane per slice
    constexpr int EP = 16 * NB;       // experts padded to the MFMA N size
    __shared__ __attribute__((aligned(16))) bf16_t xs[4][TOK][KCP];
    __shared__ float red[TOK][EP + 1];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int t0 = blockIdx.x * TOK;
    const int nchunks = (H + KC - 1) / KC;

    f32x4 acc[MB][NB];
#pragma unroll
    for (int a = 0; a < MB; ++a)
#pragma unroll
        for (int b = 0; b < NB; ++b) acc[a][b] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int lrow = lane / LPR, lcol = (lane % LPR) * 8;
    const int fr = lane & 15, fg = lane >> 4;  // fragment row / k-group
    // both the token slice and the matching router-weight fragments of the NEXT
    // slice are requested before the current slice is multiplied, so neither the
    // HBM nor the L2 round trip sits in front of an MFMA
    u32x4 xr[NLD], wr[KSTEPS][NB];
    auto load_chunk = [&](int c) {
        const int k = c * KC + lcol;
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int t = t0 + i * RPI + lrow;
            u32x4 v = u32x4{0u, 0u, 0u, 0u};
            if (t < T && k < H) v = *reinterpret_cast<const u32x4*>(x + (size_t)t * H + k);
            xr[i] = v;
        }
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s) {
            const int kw = c * KC + s * 32 + fg * 8;
#pragma unroll
            for (int b2 = 0; b2 < NB; ++b2) {
                const int e = b2 * 16 + fr;
                u32x4 v = u32x4{0u, 0u, 0u, 0u};
                if (e < E && kw < H) v = *reinterpret_cast<const u32x4*>(w + (size_t)e * H + kw);
                wr[s][b2] = v;
            }
        }
    };

    // workgroups start at different slices of the hidden dimension: the rows of x
    // and of the router weight lie a whole row apart, so workgroups that walk the
    // slices in step would all ask the same few memory channels at a time
    const int rot = (int)((blockIdx.x * 7u) % (unsigned)nchunks);
    auto slice_of = [&](int c) { const int cc = c + rot; return cc >= nchunks ? cc - nchunks : cc; };
    if (wave < nchunks) load_chunk(slice_of(wave));
    for (int c = wave; c < nchunks; c += 4) {
        bf16x8 bfrag[KSTEPS][NB];
#pragma unroll
        for (int i = 0; i < NLD; ++i)
            *reinterpret_cast<u32x4*>(&xs[wave][i * RPI + lrow][lcol]) = xr[i];
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s)
#pragma unroll
            for (int b2 = 0; b2 < NB; ++b2) bfrag[s][b2] = __builtin_bit_cast(bf16x8, wr[s][b2]);
        if (c + 4 < nchunks) load_chunk(slice_of(c + 4));
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s) {
#pragma unroll
            for (int a = 0; a < MB; ++a) {
                const u32x4 av = *reinterpret_cast<const u32x4*>(&xs[wave][a * 16 + fr][s * 32 + fg * 8]);
                const bf16x8 afrag = __builtin_bit_cast(bf16x8, av);
#pragma unroll
                for (int b2 = 0; b2 < NB; ++b2)
                    acc[a][b2] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(afrag, bfrag[s][b2], acc[a][b2], 0, 0, 0);
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }

    // fold the four partial sums in wave order 0,1,2,3 (fixed => reproducible)
    for (int ww = 0; ww < 4; ++ww) {
        if (wave == ww) {
#pragma unroll
            for (int a = 0; a < MB; ++a)
#pragma unroll
                for (int b = 0; b < NB; ++b)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        float* p = &red[a * 16 + fg * 4 + r][b * 16 + fr];
                        *p = (ww == 0) ? acc[a][b][r] : (*p + acc[a][b][r]);
                    }
        }
        __syncthreads();
    }
    // bias, write logits
    for (int i = threadIdx.x; i < TOK * E; i += 256) {
        const int lt = i / E, e = i - lt * E;
        float v = red[lt][e];
        if (bias) v += bias[e];
        red[lt][e] = v;
        if (t0 + lt < T) logits[(size_t)(t0 + lt) * E + e] = v;
    }
    __syncthreads();
    select_tokens(&red[0][0], EP + 1, TOK, t0, T, E, K, renorm, topk_idx, topk_gate);
}

// ------------------------------------------------------------------ fp32 / VALU
// One wave per token; lanes stride the hidden dimension, one expert at a time.
__global__ __launch_bounds__(256) void router_f32_kernel(
    const float* __restrict__ x, const float* __restrict__ w, const float* __restrict__ bias,
    float* __restrict__ logits, int T, int H, int E, int K, int renorm,
    int32_t* __restrict__ topk_idx, float* __restrict__ topk_gate) {
    __shared__ float red[4][kMaxExperts + 1];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int t0 = blockIdx.x * 4;
    const int t = t0 + wave;
    if (t < T) {
        const float* xr = x + (size_t)t * H;
        for (int e = 0; e < E; ++e) {
            const float* wr = w + (size_t)e * H;
            float s = 0.f;
            for (int h = lane * 4; h < H; h += 256) {
                const f32x4 a = *reinterpret_cast<const f32x4*>(xr + h);
                const f32x4 b = *reinterpret_cast<const f32x4*>(wr + h);
                s = fmaf(a[0], b[0], s);
                s = fmaf(a[1], b[1], s);
                s = fmaf(a[2], b[2], s);
                s = fmaf(a[3], b[3], s);
            }
            for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
            if (bias) s += bias[e];
            if (lane == 0) {
                red[wave][e] = s;
                logits[(size_t)t * E + e] = s;
            }
        }
    }
    __syncthreads();
    select_tokens(&red[0][0], kMaxExperts + 1, 4, t0, T, E, K, renorm, topk_idx, topk_gate);
}

// ------------------------------------------------------------------ selection only
constexpr int kTopkTileFloats = 12288;

// tokens per tile of the selection-only kernel: one pass of the workgroup
__host__ __device__ inline int topk_tile_tokens(int E, int K) {
    if (K <= 8) return 256 / lanes_per_token(E);
    const int fit = kTopkTileFloats / (E | 1);
    return fit > 256 ? 256 : fit;
}

__global__ __launch_bounds__(256) void topk_only_kernel(const float* __restrict__ logits, int T,
                                                        int E, int K, int renorm,
                                                        int32_t* __restrict__ topk_idx,
                                                        float* __restrict__ topk_gate) {
    // a tile of tokens is copied to LDS with coalesced loads (row stride odd),
    // then selected from there
    __shared__ float tile[kTopkTileFloats];
    const int ld = E | 1;
    const int per_block = topk_tile_tokens(E, K);
    for (int t0 = blockIdx.x * per_block; t0 < T; t0 += gridDim.x * per_block) {
        const int ntok = min(per_block, T - t0);
        const float* src = logits + (size_t)t0 * E;
        for (int i = threadIdx.x; i < ntok * E; i += 256) {
            const int lt = i / E, e = i - lt * E;
            tile[lt * ld + e] = src[i];
        }
        __syncthreads();
        select_tokens(tile, ld, ntok, t0, T, E, K, renorm, topk_idx, topk_gate);
        __syncthreads();
    }
}

template <int MB, int NB>
void launch_bf16(const void* x, const void* w, const float* bias, float* logits, int T, int H, int E,
                 int K, int renorm, int32_t* idx, float* gate, hipStream_t s) {
    const int grid = (T + 16 * MB - 1) / (16 * MB);
    hipLaunchKernelGGL((router_bf16_kernel<MB, NB>), dim3(grid), dim3(256), 0, s,
                       static_cast<const bf16_t*>(x), static_cast<const bf16_t*>(w), bias, logits, T,
                       H, E, K, renorm, idx, gate);
}

}  // namespace

static int g_router_tile = 0;  // 16-token blocks per workgroup; 0 = chosen from T and E
void set_router_tile(int mb) { g_router_tile = mb; }

void launch_router(const void* x, const void* w, const float* bias, float* logits, int T, int H,
                   int E, int K, int renorm, moe_dtype_t dt, int32_t* idx, float* gate,
                   hipStream_t s) {
    if (x == nullptr) {
        const int per_block = topk_tile_tokens(E, K);
        int grid = (T + per_block - 1) / per_block;
        if (grid > 4096) grid = 4096;
        hipLaunchKernelGGL(topk_only_kernel, dim3(grid), dim3(256), 0, s, logits, T, E, K, renorm, idx, gate);
        return;
    }
    if (dt == MOE_F32) {
        hipLaunchKernelGGL(router_f32_kernel, dim3((T + 3) / 4), dim3(256), 0, s,
                           static_cast<const float*>(x), static_cast<const float*>(w), bias, logits,
                           T, H, E, K, renorm, idx, gate);
        return;
    }
    const int nb = (E + 15) / 16;
    // tokens per workgroup: enough workgroups to fill 256 CUs, but from 16
    // experts on a taller tile so the router weight is re-read less often
    int mb = (T >= 32768) ? 4 : (T >= 16384 ? 2 : 1);
    if (E >= 16 && mb < 2) mb = 2;
    if (g_router_tile == 1 || g_router_tile == 2 || g_router_tile == 4) mb = g_router_tile;
#define ROUTER_CASE(M, N)                                                          \
    launch_bf16<M, N>(x, w, bias, logits, T, H, E, K, renorm, idx, gate, s);       \
    return;
    if (nb <= 1) {
        if (mb == 4) { ROUTER_CASE(4, 1) } else if (mb == 2) { ROUTER_CASE(2, 1) } else { ROUTER_CASE(1, 1) }
    } else if (nb <= 2) {
        if (mb == 4) { ROUTER_CASE(4, 2) } else if (mb == 2) { ROUTER_CASE(2, 2) } else { ROUTER_CASE(1, 2) }
    } else if (nb <= 4) {
        if (mb == 4) { ROUTER_CASE(4, 4) } else if (mb == 2) { ROUTER_CASE(2, 4) } else { ROUTER_CASE(1, 4) }
    } else if (nb <= 8) {
        ROUTER_CASE(2, 8)
    } else {
        ROUTER_CASE(1, 16)
    }
#undef ROUTER_CASE
}

}  // namespace moe
