// Pieces shared by the grouped-GEMM kernels: the ragged tile scheduler and the
// accumulator epilogue.
#pragma once

#include "common.h"

namespace moe {

__device__ __forceinline__ void wait_vmcnt0() {
    // s_waitcnt vmcnt(0) only (expcnt, lgkmcnt left at their maxima)
    __builtin_amdgcn_s_waitcnt(0x0F70);
}

struct Tile {
    int expert;
    int row0;    // first row (absolute, in x_perm) of this tile
    int rows;    // valid rows in the tile (1..BM)
    int row_end; // one past the expert's last row
    int ntile;
    bool valid;
};

// Scan the expert offsets and map blockIdx.x to a tile.  `sh` needs
// kMaxExperts + 2 ints of LDS.  All threads of the workgroup must call this.
template <int BM>
__device__ __forceinline__ Tile find_tile(const int32_t* __restrict__ offsets, int E, int ntn,
                                          int* sh) {
    constexpr int MG = 8;  // M-tiles per group (compact L2 footprint)
    const int tid = threadIdx.x;
    if (tid < 64) {
        // lane handles experts 4*lane .. 4*lane+3
        int mt[4], s = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int e = tid * 4 + j;
            int n = 0;
            if (e < E) n = offsets[e + 1] - offsets[e];
            mt[j] = (n > 0) ? (n + BM - 1) / BM : 0;
            s += mt[j];
        }
        int incl = s;
        for (int d = 1; d < 64; d <<= 1) {
            const int o = __shfl_up(incl, d, 64);
            if (tid >= d) incl += o;
        }
        int run = incl - s;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int e = tid * 4 + j;
            if (e < E) sh[e] = run;  // exclusive prefix P[e]
            run += mt[j];
        }
        if (tid == 63) sh[E] = incl;  // P[E] = total number of M-tiles
    }
    __syncthreads();
    Tile t;
    t.valid = false;
    t.expert = 0; t.row0 = 0; t.rows = 0; t.row_end = 0; t.ntile = 0;
    const int MT = sh[E];
    const long long total = (long long)MT * ntn;
    const long long per = (total + 7) / 8;
    const int xcd = blockIdx.x & 7;
    const long long j = blockIdx.x >> 3;
    const long long L = (long long)xcd * per + j;
    if (j >= per || L >= total) return t;
    const int qm = (int)(L / ntn);
    // the expert whose M-tile range holds qm
    if (tid < E && sh[tid] <= qm && qm < sh[tid + 1]) sh[kMaxExperts + 1] = tid;
    __syncthreads();
    const int e = sh[kMaxExperts + 1];
    const int mt_e = sh[e + 1] - sh[e];
    const int Le = (int)(L - (long long)sh[e] * ntn);
    // the expert's M-tiles are cut into ceil(mt/MG) groups of (nearly) equal size,
    // so that no group is left with a single M-tile (a 1 x 32 block of tiles
    // shares almost nothing in L2)
    const int ng = (mt_e + MG - 1) / MG;
    const int gbase = mt_e / ng, grem = mt_e % ng;   // the first grem groups hold gbase + 1 tiles
    const int big = grem * (gbase + 1) * ntn;        // tiles in those larger groups
    int g, gsz, m_first, rem;
    if (Le < big) {
        gsz = gbase + 1;
        g = Le / (gsz * ntn);
        rem = Le - g * gsz * ntn;
        m_first = g * gsz;
    } else {
        gsz = gbase;
        g = (Le - big) / (gsz * ntn);
        rem = (Le - big) - g * gsz * ntn;
        m_first = grem * (gbase + 1) + g * gsz;
    }
    const int n = rem / gsz;
    const int m = m_first + rem - n * gsz;
    const int lo = offsets[e], hi = offsets[e + 1];
    t.expert = e;
    t.row0 = lo + m * BM;
    t.row_end = hi;
    t.rows = min(BM, hi - t.row0);
    t.ntile = n;
    t.valid = true;
    return t;
}


// Accumulator epilogue of the 32x32x16 MFMA kernels.  The MFMA was issued with
// the weight fragment first, so for fragment (i, j) lane l holds output row
// (l % 32) and columns 8q + 4(l / 32) + 0..3, q = 0..3.  SWIGLU: fragments
// j < FN/2 are the gate, j + FN/2 the matching up projection; h = silu(g) * u.
template <int FM, int FN, int WM, int WN, int BN, bool SWIGLU>
__device__ __forceinline__ void store_tile(f32x16 (&acc)[FM][FN], const Tile& tile,
                                           bf16_t* __restrict__ C, int N, int n0, int wm, int wn,
                                           int lane) {
    const int fr = lane & 31, fk = lane >> 5;
#pragma unroll
    for (int i = 0; i < FM; ++i) {
        const int r = wm * WM + i * 32 + fr;
        if (r >= tile.rows) continue;
        bf16_t* crow = C + (size_t)(tile.row0 + r) * N;
        if (SWIGLU) {
            constexpr int half = FN / 2;
#pragma unroll
            for (int j = 0; j < half; ++j) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int col = n0 + wn * (WN / 2) + j * 32 + 8 * q + 4 * fk;
                    float hv[4];
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const float g = acc[i][j][4 * q + v];
                        const float u = acc[i][j + half][4 * q + v];
                        hv[v] = (g / (1.f + __expf(-g))) * u;
                    }
                    if (col < N) {
                        u32x2 o;
                        o[0] = pack2_bf16(hv[0], hv[1]);
                        o[1] = pack2_bf16(hv[2], hv[3]);
                        *reinterpret_cast<u32x2*>(crow + col) = o;
                    }
                }
            }
        } else {
#pragma unroll
            for (int j = 0; j < FN; ++j) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int col = n0 + wn * WN + j * 32 + 8 * q + 4 * fk;
                    if (col < N) {
                        u32x2 o;
                        o[0] = pack2_bf16(acc[i][j][4 * q + 0], acc[i][j][4 * q + 1]);
                        o[1] = pack2_bf16(acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
                        *reinterpret_cast<u32x2*>(crow + col) = o;
                    }
                }
            }
        }
    }
}

// Static upper bound on the grid: sum_e ceil(n_e / BM) <= R_max / BM + (number
// of non-empty experts), rounded so that each of the 8 XCD shares is whole.
inline int grid_for(int r_max, int E, int BM, int ntn) {
    const long long ub_mt = (long long)r_max / BM + (E < r_max ? E : r_max);
    const long long per = (ub_mt * ntn + 7) / 8;
    return (int)(per * 8);
}


// pipelined MFMA kernels with three activation stages (gemm_pipe3.hip); returns
// false for an unknown variant
bool launch_pipe3_ffn(const void* x_perm, const int32_t* offsets, int r_max, int H, int F, int E,
                      const void* w_gate, const void* w_up, const void* w_down, void* h,
                      void* y_perm, int variant, int phase, hipStream_t s);

// persistent kernels, one workgroup per compute unit (gemm_persist.hip)
bool launch_persist_ffn(const void* x_perm, const int32_t* offsets, int r_max, int H, int F, int E,
                        const void* w_gate, const void* w_up, const void* w_down, void* h,
                        void* y_perm, int variant, int phase, hipStream_t s);

}  // namespace moe
