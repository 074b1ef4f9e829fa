// Pieces shared by the persistent grouped-GEMM kernels (bf16 and FP8): the
// register-resident tile scheduler and small helpers.
#pragma once

#include "gemm_tile.h"

namespace moe {

// workgroups a persistent grouped-GEMM kernel is launched with: one per compute
// unit unless overridden (at least 8, one per tile share)
int persist_grid();

namespace {

// force a wave-uniform value into scalar registers
__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ uint32_t uni(uint32_t v) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)v); }
__device__ __forceinline__ const uint8_t* uni(const uint8_t* p) {
    const uint64_t u = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = uni((uint32_t)u), hi = uni((uint32_t)(u >> 32));
    return reinterpret_cast<const uint8_t*>(((uint64_t)hi << 32) | lo);
}

// wave-uniform description of one output tile
struct PTile {
    const uint8_t* a;   // first activation row of the tile (k = 0)
    const uint8_t* b0;  // first weight row: gate (SwiGLU) or down projection
    const uint8_t* b1;  // first up-projection row (SwiGLU only)
    uint32_t a_lim;     // byte offset (from a) of the last valid activation row
    uint32_t b_lim;     // byte offset (from b0 / b1) of the last valid weight row
    int row0, rows, n0;
    bool valid;
};

// Every wave keeps the whole schedule in registers: lane l describes experts
// 4l .. 4l+3 (first row, row count, exclusive prefix of M-tile counts).
template <int BM>
struct TileSched {
    int lo[4], n[4], pex[4], pend;
    int MT, ntn, per, nwx, wgx, xcd, total;

    __device__ __forceinline__ void init(const int32_t* __restrict__ offsets, int E, int ntn_, int lane) {
        int mt[4], s = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int e = lane * 4 + j;
            lo[j] = 0;
            n[j] = 0;
            if (e < E) {
                lo[j] = offsets[e];
                n[j] = offsets[e + 1] - lo[j];
            }
            mt[j] = (n[j] > 0) ? (n[j] + BM - 1) / BM : 0;
            s += mt[j];
        }
        int incl = s;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int o = __shfl_up(incl, d, 64);
            if (lane >= d) incl += o;
        }
        pex[0] = incl - s;
#pragma unroll
        for (int j = 1; j < 4; ++j) pex[j] = pex[j - 1] + mt[j - 1];
        pend = incl;
        MT = __builtin_amdgcn_readlane(incl, 63);
        ntn = ntn_;
        total = MT * ntn;
        per = (total + 7) / 8;              // tiles per XCD share
        xcd = blockIdx.x & 7;               // workgroups are dealt round-robin to the 8 XCDs
        wgx = blockIdx.x >> 3;
        nwx = (gridDim.x + 7 - xcd) >> 3;   // workgroups of this launch that share the XCD
    }

    // the i-th tile of this workgroup
    // row_bytes: bytes per operand row (contraction length times element size)
    __device__ __forceinline__ PTile get(int i, const uint8_t* A, const uint8_t* B0, const uint8_t* B1, int N,
                                         size_t row_bytes, int outn) const {
        constexpr int MG = 8;
        PTile t;
        t.a = A; t.b0 = B0; t.b1 = B1; t.a_lim = 0; t.b_lim = 0; t.row0 = 0; t.rows = 0; t.n0 = 0;
        const int j = wgx + i * nwx;
        const int L = xcd * per + j;
        t.valid = (j < per) && (L < total);
        if (!t.valid) return t;
        const int qm = L / ntn;
        int hit = -1, my_p = 0, my_end = 0, my_lo = 0, my_n = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int end = (q < 3) ? pex[q + 1] : pend;
            if (pex[q] <= qm && qm < end) {
                hit = q; my_p = pex[q]; my_end = end; my_lo = lo[q]; my_n = n[q];
            }
        }
        const uint64_t bal = __ballot(hit >= 0);  // exactly one lane: the M-tile ranges partition [0, MT)
        const int src = __builtin_amdgcn_readfirstlane(__ffsll((unsigned long long)bal) - 1);
        const int e = 4 * src + __builtin_amdgcn_readlane(hit, src);
        const int p_e = __builtin_amdgcn_readlane(my_p, src);
        const int mt_e = __builtin_amdgcn_readlane(my_end, src) - p_e;
        const int lo_e = __builtin_amdgcn_readlane(my_lo, src);
        const int n_e = __builtin_amdgcn_readlane(my_n, src);
        // inside an expert: ceil(mt/MG) groups of near-equal size, tiles ordered
        // (M-group, N, M-in-group) so that concurrently running tiles share panels in L2
        const int Le = L - p_e * ntn;
        const int ng = (mt_e + MG - 1) / MG;
        const int gbase = mt_e / ng, grem = mt_e % ng;
        const int big = grem * (gbase + 1) * ntn;
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
        const int nt = rem / gsz;
        const int m = m_first + rem - nt * gsz;
        t.row0 = uni(lo_e + m * BM);
        t.rows = uni(min(BM, lo_e + n_e - t.row0));
        t.n0 = uni(nt * outn);
        const size_t k2 = row_bytes;
        t.a = uni(A + (size_t)t.row0 * k2);
        const size_t brow = ((size_t)e * N + t.n0) * k2;
        t.b0 = uni(B0 + brow);
        t.b1 = uni(B1 + brow);
        t.a_lim = uni((uint32_t)(t.rows - 1) * (uint32_t)k2);
        t.b_lim = uni((uint32_t)(min(outn, N - t.n0) - 1) * (uint32_t)k2);
        return t;
    }
};

}  // namespace

}  // namespace moe
