// Pieces shared by the persistent grouped-GEMM kernels (bf16 and FP8): the
// register-resident tile scheduler and small helpers.
#pragma once

#include "gemm_tile.h"

namespace moe {

// workgroups a persistent grouped-GEMM kernel is launched with: one per compute
// unit unless overridden (at least 8, one per tile share)
int persist_grid();
// whether a launch over E experts uses the kernels whose waves without valid rows skip the multiplications
bool persist_idle_skip(int E);

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
    int kt;             // k-tiles of this output tile (weight-gradient form; 0 = the launch's common count)
    int krows;          // row-major weight-gradient form: rows of the expert, i.e. valid length of the contraction
    bool valid;
};

// Every wave keeps the whole schedule in registers: lane l describes experts
// 4l .. 4l+3 (first row, row count, exclusive prefix of M-tile counts).
template <int BM, bool BY_ROUND = true>
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
        t.a = A; t.b0 = B0; t.b1 = B1; t.a_lim = 0; t.b_lim = 0; t.row0 = 0; t.rows = 0; t.n0 = 0; t.kt = 0; t.krows = 0;
        // BY_ROUND: whole rounds (one tile per workgroup of the launch) are dealt to the XCDs round by round: in
        // round i XCD x runs the nwx consecutive tiles from (8 i + x) nwx on, so at any time the eight XCDs work on
        // neighbouring stretches of the list and what they have in common (activation panels of one M-group) is
        // fetched from memory once and found in the memory-side cache by the others.  The tiles left over after
        // the last whole round are cut into eight contiguous shares.  Otherwise every XCD takes a contiguous
        // eighth of the list.
        int L;
        if (BY_ROUND && (gridDim.x & 7) == 0) {
            const int round_tiles = 8 * nwx, whole = total / round_tiles;
            if (i < whole) {
                L = (i * 8 + xcd) * nwx + wgx;
                t.valid = true;
            } else {
                const int left = total - whole * round_tiles, share = (left + 7) >> 3;
                const int j = wgx + (i - whole) * nwx;
                L = whole * round_tiles + xcd * share + j;
                t.valid = (j < share) && (L < total);
            }
        } else {
            const int j = wgx + i * nwx;
            L = xcd * per + j;
            t.valid = (j < per) && (L < total);
        }
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

// Schedule of the weight-gradient form: C [E, M, N], for expert e the product of
// A_t[:, seg_e] and B_t[:, seg_e]^T over the expert's zero-padded column segment
// (padded length = 0 for an expert without rows, else max(128, n rounded up to
// 64)).  Every non-empty expert has the same mt x nt output tiles; what differs
// from tile to tile is the number of k-tiles, so the XCD shares are cut by work,
// not by tile count: every XCD takes the same eighth of EVERY expert's tiles (a
// contiguous block of the expert's tile order, so the tiles an XCD runs at once
// still share panels in its L2), and its workgroups walk that list round-robin.
// Lane l describes experts 4l..4l+3.
template <int BM, int BN>
struct WgradSched {
    int seg[4], len[4], pex[4], pend;   // segment start / padded length (elements), prefix of non-empty experts
    int mt, nt, tpe, nwx, wgx, part0, part_n, total;   // part0/part_n: this XCD's slice of an expert's tiles

    __device__ __forceinline__ void init(const int32_t* __restrict__ offsets, int E, int M, int N, int lane) {
        int s_len = 0, s_cnt = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int e = lane * 4 + j;
            int n = 0;
            if (e < E) n = offsets[e + 1] - offsets[e];
            len[j] = n <= 0 ? 0 : max(128, (n + 63) & ~63);
            s_len += len[j];
            s_cnt += len[j] > 0;
        }
        int incl_len = s_len, incl_cnt = s_cnt;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int ol = __shfl_up(incl_len, d, 64), oc = __shfl_up(incl_cnt, d, 64);
            if (lane >= d) {
                incl_len += ol;
                incl_cnt += oc;
            }
        }
        seg[0] = incl_len - s_len;
        pex[0] = incl_cnt - s_cnt;
#pragma unroll
        for (int j = 1; j < 4; ++j) {
            seg[j] = seg[j - 1] + len[j - 1];
            pex[j] = pex[j - 1] + (len[j - 1] > 0);
        }
        pend = incl_cnt;
        mt = (M + BM - 1) / BM;
        nt = (N + BN - 1) / BN;
        tpe = mt * nt;
        const int xcd = blockIdx.x & 7;
        part0 = (int)((long long)xcd * tpe / 8);
        part_n = (int)((long long)(xcd + 1) * tpe / 8) - part0;
        total = __builtin_amdgcn_readlane(incl_cnt, 63) * part_n;   // tiles of this XCD
        wgx = blockIdx.x >> 3;
        nwx = (gridDim.x + 7 - xcd) >> 3;
    }

    // the i-th tile of this workgroup; ld = elements per row of A_t and B_t
    __device__ __forceinline__ PTile get(int i, const uint8_t* A, const uint8_t* B, int M, int N, int ld) const {
        constexpr int MG = 8;
        PTile t;
        t.a = A; t.b0 = B; t.b1 = B; t.a_lim = 0; t.b_lim = 0; t.row0 = 0; t.rows = 0; t.n0 = 0; t.kt = 0; t.krows = 0;
        const int j = wgx + i * nwx;
        t.valid = j < total;
        if (!t.valid) return t;
        const int qe = j / part_n;   // index among the non-empty experts (part_n > 0 since total > 0)
        int hit = -1, my_seg = 0, my_len = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q)
            if (len[q] > 0 && pex[q] == qe) {
                hit = q; my_seg = seg[q]; my_len = len[q];
            }
        const uint64_t bal = __ballot(hit >= 0);  // exactly one lane holds the qe-th non-empty expert
        const int src = __builtin_amdgcn_readfirstlane(__ffsll((unsigned long long)bal) - 1);
        const int e = 4 * src + __builtin_amdgcn_readlane(hit, src);
        const int seg_e = __builtin_amdgcn_readlane(my_seg, src);
        const int len_e = __builtin_amdgcn_readlane(my_len, src);
        // inside an expert: groups of MG M-tiles, ordered (M-group, N, M-in-group)
        const int Le = part0 + j - qe * part_n;
        const int full = (mt / MG) * MG * nt;
        int m, n;
        if (Le < full) {
            const int g = Le / (MG * nt), rem = Le - g * MG * nt;
            n = rem / MG;
            m = g * MG + rem - n * MG;
        } else {
            const int tail = mt % MG, rem = Le - full;   // tail > 0 here
            n = rem / tail;
            m = (mt / MG) * MG + rem - n * tail;
        }
        const size_t k2 = (size_t)ld * 2;
        t.rows = uni(min(BM, M - m * BM));
        t.row0 = uni(e * M + m * BM);
        t.n0 = uni(n * BN);
        t.kt = uni(len_e / 64);
        t.a = uni(A + (size_t)(m * BM) * k2 + (size_t)seg_e * 2);
        t.b0 = uni(B + (size_t)(n * BN) * k2 + (size_t)seg_e * 2);
        t.b1 = t.b0;
        t.a_lim = uni((uint32_t)(t.rows - 1) * (uint32_t)k2);
        t.b_lim = uni((uint32_t)(min(BN, N - t.n0) - 1) * (uint32_t)k2);
        return t;
    }
};

// Schedule of the weight-gradient form on ROW-MAJOR activations: C [E, M, N], for expert e the product
// A[rows_e, :]^T B[rows_e, :] with A [rows, lda] and B [rows, ldb] as the layer holds them (rows grouped by expert).
// The contraction runs over the expert's rows in k-tiles of 64 rows; rows past the expert's last one are read from a
// zero row by the kernel.  Tile order and XCD shares as in WgradSched.  Every tile gets at least two k-tiles (the
// k stream needs them; the second of a short expert is all zero rows).  Lane l describes experts 4l .. 4l+3.
template <int BM, int BN>
struct WgradSchedKM {
    int lo[4], n[4], pex[4], pend;
    int mt, nt, tpe, nwx, wgx, part0, part_n, total;

    __device__ __forceinline__ void init(const int32_t* __restrict__ offsets, int E, int M, int N, int lane) {
        int s_cnt = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int e = lane * 4 + j;
            lo[j] = 0;
            n[j] = 0;
            if (e < E) {
                lo[j] = offsets[e];
                n[j] = max(0, offsets[e + 1] - lo[j]);
            }
            s_cnt += n[j] > 0;
        }
        int incl_cnt = s_cnt;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int oc = __shfl_up(incl_cnt, d, 64);
            if (lane >= d) incl_cnt += oc;
        }
        pex[0] = incl_cnt - s_cnt;
#pragma unroll
        for (int j = 1; j < 4; ++j) pex[j] = pex[j - 1] + (n[j - 1] > 0);
        pend = incl_cnt;
        mt = (M + BM - 1) / BM;
        nt = (N + BN - 1) / BN;
        tpe = mt * nt;
        const int xcd = blockIdx.x & 7;
        part0 = (int)((long long)xcd * tpe / 8);
        part_n = (int)((long long)(xcd + 1) * tpe / 8) - part0;
        total = __builtin_amdgcn_readlane(incl_cnt, 63) * part_n;
        wgx = blockIdx.x >> 3;
        nwx = (gridDim.x + 7 - xcd) >> 3;
    }

    // lda, ldb: elements per row of A and B
    __device__ __forceinline__ PTile get(int i, const uint8_t* A, const uint8_t* B, int M, int N, int lda,
                                         int ldb) const {
        constexpr int MG = 8;
        PTile t;
        t.a = A; t.b0 = B; t.b1 = B; t.a_lim = 0; t.b_lim = 0; t.row0 = 0; t.rows = 0; t.n0 = 0; t.kt = 0; t.krows = 0;
        const int j = wgx + i * nwx;
        t.valid = j < total;
        if (!t.valid) return t;
        const int qe = j / part_n;
        int hit = -1, my_lo = 0, my_n = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q)
            if (n[q] > 0 && pex[q] == qe) {
                hit = q; my_lo = lo[q]; my_n = n[q];
            }
        const uint64_t bal = __ballot(hit >= 0);
        const int src = __builtin_amdgcn_readfirstlane(__ffsll((unsigned long long)bal) - 1);
        const int e = 4 * src + __builtin_amdgcn_readlane(hit, src);
        const int lo_e = __builtin_amdgcn_readlane(my_lo, src);
        const int n_e = __builtin_amdgcn_readlane(my_n, src);
        const int Le = part0 + j - qe * part_n;
        const int full = (mt / MG) * MG * nt;
        int m, nn;
        if (Le < full) {
            const int g = Le / (MG * nt), rem = Le - g * MG * nt;
            nn = rem / MG;
            m = g * MG + rem - nn * MG;
        } else {
            const int tail = mt % MG, rem = Le - full;
            nn = rem / tail;
            m = (mt / MG) * MG + rem - nn * tail;
        }
        t.rows = uni(min(BM, M - m * BM));
        t.row0 = uni(e * M + m * BM);
        t.n0 = uni(nn * BN);
        t.krows = uni(n_e);
        t.kt = uni(max(2, (n_e + 63) / 64));
        t.a = uni(A + ((size_t)lo_e * lda + (size_t)m * BM) * 2);
        t.b0 = uni(B + ((size_t)lo_e * ldb + (size_t)t.n0) * 2);
        t.b1 = t.b0;
        // last 16-byte piece of a tile row that still lies inside the matrix row
        t.a_lim = uni((uint32_t)(t.rows * 2 - 16));
        t.b_lim = uni((uint32_t)(min(BN, N - t.n0) * 2 - 16));
        return t;
    }
};

}  // namespace

}  // namespace moe
