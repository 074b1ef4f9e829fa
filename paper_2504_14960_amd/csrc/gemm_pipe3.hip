// Grouped expert GEMM (a3), pipelined kernel with uneven LDS staging: three
// stages for the activation tile, two for the weight tile (3 x 32 KiB + 2 x
// 32 KiB = all 160 KiB of a CU's LDS for a 256 x 256 x 64 tile).
//
// Why: the direct global->LDS path of one CU moves ~40-50 B/clk, and a 256x256
// tile needs 64 KiB per 64-wide k-tile, so that path is busy for most of a
// k-tile.  With two stages for both operands every load of tile t+1 has to
// have landed by the single barrier of tile t, and the waves queue up behind
// the texture unit there.  Here only the weight tile of t+1 (issued first in
// each period) has to be complete at the barrier; the activation tile fetched
// in the same period is the one for t+2 and gets a whole extra period to land
// (`s_waitcnt vmcnt(PA)` leaves exactly those loads in flight).
//
// Everything else (XOR-swizzled 128-byte LDS rows, 32x32x16 bf16 MFMA with
// the weight fragment first, fragment double buffering, source-ordered
// interleave frozen by scheduling barriers, ragged tile scheduler, fused
// SwiGLU epilogue) is shared with the persistent kernel in gemm_persist.hip,
// which is this engine without the per-tile prologue and with a coalesced
// epilogue; this file is the one-workgroup-per-tile form of it.
#include "gemm_tile.h"

namespace moe {


namespace {

// GROUPK = false: the forward's grouped GEMM, rows grouped by expert (ragged M),
// one contraction length K for all.
// GROUPK = true: the weight-gradient form.  C [E, M, N] = for every expert e,
// A[:, seg_e] . B[:, seg_e]^T, where A [M, ld] and B [N, ld] hold transposed
// activations whose columns are grouped by expert: segment e starts at the sum of
// the padded lengths of the experts before it and is padded with zeros to
// padded(n_e) = max(128, n_e rounded up to 64) columns (0 for an empty expert).
// One workgroup per (expert, M-tile, N-tile); its contraction runs over the
// expert's segment only; `K` carries ld, `ntn` the N-tile count, `M` the rows.
template <int BM, int BN, int WGM, int WGN, bool SWIGLU, bool GROUPK = false>
__global__ __launch_bounds__(WGM* WGN * 64) void gemm_bf16_pipe3_kernel(
    const bf16_t* __restrict__ A, const int32_t* __restrict__ offsets, int E, int N, int K,
    const bf16_t* __restrict__ B0, const bf16_t* __restrict__ B1, bf16_t* __restrict__ C, int ntn, int M) {
    constexpr int BK = 64;
    constexpr int NT = WGM * WGN * 64;
    constexpr int WM = BM / WGM, WN = BN / WGN;
    constexpr int FM = WM / 32, FN = WN / 32;
    constexpr int CPR = BK / 8;
    constexpr int RPP = NT / CPR;
    constexpr int PA = BM / RPP, PB = BN / RPP;
    constexpr int ROWB = BK * 2;
    constexpr int A_BYTES = BM * ROWB, B_BYTES = BN * ROWB;
    // three activation slots (the "late" operand, fetched two k-tiles ahead) and
    // two weight slots (the "early" operand that must be complete at the barrier)
    constexpr bool TRI_B = false;                // true would swap the roles of the operands
    constexpr int A_SLOTS = 3, B_SLOTS = 2;
    constexpr int B_REGION = A_SLOTS * A_BYTES;  // B slots start after the A slots
    constexpr int PE = PB;                       // passes of the early (2-slot) operand
    constexpr int PL = PA;                       // passes of the late (3-slot) operand
    constexpr int E_BYTES = B_BYTES, L_BYTES = A_BYTES;
    constexpr int OUTN = SWIGLU ? BN / 2 : BN;
    constexpr int NLOAD = PA + PB;             // direct loads per thread per period
    constexpr int NREAD = FM + FN;
    constexpr int NMFMA = FM * FN;
    constexpr int NSLOT = NREAD;
    constexpr int MPS = NMFMA / NSLOT;
    // a period's NLOAD loads (weight tile first) go in thirds under the k-steps
    // 3 (of the previous tile), 0 and 1, one per slot
    constexpr int LA = NLOAD / 3;                  // under k-step 3 (previous tile)
    constexpr int LB = LA + (NLOAD - LA + 1) / 2;  // end of k-step 0's share
    constexpr int LC = NLOAD;                      // end of k-step 1's share
    constexpr int LSTRIDE = 1;                     // slots between two loads
    static_assert(BM % RPP == 0 && BN % RPP == 0, "tile rows must divide into fetch passes");
    static_assert(!SWIGLU || ((BN / 2) % RPP == 0 && FN % 2 == 0), "gate/up halves must be pass- and fragment-aligned");
    static_assert(LA <= PE, "only early-operand loads may be issued under k-step 3");
    static_assert(LSTRIDE >= 1 && (LB - LA) * LSTRIDE <= NSLOT && (LC - LB) * LSTRIDE <= NSLOT &&
                      (NLOAD - LC) * LSTRIDE <= NSLOT && LA * LSTRIDE <= NSLOT, "not enough slots for the loads");
    static_assert(PL < 64, "vmcnt holds 6 bits");
    static_assert(A_SLOTS * A_BYTES + B_SLOTS * B_BYTES <= 160 * 1024, "tile stages exceed the 160 KiB of LDS");

    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
    // the tile scheduler's scratch lives in the second weight slot, which is not
    // written before the prologue's barrier
    int* sched = reinterpret_cast<int*>(smem + (TRI_B ? A_BYTES : B_REGION + B_BYTES));  // second early slot

    Tile tile;
    int seg_off = 0, seg_len = 0;   // GROUPK: the expert's column segment
    if constexpr (GROUPK) {
        static_assert(!SWIGLU, "the weight-gradient form has one B operand");
        (void)sched;
        const int mt = (M + BM - 1) / BM;
        const int per_e = mt * ntn;
        const int e = blockIdx.x / per_e, rem = blockIdx.x - e * per_e;
        const int nt = rem / mt, m = rem - nt * mt;   // M-tiles of one weight panel are neighbours
        tile.valid = e < E;
        if (!tile.valid) return;
        for (int q = 0; q <= e; ++q) {   // wave-uniform, E <= 256 short iterations
            const int n_q = offsets[q + 1] - offsets[q];
            const int pn = n_q <= 0 ? 0 : max(128, (n_q + 63) & ~63);
            if (q < e) seg_off += pn; else seg_len = pn;
        }
        tile.expert = e;
        tile.row0 = e * M + m * BM;          // row of C
        tile.rows = min(BM, M - m * BM);
        tile.row_end = (e + 1) * M;
        tile.ntile = nt;
    } else {
        tile = find_tile<BM>(offsets, E, ntn, sched);
        if (!tile.valid) return;
    }

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WGN, wn = wave % WGN;
    const int n0 = tile.ntile * OUTN;

    const int frow = tid / CPR, fchunk = tid % CPR;
    const uint8_t* a_base = GROUPK
        ? reinterpret_cast<const uint8_t*>(A + (size_t)(tile.row0 - tile.expert * M) * K + seg_off)
        : reinterpret_cast<const uint8_t*>(A + (size_t)tile.row0 * K);
    const size_t b_row0 = GROUPK ? (size_t)n0 * K + seg_off : ((size_t)tile.expert * N + n0) * K;
    const uint8_t* b_base0 = reinterpret_cast<const uint8_t*>(B0 + b_row0);
    const uint8_t* b_base1 = SWIGLU ? reinterpret_cast<const uint8_t*>(B1 + b_row0) : b_base0;
    uint32_t a_goff[PA], b_goff[PB];
#pragma unroll
    for (int p = 0; p < PA; ++p) {
        const int r = p * RPP + frow;
        const int rr = min(r, tile.rows - 1);  // ragged tail: re-read a valid row, result discarded
        a_goff[p] = (uint32_t)rr * (uint32_t)K * 2u + (uint32_t)((fchunk ^ lds_swizzle(r)) * 16);
    }
#pragma unroll
    for (int p = 0; p < PB; ++p) {
        const int r = p * RPP + frow;
        int f = SWIGLU ? (r % (BN / 2)) : r;
        f = min(f, N - 1 - n0);
        b_goff[p] = (uint32_t)f * (uint32_t)K * 2u + (uint32_t)((fchunk ^ lds_swizzle(r)) * 16);
    }
    const int wbase = (wave * 64 / CPR) * ROWB;

    auto fetch_a = [&](int p, int kbyte, uint8_t* st) {
        __builtin_amdgcn_global_load_lds(
            (const __attribute__((address_space(1))) void*)(a_base + kbyte + a_goff[p]),
            (__attribute__((address_space(3))) void*)(st + p * RPP * ROWB + wbase), 16, 0, 0);
    };
    auto fetch_b = [&](int p, int kbyte, uint8_t* st) {
        const uint8_t* base = (SWIGLU && p >= PB / 2) ? b_base1 : b_base0;
        __builtin_amdgcn_global_load_lds(
            (const __attribute__((address_space(1))) void*)(base + kbyte + b_goff[p]),
            (__attribute__((address_space(3))) void*)(st + p * RPP * ROWB + wbase), 16, 0, 0);
    };
    // load i of a period: i < PE -> pass i of the early operand (k offset kb_e,
    // slot ld_e), else pass i-PE of the late operand (k offset kb_l, slot ld_l)
    auto fetch_one = [&](int i, int kb_e, int kb_l, uint8_t* ld_e, uint8_t* ld_l) {
        if (i < PE) {
            if (TRI_B) fetch_a(i, kb_e, ld_e); else fetch_b(i, kb_e, ld_e);
        } else {
            if (TRI_B) fetch_b(i - PE, kb_l, ld_l); else fetch_a(i - PE, kb_l, ld_l);
        }
    };

    const int fr = lane & 31, fk = lane >> 5;
    int a_off[FM], b_off[FN], a_sw[FM], b_sw[FN];
#pragma unroll
    for (int i = 0; i < FM; ++i) {
        const int r = wm * WM + i * 32 + fr;
        a_off[i] = r * ROWB;
        a_sw[i] = lds_swizzle(r);
    }
#pragma unroll
    for (int j = 0; j < FN; ++j) {
        int r;
        if (SWIGLU) {
            constexpr int half = FN / 2;
            r = (j < half) ? (wn * (WN / 2) + j * 32 + fr) : (BN / 2 + wn * (WN / 2) + (j - half) * 32 + fr);
        } else {
            r = wn * WN + j * 32 + fr;
        }
        b_off[j] = r * ROWB;
        b_sw[j] = lds_swizzle(r);
    }

    f32x16 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    bf16x8 af[2][FM], bfg[2][FN];
    auto read_one = [&](const uint8_t* sa, const uint8_t* sb, int s, int buf, int q) {
        const int c = 2 * s + fk;
        if (q < FM)
            af[buf][q] = __builtin_bit_cast(
                bf16x8, *reinterpret_cast<const u32x4*>(sa + a_off[q] + ((c ^ a_sw[q]) << 4)));
        else
            bfg[buf][q - FM] = __builtin_bit_cast(
                bf16x8, *reinterpret_cast<const u32x4*>(sb + b_off[q - FM] + ((c ^ b_sw[q - FM]) << 4)));
    };
    auto mfma_one = [&](int buf, int m) {
        const int i = m / FN, j = m % FN;
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfg[buf][j], af[buf][i], acc[i][j], 0, 0, 0);
    };
    // one k-step in issue order: NSLOT slots of {MPS MFMAs on set mf_buf; up to
    // 2 fragment reads of k-step rd_s into the other set; one direct load}
    auto kstep = [&](int mf_buf, const uint8_t* rd_a, const uint8_t* rd_b, int rd_s, int ld_begin, int ld_end,
                     int kb_b, int kb_a, uint8_t* ld_b, uint8_t* ld_a) {
        int m = 0, rd = 0, ld = ld_begin;
#pragma unroll
        for (int slot = 0; slot < NSLOT; ++slot) {
#pragma unroll
            for (int q = 0; q < MPS; ++q) {
                mfma_one(mf_buf, m);
                ++m;
            }
            // the first MFMA waits for the previous k-step's fragment reads only: keep the new reads behind it
            if (slot == 0) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int q = 0; q < 2; ++q)
                if (rd < NREAD) {
                    read_one(rd_a, rd_b, rd_s, mf_buf ^ 1, rd);
                    ++rd;
                }
            if (slot % LSTRIDE == 0 && ld < ld_end) {
                fetch_one(ld, kb_b, kb_a, ld_b, ld_a);
                ++ld;
            }
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int mm = NSLOT * MPS; mm < NMFMA; ++mm) mfma_one(mf_buf, mm);
        __builtin_amdgcn_sched_barrier(0);
    };

    const int KT = GROUPK ? seg_len / BK : K / BK;
    if (GROUPK && KT == 0) {
        // an expert without rows: its weight gradient is zero
        store_tile<FM, FN, WM, WN, BN, SWIGLU>(acc, tile, C, N, n0, wm, wn, lane);
        return;
    }
    auto kb = [&](int kt) { return min(kt, KT - 1) * (BK * 2); };  // past the end: the last tile again, never used
    uint8_t* const e_region = smem + (TRI_B ? 0 : B_REGION);   // early operand: 2 slots
    uint8_t* const l_region = smem + (TRI_B ? B_REGION : 0);   // late operand: 3 slots
    auto a_ptr = [&](int e_off, int l_off) -> const uint8_t* { return TRI_B ? e_region + e_off : l_region + l_off; };
    auto b_ptr = [&](int e_off, int l_off) -> const uint8_t* { return TRI_B ? l_region + l_off : e_region + e_off; };

    // prologue: late(0), early(0), then late(1); only the first two must have landed
#pragma unroll
    for (int i = PE; i < NLOAD; ++i) fetch_one(i, 0, kb(0), e_region, l_region);
#pragma unroll
    for (int i = 0; i < PE; ++i) fetch_one(i, kb(0), 0, e_region, l_region);
#pragma unroll
    for (int i = PE; i < NLOAD; ++i) fetch_one(i, 0, kb(1), e_region, l_region + L_BYTES);
    __builtin_amdgcn_s_waitcnt(0x0F70 | (PL & 0xF) | ((PL >> 4) << 14));  // vmcnt(PL)
    __syncthreads();
#pragma unroll
    for (int q = 0; q < NREAD; ++q) read_one(a_ptr(0, 0), b_ptr(0, 0), 0, 0, q);
    // first loads of period 0: the head of early(1) into early slot 1
#pragma unroll
    for (int i = 0; i < LA; ++i) fetch_one(i, kb(1), 0, e_region + E_BYTES, l_region);

    int l0 = 0, l1 = L_BYTES, l2 = 2 * L_BYTES;  // late-operand slots of tiles kt, kt+1, kt+2
    int e0 = 0, e1 = E_BYTES;                    // early-operand slots of tiles kt, kt+1
    for (int kt = 0; kt < KT; ++kt) {
        const uint8_t* ca = a_ptr(e0, l0);
        const uint8_t* cb = b_ptr(e0, l0);
        uint8_t* le = e_region + e1;  // early(kt+1)
        uint8_t* ll = l_region + l2;  // late(kt+2)
        const int kbe = kb(kt + 1), kbl = kb(kt + 2);
        __builtin_amdgcn_sched_barrier(0);
        kstep(0, ca, cb, 1, LA, LB, kbe, kbl, le, ll);     // k-step 0
        kstep(1, ca, cb, 2, LB, LC, kbe, kbl, le, ll);     // k-step 1
        kstep(0, ca, cb, 3, LC, NLOAD, kbe, kbl, le, ll);  // k-step 2
        // early(kt+1) was issued before late(kt+2) in this period and late(kt+1) a
        // period ago: all but the PL youngest loads must have landed; this wave's
        // reads of tile kt are in registers (lgkmcnt(0))
        __builtin_amdgcn_s_waitcnt((PL & 0xF) | ((PL >> 4) << 14));
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        // k-step 3: first fragments of tile kt+1; tile kt's early slot is free,
        // the head of early(kt+2) goes into it
        kstep(1, a_ptr(e1, l1), b_ptr(e1, l1), 0, 0, LA, kb(kt + 2), 0, e_region + e0, l_region);
        const int tl = l0;
        l0 = l1;
        l1 = l2;
        l2 = tl;
        const int te = e0;
        e0 = e1;
        e1 = te;
    }
    wait_vmcnt0();  // loads past the end of K may still be landing in LDS
    store_tile<FM, FN, WM, WN, BN, SWIGLU>(acc, tile, C, N, n0, wm, wn, lane);
}

template <int BM, int BN, int WGM, int WGN, bool SWIGLU>
void launch_pipe3(const void* A, const int32_t* offsets, int r_max, int E, int N, int K, const void* B0,
                  const void* B1, void* C, hipStream_t s) {
    constexpr int OUTN = SWIGLU ? BN / 2 : BN;
    constexpr size_t smem = (size_t)(3 * BM + 2 * BN) * 64 * 2;
    const int ntn = (N + OUTN - 1) / OUTN;
    auto kern = gemm_bf16_pipe3_kernel<BM, BN, WGM, WGN, SWIGLU, false>;
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        attr_set = true;
    }
    const int grid = grid_for(r_max, E, BM, ntn);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(WGM * WGN * 64), smem, s, static_cast<const bf16_t*>(A),
                       offsets, E, N, K, static_cast<const bf16_t*>(B0),
                       static_cast<const bf16_t*>(B1), static_cast<bf16_t*>(C), ntn, 0);
}

// weight-gradient form: C [E, M, N] from A [M, ld] and B [N, ld] (see the kernel)
template <int BM, int BN, int WGM, int WGN>
void launch_pipe3_groupk(const void* A, const void* B, const int32_t* offsets, int E, int M, int N, int ld,
                         void* C, hipStream_t s) {
    constexpr size_t smem = (size_t)(3 * BM + 2 * BN) * 64 * 2;
    const int ntn = (N + BN - 1) / BN, mt = (M + BM - 1) / BM;
    auto kern = gemm_bf16_pipe3_kernel<BM, BN, WGM, WGN, false, true>;
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        attr_set = true;
    }
    hipLaunchKernelGGL(kern, dim3(E * mt * ntn), dim3(WGM * WGN * 64), smem, s, static_cast<const bf16_t*>(A),
                       offsets, E, N, ld, static_cast<const bf16_t*>(B), static_cast<const bf16_t*>(B),
                       static_cast<bf16_t*>(C), ntn, M);
}

template <int BM, int BN, int WGM, int WGN>
void run_pipe3_pair(const void* x_perm, const int32_t* offsets, int r_max, int H, int F, int E,
                    const void* w_gate, const void* w_up, const void* w_down, void* h, void* y_perm,
                    int phase, hipStream_t s) {
    if (phase & 1) launch_pipe3<BM, BN, WGM, WGN, true>(x_perm, offsets, r_max, E, F, H, w_gate, w_up, h, s);
    if (phase & 2) launch_pipe3<BM, BN, WGM, WGN, false>(h, offsets, r_max, E, H, F, w_down, nullptr, y_perm, s);
}

}  // namespace

void launch_pipe3_wgrad(const void* a_t, const void* b_t, const int32_t* offsets, int E, int M, int N, int ld,
                        void* dw, hipStream_t s) {
    launch_pipe3_groupk<256, 256, 2, 4>(a_t, b_t, offsets, E, M, N, ld, dw, s);
}

bool launch_pipe3_ffn(const void* x_perm, const int32_t* offsets, int r_max, int H, int F, int E,
                      const void* w_gate, const void* w_up, const void* w_down, void* h,
                      void* y_perm, int variant, int phase, hipStream_t s) {
    switch (variant) {
        case 30: run_pipe3_pair<256, 256, 2, 2>(x_perm, offsets, r_max, H, F, E, w_gate, w_up, w_down, h, y_perm, phase, s); return true;
        case 31: run_pipe3_pair<256, 256, 2, 4>(x_perm, offsets, r_max, H, F, E, w_gate, w_up, w_down, h, y_perm, phase, s); return true;
        default: return false;
    }
}

}  // namespace moe
