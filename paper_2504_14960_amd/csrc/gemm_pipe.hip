// Software-pipelined bf16 MFMA kernel of the grouped expert GEMMs (a3).
//
// Same tiling, LDS layout, scheduler and epilogue as gemm_bf16_kernel, but the
// main loop is laid out by hand so that one wave keeps the matrix pipe busy on
// its own:
//   * tiles arrive with direct global->LDS loads (no staging registers), two
//     LDS stages, ONE workgroup barrier per 64-wide k-tile;
//   * the 16-byte operand fragments of k-step s+1 are read from LDS while the
//     MFMAs of k-step s run (two fragment register sets);
//   * the barrier sits before the last k-step of a tile, so the first
//     fragments of the next tile are read under that k-step's MFMAs;
//   * the interleave (n MFMAs : 1 LDS read : 1-2 direct loads) is written out
//     in program order and frozen with scheduling barriers.
// Global addresses are a wave-uniform base plus a 32-bit per-lane offset that
// is fixed for the whole K loop.
#include "gemm_tile.h"

namespace moe {

#ifdef MOE_PIPE_TIMING
// instrumentation build only: per-wave tick counters {loop, load wait, barrier wait}
__device__ unsigned long long g_pipe_ticks[4096 * 8 * 4];
#endif

namespace {

template <int BM, int BN, int WGM, int WGN, bool SWIGLU, int LMODE>
__global__ __launch_bounds__(WGM* WGN * 64) void gemm_bf16_pipe_kernel(
    const bf16_t* __restrict__ A, const int32_t* __restrict__ offsets, int E, int N, int K,
    const bf16_t* __restrict__ B0, const bf16_t* __restrict__ B1, bf16_t* __restrict__ C, int ntn) {
    constexpr int BK = 64;
    constexpr int NT = WGM * WGN * 64;
    constexpr int WM = BM / WGM, WN = BN / WGN;
    constexpr int FM = WM / 32, FN = WN / 32;
    constexpr int CPR = BK / 8;
    constexpr int RPP = NT / CPR;
    constexpr int PA = BM / RPP, PB = BN / RPP;
    constexpr int KS = BK / 16;
    constexpr int ROWB = BK * 2;
    constexpr int A_BYTES = BM * ROWB, B_BYTES = BN * ROWB;
    constexpr int STAGE = A_BYTES + B_BYTES;
    constexpr int OUTN = SWIGLU ? BN / 2 : BN;
    constexpr int NLOAD = PA + PB;           // direct loads per thread per k-tile
    constexpr int NREAD = FM + FN;           // fragment reads per k-step
    constexpr int NMFMA = FM * FN;           // MFMAs per k-step
    static_assert(BM % RPP == 0 && BN % RPP == 0, "tile rows must divide into fetch passes");
    static_assert(!SWIGLU || ((BN / 2) % RPP == 0 && FN % 2 == 0), "gate/up halves must be pass- and fragment-aligned");
    static_assert(KS == 4, "pipeline written for four k-steps per tile");

    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
    __shared__ int sched[kMaxExperts + 2];

    const Tile tile = find_tile<BM>(offsets, E, ntn, sched);
    if (!tile.valid) return;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform, keep it scalar
    const int wm = wave / WGN, wn = wave % WGN;
    const int n0 = tile.ntile * OUTN;

    // ---- fetch slots: uniform bases + per-lane 32-bit byte offsets ----
    const int frow = tid / CPR, fchunk = tid % CPR;
    const uint8_t* a_base = reinterpret_cast<const uint8_t*>(A + (size_t)tile.row0 * K);
    const size_t b_row0 = ((size_t)tile.expert * N + n0) * K;
    const uint8_t* b_base0 = reinterpret_cast<const uint8_t*>(B0 + b_row0);
    const uint8_t* b_base1 = SWIGLU ? reinterpret_cast<const uint8_t*>(B1 + b_row0) : b_base0;
    uint32_t a_goff[PA], b_goff[PB];
#pragma unroll
    for (int p = 0; p < PA; ++p) {
        const int r = p * RPP + frow;
        const int rr = min(r, tile.rows - 1);  // ragged tail: re-read a valid row, result discarded
        a_goff[p] = (uint32_t)rr * (uint32_t)K * 2u + (uint32_t)((fchunk ^ (r & 7)) * 16);
    }
#pragma unroll
    for (int p = 0; p < PB; ++p) {
        const int r = p * RPP + frow;
        int f = SWIGLU ? (r % (BN / 2)) : r;
        f = min(f, N - 1 - n0);
        b_goff[p] = (uint32_t)f * (uint32_t)K * 2u + (uint32_t)((fchunk ^ (r & 7)) * 16);
    }
    const int wbase = (wave * 64 / CPR) * ROWB;  // this wave's 1 KiB slice of a fetch pass

    auto fetch_one = [&](int i, int kbyte, uint8_t* st) {
        // i-th direct load of a k-tile: A passes first, then B passes
#ifdef MOE_PIPE_SKIPB
        if (i >= PA && kbyte != 0) return;  // diagnostic build: half the load traffic, wrong results
#endif
        if (i < PA) {
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void*)(a_base + kbyte + a_goff[i]),
                (__attribute__((address_space(3))) void*)(st + i * RPP * ROWB + wbase), 16, 0, 0);
        } else {
            const int p = i - PA;
            const uint8_t* base = (SWIGLU && p >= PB / 2) ? b_base1 : b_base0;
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void*)(base + kbyte + b_goff[p]),
                (__attribute__((address_space(3))) void*)(st + A_BYTES + p * RPP * ROWB + wbase), 16, 0, 0);
        }
    };

    // ---- fragment addressing ----
    const int fr = lane & 31, fk = lane >> 5;
    int a_off[FM], b_off[FN], a_sw[FM], b_sw[FN];
#pragma unroll
    for (int i = 0; i < FM; ++i) {
        const int r = wm * WM + i * 32 + fr;
        a_off[i] = r * ROWB;
        a_sw[i] = r & 7;
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
        b_off[j] = A_BYTES + r * ROWB;
        b_sw[j] = r & 7;
    }

    f32x16 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    bf16x8 af[2][FM], bfg[2][FN];
    // fragment q of k-step s (A fragments first, then B) into register set `buf`
    auto read_one = [&](const uint8_t* st, int s, int buf, int q) {
        const int c = 2 * s + fk;
        if (q < FM)
            af[buf][q] = __builtin_bit_cast(
                bf16x8, *reinterpret_cast<const u32x4*>(st + a_off[q] + ((c ^ a_sw[q]) << 4)));
        else
            bfg[buf][q - FM] = __builtin_bit_cast(
                bf16x8, *reinterpret_cast<const u32x4*>(st + b_off[q - FM] + ((c ^ b_sw[q - FM]) << 4)));
    };
    auto mfma_one = [&](int buf, int m) {
        const int i = m / FN, j = m % FN;
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfg[buf][j], af[buf][i], acc[i][j], 0, 0, 0);
    };
    // One k-step, written in the order it should issue: NSLOT slots of
    // {MPS MFMAs on set mf_buf; up to `rps` fragment reads of k-step rd_s into
    // the other set; up to `lps` direct loads of the next tile}, each slot
    // closed by a scheduling barrier so the compiler keeps this order.  The
    // direct loads write LDS, so the compiler would not move LDS reads across
    // them anyway: the interleave has to be in the source.
    constexpr int NSLOT = NREAD;
    constexpr int MPS = NMFMA / NSLOT;
    auto kstep = [&](int mf_buf, bool do_read, const uint8_t* rd_st, int rd_s, int rps, int ld_begin,
                     int ld_end, int lps, int kbyte, uint8_t* ld_st) {
        int m = 0, rd = 0, ld = ld_begin;
#pragma unroll
        for (int slot = 0; slot < NSLOT; ++slot) {
#pragma unroll
            for (int q = 0; q < MPS; ++q) {
                mfma_one(mf_buf, m);
                ++m;
            }
#pragma unroll
            for (int q = 0; q < 2; ++q)
                if (do_read && q < rps && rd < NREAD) {
                    read_one(rd_st, rd_s, mf_buf ^ 1, rd);
                    ++rd;
                }
#pragma unroll
            for (int q = 0; q < 2; ++q)
                if (q < lps && ld < ld_end) {
                    fetch_one(ld, kbyte, ld_st);
                    ++ld;
                }
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int mm = NSLOT * MPS; mm < NMFMA; ++mm) mfma_one(mf_buf, mm);
        __builtin_amdgcn_sched_barrier(0);
    };

    const int KT = K / BK;
    // prologue: tile 0 -> stage 0, first fragments -> set 0
#pragma unroll
    for (int i = 0; i < NLOAD; ++i) fetch_one(i, 0, smem);
    wait_vmcnt0();
    __syncthreads();
#pragma unroll
    for (int q = 0; q < NREAD; ++q) read_one(smem, 0, 0, q);

    // When the next tile's direct loads are issued (the texture path moves 64 B
    // per clock, so a tile's loads keep it busy for about half a k-tile; a burst
    // fills its queue and blocks the issuing wave, MFMAs included):
    //   LMODE 0: one per slot under k-steps 0 and 1
    //   LMODE 1: two per slot, all under k-step 0
    //   LMODE 2: one per slot, a third each under k-step 3 of the previous tile
    //            (the stage is free from that tile's barrier on), k-steps 0 and 1
    constexpr int LPS = (LMODE == 1) ? 2 : 1;
    constexpr int LA = (LMODE == 2) ? NLOAD / 3 : 0;                       // issued one tile early
    constexpr int LB = (LMODE == 2) ? LA + (NLOAD - LA + 1) / 2
                                    : ((LPS * NSLOT < NLOAD) ? LPS * NSLOT : NLOAD);  // end of k-step 0's share
    static_assert(LB - LA <= LPS * NSLOT && NLOAD - LB <= LPS * NSLOT && LA <= NSLOT, "not enough slots for the loads");
    if (LMODE == 2) {
        const int kb1 = min(1, KT - 1) * BK * 2;
#pragma unroll
        for (int i = 0; i < LA; ++i) fetch_one(i, kb1, smem + STAGE);
    }

#ifdef MOE_PIPE_TIMING
    unsigned long long tk_wait = 0, tk_bar = 0;
    const unsigned long long tk_begin = __builtin_amdgcn_s_memtime();
#endif
    for (int kt = 0; kt < KT - 1; ++kt) {
        const uint8_t* cur = smem + (kt & 1) * STAGE;
        uint8_t* nxt = smem + ((kt & 1) ^ 1) * STAGE;
        const int kbyte = (kt + 1) * BK * 2;
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (LMODE == 3) {
            // late barrier: the loads get all four k-steps to land; the price is
            // that the next tile's first fragments are read with nothing to hide them
            kstep(0, true, cur, 1, 2, 0, LB, 1, kbyte, nxt);
            kstep(1, true, cur, 2, 2, LB, NLOAD, 1, kbyte, nxt);
            kstep(0, true, cur, 3, 2, 0, 0, 0, kbyte, nxt);
            kstep(1, false, cur, 0, 0, 0, 0, 0, kbyte, nxt);
            __builtin_amdgcn_s_waitcnt(0);
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int q = 0; q < NREAD; ++q) read_one(nxt, 0, 0, (FM == FN) ? ((q & 1) ? FM + q / 2 : q / 2) : q);  // A0,B0,A1,B1,... when square
            continue;
        }
        kstep(0, true, cur, 1, 2, LA, LB, LPS, kbyte, nxt);      // k-step 0
        kstep(1, true, cur, 2, 2, LB, NLOAD, LPS, kbyte, nxt);   // k-step 1
        kstep(0, true, cur, 3, 2, 0, 0, 0, kbyte, nxt);          // k-step 2
        // next tile landed (this thread's part), this wave's reads of `cur` are
        // in registers: after the barrier `cur` may be overwritten and `nxt` read.
#ifdef MOE_PIPE_TIMING
        const unsigned long long tk0 = __builtin_amdgcn_s_memtime();
        __builtin_amdgcn_s_waitcnt(0);  // vmcnt(0), expcnt(0), lgkmcnt(0)
        const unsigned long long tk1 = __builtin_amdgcn_s_memtime();
        __builtin_amdgcn_s_barrier();
        const unsigned long long tk2 = __builtin_amdgcn_s_memtime();
        tk_wait += tk1 - tk0;
        tk_bar += tk2 - tk1;
#else
        __builtin_amdgcn_s_waitcnt(0);  // vmcnt(0), expcnt(0), lgkmcnt(0)
        __builtin_amdgcn_s_barrier();
#endif
        __builtin_amdgcn_sched_barrier(0);
        // k-step 3; the first fragments of the next tile are read early in it.
        // LMODE 2: `cur` is free now, the first loads of tile kt+2 go into it
        // (past the end of K the last tile is fetched again and never read)
        kstep(1, true, nxt, 0, 2, 0, LA, 1, min(kt + 2, KT - 1) * BK * 2, const_cast<uint8_t*>(cur));
    }
    {
        // last k-tile: nothing left to fetch
        const uint8_t* cur = smem + ((KT - 1) & 1) * STAGE;
        __builtin_amdgcn_sched_barrier(0);
        kstep(0, true, cur, 1, 2, 0, 0, 0, 0, smem);
        kstep(1, true, cur, 2, 2, 0, 0, 0, 0, smem);
        kstep(0, true, cur, 3, 2, 0, 0, 0, 0, smem);
        kstep(1, false, cur, 0, 0, 0, 0, 0, 0, smem);
    }

#ifdef MOE_PIPE_TIMING
    if (lane == 0 && blockIdx.x < 4096) {
        unsigned long long* o = g_pipe_ticks + ((size_t)blockIdx.x * 8 + wave) * 4;
        o[0] = __builtin_amdgcn_s_memtime() - tk_begin;
        o[1] = tk_wait;
        o[2] = tk_bar;
        o[3] = tk_begin;
    }
#endif
    if (LMODE == 2) wait_vmcnt0();  // the re-fetched last tile may still be landing in LDS
    store_tile<FM, FN, WM, WN, BN, SWIGLU>(acc, tile, C, N, n0, wm, wn, lane);
}

template <int BM, int BN, int WGM, int WGN, bool SWIGLU, int LMODE>
void launch_pipe(const void* A, const int32_t* offsets, int r_max, int E, int N, int K, const void* B0,
                 const void* B1, void* C, hipStream_t s) {
    constexpr int OUTN = SWIGLU ? BN / 2 : BN;
    constexpr size_t smem = 2 * (size_t)(BM + BN) * 64 * 2;
    const int ntn = (N + OUTN - 1) / OUTN;
    auto kern = gemm_bf16_pipe_kernel<BM, BN, WGM, WGN, SWIGLU, LMODE>;
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        attr_set = true;
    }
    const int grid = grid_for(r_max, E, BM, ntn);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(WGM * WGN * 64), smem, s, static_cast<const bf16_t*>(A),
                       offsets, E, N, K, static_cast<const bf16_t*>(B0),
                       static_cast<const bf16_t*>(B1), static_cast<bf16_t*>(C), ntn);
}

template <int BM, int BN, int WGM, int WGN, int LMODE>
void run_pipe_pair(const void* x_perm, const int32_t* offsets, int r_max, int H, int F, int E,
                   const void* w_gate, const void* w_up, const void* w_down, void* h, void* y_perm,
                   int phase, hipStream_t s) {
    if (phase & 1) launch_pipe<BM, BN, WGM, WGN, true, LMODE>(x_perm, offsets, r_max, E, F, H, w_gate, w_up, h, s);
    if (phase & 2) launch_pipe<BM, BN, WGM, WGN, false, LMODE>(h, offsets, r_max, E, H, F, w_down, nullptr, y_perm, s);
}

}  // namespace

bool launch_pipe_ffn(const void* x_perm, const int32_t* offsets, int r_max, int H, int F, int E,
                     const void* w_gate, const void* w_up, const void* w_down, void* h,
                     void* y_perm, int variant, int phase, hipStream_t s) {
    switch (variant) {
        case 11: run_pipe_pair<256, 256, 2, 2, 0>(x_perm, offsets, r_max, H, F, E, w_gate, w_up, w_down, h, y_perm, phase, s); return true;
        case 12: run_pipe_pair<256, 256, 2, 4, 0>(x_perm, offsets, r_max, H, F, E, w_gate, w_up, w_down, h, y_perm, phase, s); return true;
        case 13: run_pipe_pair<128, 256, 2, 2, 0>(x_perm, offsets, r_max, H, F, E, w_gate, w_up, w_down, h, y_perm, phase, s); return true;
        case 14: run_pipe_pair<256, 128, 2, 2, 0>(x_perm, offsets, r_max, H, F, E, w_gate, w_up, w_down, h, y_perm, phase, s); return true;
        case 15: run_pipe_pair<128, 128, 2, 2, 0>(x_perm, offsets, r_max, H, F, E, w_gate, w_up, w_down, h, y_perm, phase, s); return true;
        case 16: run_pipe_pair<256, 256, 2, 2, 1>(x_perm, offsets, r_max, H, F, E, w_gate, w_up, w_down, h, y_perm, phase, s); return true;
        case 17: run_pipe_pair<256, 256, 2, 4, 1>(x_perm, offsets, r_max, H, F, E, w_gate, w_up, w_down, h, y_perm, phase, s); return true;
        case 22: run_pipe_pair<256, 256, 2, 2, 3>(x_perm, offsets, r_max, H, F, E, w_gate, w_up, w_down, h, y_perm, phase, s); return true;
        case 23: run_pipe_pair<256, 256, 2, 4, 3>(x_perm, offsets, r_max, H, F, E, w_gate, w_up, w_down, h, y_perm, phase, s); return true;
        case 20: run_pipe_pair<256, 256, 2, 2, 2>(x_perm, offsets, r_max, H, F, E, w_gate, w_up, w_down, h, y_perm, phase, s); return true;
        case 21: run_pipe_pair<256, 256, 2, 4, 2>(x_perm, offsets, r_max, H, F, E, w_gate, w_up, w_down, h, y_perm, phase, s); return true;
        default: return false;
    }
}

}  // namespace moe
