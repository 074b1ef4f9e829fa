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
//   * scheduling-group barriers pin the interleave (1 LDS read : n MFMA, with
//     the next tile's global loads sprinkled over the first k-steps).
// Global addresses are a wave-uniform base plus a 32-bit per-lane offset that
// is fixed for the whole K loop.
#include "gemm_tile.h"

namespace moe {

namespace {

constexpr int SG_MFMA = 0x008, SG_VMEM_R = 0x020, SG_DS_R = 0x100;

// Interleave pattern of one k-step: NR slots, each "MPR MFMAs, one LDS read
// (the first NREAD slots), one global load (the first NLOAD slots)"; whatever
// MFMAs are left go last.
template <int I, int NR, int NREAD, int NLOAD, int MLEFT, int MPR>
__device__ __forceinline__ void pin_schedule() {
    if constexpr (I < NR) {
        // MFMAs first: their operands were read during the previous k-step, so
        // nothing issued in this slot is waited for
        constexpr int M = (MLEFT < MPR) ? MLEFT : MPR;
        if constexpr (M > 0) __builtin_amdgcn_sched_group_barrier(SG_MFMA, M, 0);
        if constexpr (I < NREAD) __builtin_amdgcn_sched_group_barrier(SG_DS_R, 1, 0);
        if constexpr (I < NLOAD) __builtin_amdgcn_sched_group_barrier(SG_VMEM_R, 1, 0);
        pin_schedule<I + 1, NR, NREAD, NLOAD, MLEFT - M, MPR>();
    } else if constexpr (MLEFT > 0) {
        __builtin_amdgcn_sched_group_barrier(SG_MFMA, MLEFT, 0);
    }
}

template <int BM, int BN, int WGM, int WGN, bool SWIGLU, bool EARLY, int DBG = 0>
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
    constexpr int MPR = (NMFMA / (2 * NREAD) > 1) ? NMFMA / (2 * NREAD) : 1;  // MFMAs between LDS reads (reads go early in the k-step)
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
    constexpr bool PF = (DBG == 3);
    constexpr int NPF = PF ? (BM + BN) / NT : 0;  // L2 prefetch touches per thread per k-tile
    __shared__ uint32_t pf_sink[PF ? NT : 1];

    // ---- fetch slots: uniform bases + per-lane 32-bit byte offsets ----
    const int frow = tid / CPR, fchunk = tid % CPR;
    const uint8_t* a_base = reinterpret_cast<const uint8_t*>(A + (size_t)(DBG == 2 ? 0 : tile.row0) * K);
    const size_t b_row0 = (DBG == 2) ? 0 : ((size_t)tile.expert * N + n0) * K;
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

    // L2 prefetch: two k-tiles ahead, every thread touches one 128-byte line of
    // "its" tile row(s) with a 4-byte direct load into a sink; nobody waits for it
    const uint8_t* pf_ptr[NPF > 0 ? NPF : 1];
    if (PF) {
#pragma unroll
        for (int q = 0; q < NPF; ++q) {
            const int r = q * NT + tid;  // 0..BM-1: A rows, BM..BM+BN-1: B rows
            if (r < BM) {
                pf_ptr[q] = a_base + (size_t)min(r, tile.rows - 1) * K * 2;
            } else {
                const int rb = r - BM;
                int f = SWIGLU ? (rb % (BN / 2)) : rb;
                f = min(f, N - 1 - n0);
                pf_ptr[q] = ((SWIGLU && rb >= BN / 2) ? b_base1 : b_base0) + (size_t)f * K * 2;
            }
        }
    }
    auto prefetch = [&](int kt_target) {
        if (PF) {
#pragma unroll
            for (int q = 0; q < NPF; ++q)
                __builtin_amdgcn_global_load_lds(
                    (const __attribute__((address_space(1))) void*)(pf_ptr[q] + (size_t)kt_target * (BK * 2)),
                    (__attribute__((address_space(3))) void*)(pf_sink + wave * 64), 4, 0, 0);
        }
    };

    auto fetch_one = [&](int i, int kbyte, uint8_t* st) {
        // i-th direct load of a k-tile: A passes first, then B passes
        if (DBG == 1 && kbyte != 0) return;
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
    auto read_frags = [&](const uint8_t* st, int s, int buf) {
        const int c = 2 * s + fk;
#pragma unroll
        for (int i = 0; i < FM; ++i)
            af[buf][i] = __builtin_bit_cast(
                bf16x8, *reinterpret_cast<const u32x4*>(st + a_off[i] + ((c ^ a_sw[i]) << 4)));
#pragma unroll
        for (int j = 0; j < FN; ++j)
            bfg[buf][j] = __builtin_bit_cast(
                bf16x8, *reinterpret_cast<const u32x4*>(st + b_off[j] + ((c ^ b_sw[j]) << 4)));
    };
    auto mfma_step = [&](int buf) {
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfg[buf][j], af[buf][i], acc[i][j], 0, 0, 0);
    };
    const int KT = K / BK;
    // prologue: tile 0 -> stage 0, first fragments -> set 0
#pragma unroll
    for (int i = 0; i < NLOAD; ++i) fetch_one(i, 0, smem);
    wait_vmcnt0();
    __syncthreads();
    read_frags(smem, 0, 0);

    // EARLY: all of the next tile's loads go out under k-step 0 (longest flight
    // time); else they are spread over k-steps 0..2
    constexpr int L0 = EARLY ? NLOAD : (NLOAD + 2) / 3;   // loads issued under k-step 0
    constexpr int L1 = EARLY ? 0 : (NLOAD - L0 + 1) / 2;  // under k-step 1
    constexpr int L2 = NLOAD - L0 - L1;                   // under k-step 2

    for (int kt = 0; kt < KT - 1; ++kt) {
        const uint8_t* cur = smem + (kt & 1) * STAGE;
        uint8_t* nxt = smem + ((kt & 1) ^ 1) * STAGE;
        const int kbyte = (kt + 1) * BK * 2;
        __builtin_amdgcn_sched_barrier(0);
        // k-step 0
#pragma unroll
        for (int i = 0; i < L0; ++i) fetch_one(i, kbyte, nxt);
        if (EARLY) prefetch(min(kt + 2, KT - 1));
        read_frags(cur, 1, 1);
        mfma_step(0);
        pin_schedule<0, (L0 + (EARLY ? NPF : 0) > NREAD ? L0 + (EARLY ? NPF : 0) : NREAD), NREAD, L0 + (EARLY ? NPF : 0), NMFMA, MPR>();
        __builtin_amdgcn_sched_barrier(0);
        // k-step 1
#pragma unroll
        for (int i = L0; i < L0 + L1; ++i) fetch_one(i, kbyte, nxt);
        read_frags(cur, 2, 0);
        mfma_step(1);
        pin_schedule<0, NREAD, NREAD, L1, NMFMA, MPR>();
        __builtin_amdgcn_sched_barrier(0);
        // k-step 2
#pragma unroll
        for (int i = L0 + L1; i < NLOAD; ++i) fetch_one(i, kbyte, nxt);
        read_frags(cur, 3, 1);
        mfma_step(0);
        pin_schedule<0, NREAD, NREAD, L2, NMFMA, MPR>();
        __builtin_amdgcn_sched_barrier(0);
        // next tile landed (this thread's part), this wave's reads of `cur` are
        // in registers: after the barrier `cur` may be overwritten and `nxt` read
        // lgkmcnt(0), expcnt(0) and vmcnt(NPF): the NPF youngest loads are this
        // iteration's L2 prefetches, which may stay in flight
        __builtin_amdgcn_s_waitcnt((NPF & 0xF) | ((NPF >> 4) << 14));
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        // k-step 3, first fragments of the next tile underneath
        read_frags(nxt, 0, 0);
        mfma_step(1);
        pin_schedule<0, NREAD, NREAD, 0, NMFMA, MPR>();
        __builtin_amdgcn_sched_barrier(0);
    }
    {
        // last k-tile: nothing left to fetch
        const uint8_t* cur = smem + ((KT - 1) & 1) * STAGE;
        __builtin_amdgcn_sched_barrier(0);
        read_frags(cur, 1, 1);
        mfma_step(0);
        pin_schedule<0, NREAD, NREAD, 0, NMFMA, MPR>();
        __builtin_amdgcn_sched_barrier(0);
        read_frags(cur, 2, 0);
        mfma_step(1);
        pin_schedule<0, NREAD, NREAD, 0, NMFMA, MPR>();
        __builtin_amdgcn_sched_barrier(0);
        read_frags(cur, 3, 1);
        mfma_step(0);
        pin_schedule<0, NREAD, NREAD, 0, NMFMA, MPR>();
        __builtin_amdgcn_sched_barrier(0);
        mfma_step(1);
        __builtin_amdgcn_sched_barrier(0);
    }

    if (PF) wait_vmcnt0();
    store_tile<FM, FN, WM, WN, BN, SWIGLU>(acc, tile, C, N, n0, wm, wn, lane);
}

template <int BM, int BN, int WGM, int WGN, bool SWIGLU, bool EARLY, int DBG = 0>
void launch_pipe(const void* A, const int32_t* offsets, int r_max, int E, int N, int K, const void* B0,
                 const void* B1, void* C, hipStream_t s) {
    constexpr int OUTN = SWIGLU ? BN / 2 : BN;
    constexpr size_t smem = 2 * (size_t)(BM + BN) * 64 * 2;
    const int ntn = (N + OUTN - 1) / OUTN;
    auto kern = gemm_bf16_pipe_kernel<BM, BN, WGM, WGN, SWIGLU, EARLY, DBG>;
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

template <int BM, int BN, int WGM, int WGN, bool EARLY, int DBG = 0>
void run_pipe_pair(const void* x_perm, const int32_t* offsets, int r_max, int H, int F, int E,
                   const void* w_gate, const void* w_up, const void* w_down, void* h, void* y_perm,
                   int phase, hipStream_t s) {
    if (phase & 1) launch_pipe<BM, BN, WGM, WGN, true, EARLY, DBG>(x_perm, offsets, r_max, E, F, H, w_gate, w_up, h, s);
    if (phase & 2) launch_pipe<BM, BN, WGM, WGN, false, EARLY, DBG>(h, offsets, r_max, E, H, F, w_down, nullptr, y_perm, s);
}

}  // namespace

bool launch_pipe_ffn(const void* x_perm, const int32_t* offsets, int r_max, int H, int F, int E,
                     const void* w_gate, const void* w_up, const void* w_down, void* h,
                     void* y_perm, int variant, int phase, hipStream_t s) {
    switch (variant) {
        case 11: run_pipe_pair<256, 256, 2, 2, false>(x_perm, offsets, r_max, H, F, E, w_gate, w_up, w_down, h, y_perm, phase, s); return true;
        case 12: run_pipe_pair<256, 256, 2, 4, false>(x_perm, offsets, r_max, H, F, E, w_gate, w_up, w_down, h, y_perm, phase, s); return true;
        case 13: run_pipe_pair<128, 256, 2, 2, false>(x_perm, offsets, r_max, H, F, E, w_gate, w_up, w_down, h, y_perm, phase, s); return true;
        case 14: run_pipe_pair<256, 128, 2, 2, false>(x_perm, offsets, r_max, H, F, E, w_gate, w_up, w_down, h, y_perm, phase, s); return true;
        case 15: run_pipe_pair<128, 128, 2, 2, false>(x_perm, offsets, r_max, H, F, E, w_gate, w_up, w_down, h, y_perm, phase, s); return true;
        case 16: run_pipe_pair<256, 256, 2, 2, true>(x_perm, offsets, r_max, H, F, E, w_gate, w_up, w_down, h, y_perm, phase, s); return true;
        case 17: run_pipe_pair<256, 256, 2, 4, true>(x_perm, offsets, r_max, H, F, E, w_gate, w_up, w_down, h, y_perm, phase, s); return true;
        case 18: run_pipe_pair<256, 256, 2, 2, true, 3>(x_perm, offsets, r_max, H, F, E, w_gate, w_up, w_down, h, y_perm, phase, s); return true;
        case 19: run_pipe_pair<256, 256, 2, 4, true, 3>(x_perm, offsets, r_max, H, F, E, w_gate, w_up, w_down, h, y_perm, phase, s); return true;
        case 91: run_pipe_pair<256, 256, 2, 2, true, 1>(x_perm, offsets, r_max, H, F, E, w_gate, w_up, w_down, h, y_perm, phase, s); return true;
        case 92: run_pipe_pair<256, 256, 2, 2, true, 2>(x_perm, offsets, r_max, H, F, E, w_gate, w_up, w_down, h, y_perm, phase, s); return true;
        case 93: run_pipe_pair<256, 256, 2, 4, true, 1>(x_perm, offsets, r_max, H, F, E, w_gate, w_up, w_down, h, y_perm, phase, s); return true;
        case 94: run_pipe_pair<256, 256, 2, 4, true, 2>(x_perm, offsets, r_max, H, F, E, w_gate, w_up, w_down, h, y_perm, phase, s); return true;
        default: return false;
    }
}

}  // namespace moe
