// Grouped expert GEMM (a3) on FP8 operands with per-tensor delayed scaling
// (Section 4.5, "FP8 Training Performance").
//
// Same persistent engine as gemm_persist.hip, byte for byte on the memory
// side: 256 x 256 output tiles, LDS rows of 128 bytes (here 128 E4M3 values,
// so a k-tile spans 128 of the contraction index), three LDS stages for the
// activation tile and two for the weight tile filled by direct global->LDS
// loads, the k-tiles of successive output tiles as one stream, register-
// resident tile scheduler, epilogue staged through the idle LDS stage.
//
// What differs: the matrix instruction is the 32x32x64 FP8 MFMA (each lane
// feeds 32 consecutive bytes of a row, two k-steps per k-tile, twice the math
// per byte moved); 4 waves of 128 x 128 (the accumulators fill the accumulation
// registers, the 2 x 64 fragment registers double-buffer the two k-steps);
// and the epilogues: the gate/up GEMM dequantises g and u, applies SwiGLU,
// records max |h| for the next step's scale and writes h as E4M3 with this
// step's (delayed) scale; the down GEMM dequantises into bf16.
#include "fp8_convert.h"
#include "gemm_persist.h"

namespace moe {

namespace {

typedef __attribute__((ext_vector_type(8))) int i32x8;

// Epilogue of the gate/up GEMM: h = silu(g) * u from the dequantised
// accumulators, one byte per value.  Staged through a wave-private LDS patch of
// W = 32*FO bytes per row (16-byte granules XOR-swizzled by the row) so that the
// global stores are whole 16-byte pieces along the rows.
template <int FM, int FN, int WM>
__device__ __forceinline__ float store_h_fp8(f32x16 (&acc)[FM][FN], int t_row0, int t_rows, int t_n0, uint8_t* C,
                                             int N, int wm, int wn, int lane, uint8_t* stage, float dq_gate,
                                             float dq_up, float scale_h, float amax) {
    constexpr int FO = FN / 2;
    constexpr int W = FO * 32;        // bytes per staged row
    constexpr int GPR = W / 16;       // granules per row
    constexpr int RP256 = 256 / W;    // rows per 256 bytes
    constexpr int RPI = 1024 / W;     // rows per 64-lane read
    static_assert(W <= 256 && 256 % W == 0 && 32 % RPI == 0, "staged row must divide the bank window");
    asm volatile("" : "+v"(lane));    // keeps the addresses below from being hoisted out of the tile loop
    const int fr = lane & 31, fk = lane >> 5;
    const int xw = (fr / RP256) & (GPR - 1);
    uint8_t* wrow = stage + fr * W + 4 * fk;
    const int rl = lane / GPR, gl = lane % GPR;
    const int col = t_n0 + wn * (FO * 32) + gl * 16;
#pragma unroll
    for (int i = 0; i < FM; ++i) {
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < FN; ++j) asm volatile("" : "+a"(acc[i][j]));   // see gemm_persist.hip
#pragma unroll
        for (int j = 0; j < FO; ++j) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float hv[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const float g = acc[i][j][4 * q + u] * dq_gate;
                    const float up = acc[i][j + FO][4 * q + u] * dq_up;
                    hv[u] = g * __builtin_amdgcn_rcpf(1.f + __expf(-g)) * up;   // silu(g) * up
                    amax = fmaxf(amax, fabsf(hv[u]));
                }
                const uint32_t packed = f32x4_to_e4m3(hv[0] * scale_h, hv[1] * scale_h, hv[2] * scale_h,
                                                      hv[3] * scale_h);
                // lane's 4 columns: bytes j*32 + 8q + 4fk .. +3 of the row
                const int gran = 2 * j + (q >> 1);
                *reinterpret_cast<uint32_t*>(wrow + ((gran ^ xw) << 4) + 8 * (q & 1)) = packed;
            }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int it = 0; it < 32 / RPI; ++it) {
            const int row = it * RPI + rl;
            const int xr = (row / RP256) & (GPR - 1);
            const u32x4 v = *reinterpret_cast<const u32x4*>(stage + row * W + ((gl ^ xr) << 4));
            const int grow = wm * WM + i * 32 + row;
            if (grow < t_rows && col < N)
                *reinterpret_cast<u32x4*>(C + (size_t)(t_row0 + grow) * N + col) = v;
        }
    }
    return amax;
}

// Epilogue of the down GEMM: y = acc * dq as bf16, staged like the bf16 kernel's.
template <int FM, int FN, int WM>
__device__ __forceinline__ void store_y_bf16(f32x16 (&acc)[FM][FN], int t_row0, int t_rows, int t_n0, bf16_t* C,
                                             int N, int wm, int wn, int lane, uint8_t* stage, float dq) {
    constexpr int W = FN * 64;
    constexpr int GPR = W / 16;
    constexpr int RP256 = 256 / W;
    constexpr int RPI = 1024 / W;
    static_assert(W <= 256 && 256 % W == 0, "staged row must divide the bank window");
    asm volatile("" : "+v"(lane));
    const int fr = lane & 31, fk = lane >> 5;
    const int xw = (fr / RP256) & (GPR - 1);
    uint8_t* wrow = stage + fr * W + 8 * fk;
    const int rl = lane / GPR, gl = lane % GPR;
    const int col = t_n0 + wn * (FN * 32) + gl * 8;
#pragma unroll
    for (int i = 0; i < FM; ++i) {
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < FN; ++j) asm volatile("" : "+a"(acc[i][j]));
#pragma unroll
        for (int j = 0; j < FN; ++j) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                u32x2 o;
                o[0] = pack2_bf16(acc[i][j][4 * q + 0] * dq, acc[i][j][4 * q + 1] * dq);
                o[1] = pack2_bf16(acc[i][j][4 * q + 2] * dq, acc[i][j][4 * q + 3] * dq);
                *reinterpret_cast<u32x2*>(wrow + (((4 * j + q) ^ xw) << 4)) = o;
            }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int it = 0; it < 32 / RPI; ++it) {
            const int row = it * RPI + rl;
            const int xr = (row / RP256) & (GPR - 1);
            const u32x4 v = *reinterpret_cast<const u32x4*>(stage + row * W + ((gl ^ xr) << 4));
            const int grow = wm * WM + i * 32 + row;
            if (grow < t_rows && col < N)
                *reinterpret_cast<u32x4*>(C + (size_t)(t_row0 + grow) * N + col) = v;
        }
    }
}

// A [rows, K] E4M3, B0/B1 [E, N, K] E4M3 (SWIGLU: gate and up), K a multiple of
// 128.  SWIGLU: C is h [rows, N] E4M3, s0/s1 dequantise g/u, s2 scales h, amax
// receives max |h|.  Otherwise C is y [rows, N] bf16 and s0 dequantises it.
// DEEP_B: the weight tile, not the activation tile, gets the three LDS stages (see gemm_persist.hip).
template <bool SWIGLU, bool IDLE_SKIP = false, bool DEEP_B = false>
__global__ __launch_bounds__(256) void gemm_fp8_persist_kernel(
    const uint8_t* __restrict__ A, const int32_t* __restrict__ offsets, int E, int N, int K,
    const uint8_t* __restrict__ B0, const uint8_t* __restrict__ B1, void* __restrict__ C, int ntn, float s0,
    float s1, float s2, float* __restrict__ amax_out) {
    constexpr int BM = 256, BN = 256, WGM = 2, WGN = 2;
    constexpr int NW = WGM * WGN;
    constexpr int NT = NW * 64;
    constexpr int WM = BM / WGM, WN = BN / WGN;
    constexpr int FM = WM / 32, FN = WN / 32;
    constexpr int ROWB = 128;                   // bytes (= E4M3 values) per tile row and k-tile
    constexpr int CPR = ROWB / 16;
    constexpr int RPP = NT / CPR;
    constexpr int PA = BM / RPP, PB = BN / RPP;
    constexpr int A_BYTES = BM * ROWB, B_BYTES = BN * ROWB;
    constexpr int B_REGION = (DEEP_B ? 2 : 3) * A_BYTES;
    // "early" operand: two slots, fetched one k-tile ahead, issued first in a period; "late": three slots
    constexpr int PE = DEEP_B ? PA : PB, PL = DEEP_B ? PB : PA;
    constexpr int OUTN = SWIGLU ? BN / 2 : BN;
    constexpr int NLOAD = PA + PB;
    constexpr int NREAD = 2 * (FM + FN);        // 16-byte LDS reads per k-step: two per fragment
    constexpr int NMFMA = FM * FN;
    constexpr int NSLOT = NMFMA;                // one MFMA (64 cycles) per slot
    // a period's loads: the head of the weight tile under k-step 1 of the previous
    // k-tile (after the barrier), the rest and the activation tile under k-step 0
    constexpr int LA = NLOAD / 3;
    static_assert(LA <= PE && NLOAD - LA <= NSLOT && LA <= NSLOT && NREAD <= 2 * NSLOT, "slots");
    static_assert(3 * A_BYTES + 2 * B_BYTES <= 160 * 1024, "tile stages exceed the 160 KiB of LDS");
    static_assert(NW * 32 * (FN * 64) <= (DEEP_B ? B_BYTES : A_BYTES), "epilogue patches must fit into one slot of the late operand");

    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WGN, wn = wave % WGN;

    const uint8_t* const B1b = SWIGLU ? B1 : B0;
    TileSched<BM> sched;
    sched.init(offsets, E, ntn, lane);
    int ti = 0;
    const uint8_t *c_a, *c_b0, *c_b1, *n_a, *n_b0, *n_b1;
    uint32_t c_alim, c_blim, n_alim, n_blim;
    int c_row0, c_rows, c_n0, n_row0, n_rows, n_n0;
    bool n_valid;
    {
        const PTile t = sched.get(0, A, B0, B1b, N, (size_t)K, OUTN);
        if (!t.valid) return;
        c_a = t.a; c_b0 = t.b0; c_b1 = t.b1; c_alim = t.a_lim; c_blim = t.b_lim;
        c_row0 = t.row0; c_rows = t.rows; c_n0 = t.n0;
    }
    auto fetch_next_tile = [&](int i) {
        const PTile t = sched.get(i, A, B0, B1b, N, (size_t)K, OUTN);
        n_a = t.a; n_b0 = t.b0; n_b1 = t.b1; n_alim = t.a_lim; n_blim = t.b_lim;
        n_row0 = t.row0; n_rows = t.rows; n_n0 = t.n0; n_valid = t.valid;
    };
    fetch_next_tile(1);

    // global side of the direct loads (see gemm_persist.hip)
    const int frow = tid / CPR, fchunk = tid % CPR;
    const uint32_t rowb = (uint32_t)K;
    const uint32_t vrow = (uint32_t)frow * rowb;
    const uint32_t vswz = (uint32_t)((fchunk ^ lds_swizzle(frow)) * 16);
    const uint32_t step = (uint32_t)RPP * rowb;
    const int wbase = (wave * 64 / CPR) * ROWB;
    auto fetch_a = [&](int p, const uint8_t* base, uint32_t lim, uint8_t* st) {
        const uint32_t off = min(vrow + (uint32_t)p * step, lim) + vswz;
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(base + off),
                                         (__attribute__((address_space(3))) void*)(st + p * RPP * ROWB + wbase), 16,
                                         0, 0);
    };
    auto fetch_b = [&](int p, const uint8_t* base0, const uint8_t* base1, uint32_t lim, uint8_t* st) {
        const int pp = SWIGLU ? p % (PB / 2) : p;
        const uint8_t* base = (SWIGLU && p >= PB / 2) ? base1 : base0;
        const uint32_t off = min(vrow + (uint32_t)pp * step, lim) + vswz;
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(base + off),
                                         (__attribute__((address_space(3))) void*)(st + p * RPP * ROWB + wbase), 16,
                                         0, 0);
    };
    struct Src {
        const uint8_t* a;
        const uint8_t* b0;
        const uint8_t* b1;
        uint32_t a_lim, b_lim;
    };
    const int KT = K / ROWB;
    auto src = [&](int kk) -> Src {
        const bool in_cur = kk < KT;
        const bool use_cur = in_cur || !n_valid;  // past the last tile: its last k-tile again, never used
        const int k = in_cur ? kk : (n_valid ? kk - KT : KT - 1);
        const size_t kbyte = (size_t)k * ROWB;
        Src s;
        s.a = (use_cur ? c_a : n_a) + kbyte;
        s.b0 = (use_cur ? c_b0 : n_b0) + kbyte;
        s.b1 = (use_cur ? c_b1 : n_b1) + kbyte;
        s.a_lim = use_cur ? c_alim : n_alim;
        s.b_lim = use_cur ? c_blim : n_blim;
        return s;
    };
    // load i of a period: the early operand's passes first (source se), then the late operand's (source sl)
    auto fetch_one = [&](int i, const Src& se, const Src& sl, uint8_t* ld_b, uint8_t* ld_a) {
        if constexpr (DEEP_B) {
            if (i < PA)
                fetch_a(i, se.a, se.a_lim, ld_a);
            else
                fetch_b(i - PA, sl.b0, sl.b1, sl.b_lim, ld_b);
        } else {
            if (i < PB)
                fetch_b(i, se.b0, se.b1, se.b_lim, ld_b);
            else
                fetch_a(i - PB, sl.a, sl.a_lim, ld_a);
        }
    };

    const int fr = lane & 31, fk = lane >> 5;
    int a_off[FM], b_off[FN];
    const int f_sw = lds_swizzle(fr);
#pragma unroll
    for (int i = 0; i < FM; ++i) a_off[i] = (wm * WM + i * 32 + fr) * ROWB;
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
    }

    f32x16 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // fragment registers as 16-byte halves: half h of fragment q of set buf.  A
    // lane's 32 bytes of k-step s are the granules 4s + 2fk and 4s + 2fk + 1 of
    // its row (activations and weights use the same bytes, which is all the
    // instruction needs).
    u32x4 afh[2][FM][2], bfh[2][FN][2];
    auto read_one = [&](const uint8_t* sa, const uint8_t* sb, int s, int buf, int r) {
        const int q = r >> 1, h = r & 1;
        const int c = ((4 * s + 2 * fk + h) ^ f_sw) << 4;
        if (q < FM)
            afh[buf][q][h] = *reinterpret_cast<const u32x4*>(sa + a_off[q] + c);
        else
            bfh[buf][q - FM][h] = *reinterpret_cast<const u32x4*>(sb + b_off[q - FM] + c);
    };
    auto frag = [&](const u32x4 (&h)[2]) -> i32x8 {
        i32x8 v;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            v[t] = (int)h[0][t];
            v[4 + t] = (int)h[1][t];
        }
        return v;
    };
    auto mfma_one = [&](int buf, int m) {
        // boustrophedon over the wave's blocks: successive MFMAs share one operand fragment
        const int i = m / FN, j = (i & 1) ? FN - 1 - m % FN : m % FN;
        // E4M3 x E4M3 (formats 0, 0), no block scales; weight fragment first as in the bf16 kernels
        acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(frag(bfh[buf][j]), frag(afh[buf][i]), acc[i][j],
                                                                    0, 0, 0, 0, 0, 0);
    };
    // one k-step in issue order: NSLOT slots of {one MFMA on set mf_buf; up to 2
    // fragment reads of k-step rd_s into the other set; one direct load}
    // `aside`: scalar bookkeeping run under the MFMA of a late slot (the next period's load sources; see
    // gemm_persist.hip: with one wave per SIMD nothing else covers it)
    auto kstep = [&](int mf_buf, const uint8_t* rd_a, const uint8_t* rd_b, int rd_s, int ld_begin, int ld_end,
                     const Src& se, const Src& sl, uint8_t* ld_b, uint8_t* ld_a, auto&& aside) {
        int rd = 0, ld = ld_begin;
#pragma unroll
        for (int slot = 0; slot < NSLOT; ++slot) {
            mfma_one(mf_buf, slot);
            if (slot == NSLOT - 4) aside();
            // the first MFMA waits for the previous k-step's fragment reads only: keep the new reads behind it
            if (slot == 0) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int q = 0; q < 2; ++q)
                if (rd < NREAD) {
                    read_one(rd_a, rd_b, rd_s, mf_buf ^ 1, rd);
                    ++rd;
                }
            if (ld < ld_end) {
                fetch_one(ld, se, sl, ld_b, ld_a);
                ++ld;
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    uint8_t* const a_region = smem;
    uint8_t* const b_region = smem + B_REGION;
    {
        // late(0), early(0), late(1); the first two must have landed before the first fragment reads
        const Src q0 = src(0), q1 = src(1);
#pragma unroll
        for (int i = PE; i < NLOAD; ++i) fetch_one(i, q0, q0, b_region, a_region);
#pragma unroll
        for (int i = 0; i < PE; ++i) fetch_one(i, q0, q0, b_region, a_region);
#pragma unroll
        for (int i = PE; i < NLOAD; ++i)
            fetch_one(i, q1, q1, b_region + (DEEP_B ? B_BYTES : 0), a_region + (DEEP_B ? 0 : A_BYTES));
        __builtin_amdgcn_s_waitcnt(0x0F70 | (PL & 0xF) | ((PL >> 4) << 14));  // vmcnt(PL)
        __builtin_amdgcn_s_barrier();
#pragma unroll
        for (int r = 0; r < NREAD; ++r) read_one(a_region, b_region, 0, 0, r);
#pragma unroll
        for (int i = 0; i < LA; ++i) fetch_one(i, q1, q1, b_region + B_BYTES, a_region + A_BYTES);
    }

    float amax = 0.f;
    // slots of k-tiles kt, kt+1 (, kt+2): three for the late operand, two for the early one
    int a0 = 0, a1 = A_BYTES, a2 = DEEP_B ? 0 : 2 * A_BYTES;
    int b0 = 0, b1 = B_BYTES, b2 = DEEP_B ? 2 * B_BYTES : 0;
    auto rotate = [&]() {
        if constexpr (DEEP_B) {
            const int ta = a0; a0 = a1; a1 = ta;
            const int tb = b0; b0 = b1; b1 = b2; b2 = tb;
        } else {
            const int ta = a0; a0 = a1; a1 = a2; a2 = ta;
            const int tb = b0; b0 = b1; b1 = tb;
        }
    };
    for (;;) {
        // IDLE_SKIP (launches with many experts): a wave whose rows of the tile all lie past its last valid row
        // only issues its share of the loads and meets the barriers (see gemm_persist.hip)
        const bool wave_idle = IDLE_SKIP && wm * WM >= c_rows;   // wave-uniform
        if (!wave_idle) {
        // the load sources of k-tiles kt+1 and kt+2 are carried from period to period; the one a period adds is
        // formed under the MFMAs of the previous period (a tile's first period forms its own)
        Src q1 = src(1), q2 = src(2), q3 = q2;
        auto nothing = [] {};
        for (int kt = 0; kt < KT; ++kt) {
            __builtin_amdgcn_sched_barrier(0);
            // k-step 0: rest of early(kt+1), all of late(kt+2)
            kstep(0, a_region + a0, b_region + b0, 1, LA, NLOAD, q1, q2, b_region + (DEEP_B ? b2 : b1),
                  a_region + (DEEP_B ? a1 : a2), [&] { q3 = src(kt + 3); });
            // all but the PL youngest loads (those of late(kt+2)) have landed; this
            // wave's fragment reads of k-tile kt are in registers
            __builtin_amdgcn_s_waitcnt((PL & 0xF) | ((PL >> 4) << 14));
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);
            // k-step 1: first fragments of k-tile kt+1, head of early(kt+2) into the freed slot
            kstep(1, a_region + a1, b_region + b1, 0, 0, LA, q2, q2, b_region + b0, a_region + a0, nothing);
            rotate();
            q1 = q2;
            q2 = q3;
        }
        } else {
            for (int kt = 0; kt < KT; ++kt) {
                const Src q1 = src(kt + 1), q2 = src(kt + 2);
#pragma unroll
                for (int i = LA; i < NLOAD; ++i)
                    fetch_one(i, q1, q2, b_region + (DEEP_B ? b2 : b1), a_region + (DEEP_B ? a1 : a2));
                __builtin_amdgcn_s_waitcnt((PL & 0xF) | ((PL >> 4) << 14));
                __builtin_amdgcn_s_barrier();
#pragma unroll
                for (int i = 0; i < LA; ++i) fetch_one(i, q2, q2, b_region + b0, a_region + a0);
                rotate();
            }
            if (n_valid) {   // the next tile may have rows for this wave: its first fragments
#pragma unroll
                for (int r = 0; r < NREAD; ++r) read_one(a_region + a0, b_region + b0, 0, 0, r);
            }
        }
        uint8_t* stage = (DEEP_B ? b_region + b2 : a_region + a2) + wave * (32 * FN * 64);
        if (SWIGLU)
            amax = store_h_fp8<FM, FN, WM>(acc, c_row0, c_rows, c_n0, static_cast<uint8_t*>(C), N, wm, wn, lane, stage,
                                           s0, s1, s2, amax);
        else
            store_y_bf16<FM, FN, WM>(acc, c_row0, c_rows, c_n0, static_cast<bf16_t*>(C), N, wm, wn, lane, stage, s0);
        if (!n_valid) break;
        c_a = n_a; c_b0 = n_b0; c_b1 = n_b1; c_alim = n_alim; c_blim = n_blim;
        c_row0 = n_row0; c_rows = n_rows; c_n0 = n_n0;
        ++ti;
        fetch_next_tile(ti + 1);
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
        __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): this wave is done with its patch
        __builtin_amdgcn_s_barrier();
    }
    wait_vmcnt0();  // loads past the end of the last tile may still be landing in LDS
    if (SWIGLU && amax_out) {
        // max |h| over the wave, then one atomic per wave; h >= 0 as a float compares like its bit pattern.
        // Rows past the tile's valid rows may have contributed garbage: they were computed from re-read valid
        // rows of the same expert, so they are values h takes anyway.
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off, 64));
        if (lane == 0 && amax > __builtin_nontemporal_load(amax_out))   // *amax_out only grows; NaN compares false
            atomicMax(reinterpret_cast<int*>(amax_out), __float_as_int(amax));
    }
}

static int g_fp8_deep_b = 1;   // three LDS stages for the weight tile (0: for the activation tile)

template <bool SWIGLU>
void launch_fp8(const void* A, const int32_t* offsets, int r_max, int E, int N, int K, const void* B0, const void* B1,
                void* C, float s0, float s1, float s2, float* amax, hipStream_t s) {
    constexpr int OUTN = SWIGLU ? 128 : 256;
    constexpr size_t smem = (size_t)(3 * 256 + 2 * 256) * 128;
    const int ntn = (N + OUTN - 1) / OUTN;
    // (the gate/up kernel has no registers to spare for the second loop: down projection only)
    const bool idle_skip = !SWIGLU && persist_idle_skip(E);
    const bool deep = g_fp8_deep_b != 0;
    auto kern = deep ? (idle_skip ? gemm_fp8_persist_kernel<SWIGLU, !SWIGLU, true> : gemm_fp8_persist_kernel<SWIGLU, false, true>)
                     : (idle_skip ? gemm_fp8_persist_kernel<SWIGLU, !SWIGLU, false> : gemm_fp8_persist_kernel<SWIGLU, false, false>);
    static bool attr_set[2][2] = {{false, false}, {false, false}};
    if (!attr_set[deep][idle_skip]) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  (int)smem);
        attr_set[deep][idle_skip] = true;
    }
    const int grid = min(persist_grid(), grid_for(r_max, E, 256, ntn));
    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), smem, s, static_cast<const uint8_t*>(A), offsets, E, N, K,
                       static_cast<const uint8_t*>(B0), static_cast<const uint8_t*>(B1), C, ntn, s0, s1, s2, amax);
}

}  // namespace

void set_fp8_deep_b(int v) { g_fp8_deep_b = v; }

bool fp8_ffn_supported(int H, int F) { return H % 128 == 0 && F % 128 == 0 && H >= 256 && F >= 256; }

void launch_expert_ffn_fp8(const void* x_perm, const int32_t* offsets, int r_max, int H, int F, int E,
                           const void* w_gate, const void* w_up, const void* w_down, float dq_gate, float dq_up,
                           float scale_h, float dq_down, void* h, float* amax_h, void* y_perm, int phase,
                           hipStream_t s) {
    if (phase & 1)
        launch_fp8<true>(x_perm, offsets, r_max, E, F, H, w_gate, w_up, h, dq_gate, dq_up, scale_h, amax_h, s);
    if (phase & 2)
        launch_fp8<false>(h, offsets, r_max, E, H, F, w_down, nullptr, y_perm, dq_down, 0.f, 0.f, nullptr, s);
}

}  // namespace moe
