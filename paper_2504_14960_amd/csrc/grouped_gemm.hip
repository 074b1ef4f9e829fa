// a3. Grouped SwiGLU expert FFN (Section 3.1.2 "Expert Computation"; f_e of
// Eq. 1): for every expert e, over its contiguous rows,
//     h = silu(X_e W_gate,e^T) * (X_e W_up,e^T),   Y_e = h W_down,e^T.
//
// Both products are "NT" GEMMs (activations [rows, K] and weights [N, K] are
// both contiguous along the contraction index), which is exactly the operand
// order the gfx950 bf16 MFMA wants: each lane feeds 8 consecutive-K values.
//
// Fast path (bf16): one workgroup per (expert, M-tile, N-tile).  A and B tiles
// are staged in LDS in 16-byte chunks whose position inside a row is XOR-ed
// with the row number, so the 16-byte fragment reads of 32 different rows hit
// different banks.  Two LDS stages; the next tile is fetched (through registers
// or with direct global->LDS loads) while the current one feeds
// v_mfma_f32_32x32x16_bf16.  The MFMA is issued with the weight fragment as its
// first operand, which leaves each lane holding 4 consecutive output columns of
// one row, so the epilogue stores 8-byte packed bf16.  For the first GEMM a
// B-tile holds 128 gate rows and the 128 matching up rows and every wave owns
// the same feature range of both, so silu(g)*u happens in registers and only h
// is written.
//
// Ragged scheduling: the per-expert row offsets live in device memory.  Every
// workgroup scans them (E <= 256), derives the real number of tiles and maps
// its block id to a tile so that (a) the 8 XCDs get equal contiguous shares of
// the REAL tiles and (b) the ~32 tiles an XCD runs at once form a compact
// (M-group x N-range) block that shares A and B panels in that XCD's L2.
#include "gemm_tile.h"

namespace moe {

namespace {

// ---------------------------------------------------------------------------
// bf16 MFMA kernel.
//   A  [rows, K] row-major (lda = K), rows of expert e = [offsets[e], offsets[e+1])
//   B0 [E, N, K], B1 [E, N, K] (SWIGLU: gate and up; else B1 unused)
//   C  [rows, N] bf16
// BN counts B-tile rows: for SWIGLU BN/2 gate rows + BN/2 up rows, producing
// BN/2 output columns; else BN output columns.
// DIRECT: fetch tiles with global->LDS loads (no staging registers).
template <int BM, int BN, int BK, int WGM, int WGN, bool SWIGLU, bool DIRECT>
__global__ __launch_bounds__(WGM* WGN * 64) void gemm_bf16_kernel(
    const bf16_t* __restrict__ A, const int32_t* __restrict__ offsets, int E, int N, int K,
    const bf16_t* __restrict__ B0, const bf16_t* __restrict__ B1, bf16_t* __restrict__ C, int ntn) {
    constexpr int NT = WGM * WGN * 64;
    constexpr int WM = BM / WGM, WN = BN / WGN;
    constexpr int FM = WM / 32, FN = WN / 32;
    constexpr int CPR = BK / 8;                  // 16-byte chunks per tile row
    constexpr int RPP = NT / CPR;                // tile rows fetched per pass
    constexpr int PA = BM / RPP, PB = BN / RPP;  // passes
    constexpr int KS = BK / 16;                  // MFMA k-steps per tile
    constexpr int ROWB = BK * 2;                 // bytes per tile row
    constexpr int A_BYTES = BM * ROWB, B_BYTES = BN * ROWB;
    constexpr int STAGE = A_BYTES + B_BYTES;
    constexpr int OUTN = SWIGLU ? BN / 2 : BN;   // output columns per tile
    static_assert(BM % RPP == 0 && BN % RPP == 0, "tile rows must divide into fetch passes");
    static_assert(!SWIGLU || (FN % 2 == 0), "SwiGLU needs gate and up fragments in one wave");
    static_assert(BK == 64 || BK == 32, "swizzle written for 64- or 128-byte rows");

    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
    __shared__ int sched[kMaxExperts + 2];

    const Tile tile = find_tile<BM>(offsets, E, ntn, sched);
    if (!tile.valid) return;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int n0 = tile.ntile * OUTN;  // first output column of the tile

    auto swz = [](int row) -> int { return (BK == 64) ? (row & 7) : ((row >> 1) & 3); };

    // ---- global source pointers of this thread's fetch slots ----
    // slot p covers tile row (p*RPP + tid/CPR), physical chunk tid%CPR; it reads
    // the logical chunk (phys ^ swz(row)) so that LDS holds the swizzled layout.
    const int frow = tid / CPR, fchunk = tid % CPR;
    const bf16_t* a_src[PA];
    const bf16_t* b_src[PB];
#pragma unroll
    for (int p = 0; p < PA; ++p) {
        const int r = p * RPP + frow;
        int grow = tile.row0 + r;
        grow = min(grow, tile.row_end - 1);  // ragged tail: re-read a valid row, result discarded
        a_src[p] = A + (size_t)grow * K + ((fchunk ^ swz(r)) * 8);
    }
#pragma unroll
    for (int p = 0; p < PB; ++p) {
        const int r = p * RPP + frow;
        const bf16_t* base;
        int feat;
        if (SWIGLU) {
            base = (r < BN / 2) ? B0 : B1;
            feat = n0 + (r % (BN / 2));
        } else {
            base = B0;
            feat = n0 + r;
        }
        feat = min(feat, N - 1);
        b_src[p] = base + ((size_t)tile.expert * N + feat) * K + ((fchunk ^ swz(r)) * 8);
    }
    const int lds_slot = frow * ROWB + fchunk * 16;  // + p*RPP*ROWB (+ A_BYTES for B)

    u32x4 ra[DIRECT ? 1 : PA], rb[DIRECT ? 1 : PB];
    auto fetch = [&](int kt, int stage) {
        const int k0 = kt * BK;
        if (DIRECT) {
            uint8_t* sa = smem + stage * STAGE;
            // every wave-wide load fills 1 KiB of consecutive LDS bytes: the LDS
            // base passed is the wave's (lane 0's) slot
            const int wbase = (wave * 64 / CPR) * ROWB;
#pragma unroll
            for (int p = 0; p < PA; ++p)
                __builtin_amdgcn_global_load_lds(
                    (const __attribute__((address_space(1))) void*)(a_src[p] + k0),
                    (__attribute__((address_space(3))) void*)(sa + p * RPP * ROWB + wbase), 16, 0, 0);
#pragma unroll
            for (int p = 0; p < PB; ++p)
                __builtin_amdgcn_global_load_lds(
                    (const __attribute__((address_space(1))) void*)(b_src[p] + k0),
                    (__attribute__((address_space(3))) void*)(sa + A_BYTES + p * RPP * ROWB + wbase), 16, 0, 0);
        } else {
#pragma unroll
            for (int p = 0; p < PA; ++p) ra[p] = *reinterpret_cast<const u32x4*>(a_src[p] + k0);
#pragma unroll
            for (int p = 0; p < PB; ++p) rb[p] = *reinterpret_cast<const u32x4*>(b_src[p] + k0);
        }
    };
    auto stash = [&](int stage) {
        if (!DIRECT) {
            uint8_t* sa = smem + stage * STAGE;
#pragma unroll
            for (int p = 0; p < PA; ++p)
                *reinterpret_cast<u32x4*>(sa + p * RPP * ROWB + lds_slot) = ra[p];
#pragma unroll
            for (int p = 0; p < PB; ++p)
                *reinterpret_cast<u32x4*>(sa + A_BYTES + p * RPP * ROWB + lds_slot) = rb[p];
        }
    };

    // ---- fragment addressing ----
    // lane l reads, for k-step s, chunk (2s + l/32) of tile row (frag row0 + l%32)
    const int fr = lane & 31, fk = lane >> 5;
    int a_off[FM], b_off[FN];
    int a_sw[FM], b_sw[FN];
#pragma unroll
    for (int i = 0; i < FM; ++i) {
        const int r = wm * WM + i * 32 + fr;
        a_off[i] = r * ROWB;
        a_sw[i] = swz(r);
    }
#pragma unroll
    for (int j = 0; j < FN; ++j) {
        int r;
        if (SWIGLU) {
            const int half = FN / 2;  // fragments 0..half-1 gate, half..FN-1 up, same features
            r = (j < half) ? (wn * (WN / 2) + j * 32 + fr) : (BN / 2 + wn * (WN / 2) + (j - half) * 32 + fr);
        } else {
            r = wn * WN + j * 32 + fr;
        }
        b_off[j] = A_BYTES + r * ROWB;
        b_sw[j] = swz(r);
    }

    f32x16 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int KT = K / BK;
    fetch(0, 0);
    stash(0);
    if (DIRECT) wait_vmcnt0();
    __syncthreads();

    for (int kt = 0; kt < KT; ++kt) {
        const int stage = kt & 1;
        if (kt + 1 < KT) fetch(kt + 1, stage ^ 1);
        const uint8_t* sa = smem + stage * STAGE;
        bf16x8 af[2][FM], bfg[2][FN];
        auto read_frags = [&](int s, int buf) {
            const int c = 2 * s + fk;
#pragma unroll
            for (int i = 0; i < FM; ++i)
                af[buf][i] = __builtin_bit_cast(
                    bf16x8, *reinterpret_cast<const u32x4*>(sa + a_off[i] + ((c ^ a_sw[i]) << 4)));
#pragma unroll
            for (int j = 0; j < FN; ++j)
                bfg[buf][j] = __builtin_bit_cast(
                    bf16x8, *reinterpret_cast<const u32x4*>(sa + b_off[j] + ((c ^ b_sw[j]) << 4)));
        };
        read_frags(0, 0);
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            if (s + 1 < KS) read_frags(s + 1, (s + 1) & 1);
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfg[s & 1][j], af[s & 1][i],
                                                                         acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < KT) {
            stash(stage ^ 1);
            if (DIRECT) wait_vmcnt0();
        }
        __syncthreads();
    }

    store_tile<FM, FN, WM, WN, BN, SWIGLU>(acc, tile, C, N, n0, wm, wn, lane);
}

// ---------------------------------------------------------------------------
// Plain tiled kernel for fp32 layers and for bf16 shapes the MFMA kernel does
// not take (K not a multiple of 64).  64x64 outputs per workgroup, 16-wide K
// slices in LDS, 4x4 outputs per thread, fp32 FMA.  Every access is guarded.
template <typename TIn, bool SWIGLU>
__global__ __launch_bounds__(256) void gemm_simple_kernel(
    const TIn* __restrict__ A, const int32_t* __restrict__ offsets, int E, int N, int K,
    const TIn* __restrict__ B0, const TIn* __restrict__ B1, TIn* __restrict__ C, int ntn) {
    constexpr int BM = 64, BN = 64, BK = 16;
    __shared__ float As[BK][BM + 4];
    __shared__ float Bs[SWIGLU ? 2 : 1][BK][BN + 4];
    __shared__ int sched[kMaxExperts + 2];
    const Tile tile = find_tile<BM>(offsets, E, ntn, sched);
    if (!tile.valid) return;
    const int tid = threadIdx.x;
    const int tx = tid % 16, ty = tid / 16;
    const int n0 = tile.ntile * BN;
    auto ldv = [](const TIn* p) -> float {
        if constexpr (sizeof(TIn) == 2) return bf16_to_f32(*reinterpret_cast<const bf16_t*>(p));
        else return *reinterpret_cast<const float*>(p);
    };
    float acc[SWIGLU ? 2 : 1][4][4];
#pragma unroll
    for (int z = 0; z < (SWIGLU ? 2 : 1); ++z)
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[z][i][j] = 0.f;

    for (int k0 = 0; k0 < K; k0 += BK) {
        for (int i = tid; i < BM * BK; i += 256) {
            const int r = i / BK, k = i % BK;
            float v = 0.f;
            if (r < tile.rows && k0 + k < K) v = ldv(A + (size_t)(tile.row0 + r) * K + k0 + k);
            As[k][r] = v;
        }
        for (int i = tid; i < BN * BK; i += 256) {
            const int r = i / BK, k = i % BK;
            float v0 = 0.f, v1 = 0.f;
            if (n0 + r < N && k0 + k < K) {
                const size_t at = ((size_t)tile.expert * N + n0 + r) * K + k0 + k;
                v0 = ldv(B0 + at);
                if (SWIGLU) v1 = ldv(B1 + at);
            }
            Bs[0][k][r] = v0;
            if (SWIGLU) Bs[SWIGLU ? 1 : 0][k][r] = v1;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < BK; ++k) {
            float a[4], b[SWIGLU ? 2 : 1][4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[k][ty * 4 + i];
#pragma unroll
            for (int z = 0; z < (SWIGLU ? 2 : 1); ++z)
#pragma unroll
                for (int j = 0; j < 4; ++j) b[z][j] = Bs[z][k][tx * 4 + j];
#pragma unroll
            for (int z = 0; z < (SWIGLU ? 2 : 1); ++z)
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[z][i][j] = fmaf(a[i], b[z][j], acc[z][i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = ty * 4 + i;
        if (r >= tile.rows) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int col = n0 + tx * 4 + j;
            if (col >= N) continue;
            float v;
            if (SWIGLU) {
                const float g = acc[0][i][j];
                v = (g / (1.f + expf(-g))) * acc[SWIGLU ? 1 : 0][i][j];
            } else {
                v = acc[0][i][j];
            }
            TIn* dst = C + (size_t)(tile.row0 + r) * N + col;
            if constexpr (sizeof(TIn) == 2) *reinterpret_cast<bf16_t*>(dst) = f32_to_bf16(v);
            else *reinterpret_cast<float*>(dst) = v;
        }
    }
}

template <int BM, int BN, int BK, int WGM, int WGN, bool SWIGLU, bool DIRECT>
void launch_bf16_gemm(const void* A, const int32_t* offsets, int r_max, int E, int N, int K,
                      const void* B0, const void* B1, void* C, hipStream_t s) {
    constexpr int OUTN = SWIGLU ? BN / 2 : BN;
    constexpr size_t smem = 2 * (size_t)(BM + BN) * BK * 2;
    const int ntn = (N + OUTN - 1) / OUTN;
    auto kern = gemm_bf16_kernel<BM, BN, BK, WGM, WGN, SWIGLU, DIRECT>;
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        attr_set = true;
    }
    const int grid = grid_for(r_max, E, BM, ntn);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(WGM * WGN * 64), smem, s,
                       static_cast<const bf16_t*>(A), offsets, E, N, K,
                       static_cast<const bf16_t*>(B0), static_cast<const bf16_t*>(B1),
                       static_cast<bf16_t*>(C), ntn);
}

template <typename TIn, bool SWIGLU>
void launch_simple_gemm(const void* A, const int32_t* offsets, int r_max, int E, int N, int K,
                        const void* B0, const void* B1, void* C, hipStream_t s) {
    const int ntn = (N + 63) / 64;
    const int grid = grid_for(r_max, E, 64, ntn);
    hipLaunchKernelGGL((gemm_simple_kernel<TIn, SWIGLU>), dim3(grid), dim3(256), 0, s,
                       static_cast<const TIn*>(A), offsets, E, N, K, static_cast<const TIn*>(B0),
                       static_cast<const TIn*>(B1), static_cast<TIn*>(C), ntn);
}

template <int BM, int BN, int BK, int WGM, int WGN, bool DIRECT>
void run_pair(const void* x_perm, const int32_t* offsets, int r_max, int H, int F, int E,
              const void* w_gate, const void* w_up, const void* w_down, void* h, void* y_perm,
              int phase, hipStream_t s) {
    if (phase & 1) launch_bf16_gemm<BM, BN, BK, WGM, WGN, true, DIRECT>(x_perm, offsets, r_max, E, F, H, w_gate, w_up, h, s);
    if (phase & 2) launch_bf16_gemm<BM, BN, BK, WGM, WGN, false, DIRECT>(h, offsets, r_max, E, H, F, w_down, nullptr, y_perm, s);
}

}  // namespace

bool launch_expert_ffn(const void* x_perm, const int32_t* offsets, int r_max, int H, int F, int E,
                       const void* w_gate, const void* w_up, const void* w_down, moe_dtype_t dt,
                       void* h, void* y_perm, int variant, int phase, hipStream_t s) {
    if (dt == MOE_F32) {
        if (phase & 1) launch_simple_gemm<float, true>(x_perm, offsets, r_max, E, F, H, w_gate, w_up, h, s);
        if (phase & 2) launch_simple_gemm<float, false>(h, offsets, r_max, E, H, F, w_down, nullptr, y_perm, s);
        return true;
    }
    const bool fast = (H % 64 == 0) && (F % 64 == 0);
    if (!fast || variant == 99) {
        if (phase & 1) launch_simple_gemm<bf16_t, true>(x_perm, offsets, r_max, E, F, H, w_gate, w_up, h, s);
        if (phase & 2) launch_simple_gemm<bf16_t, false>(h, offsets, r_max, E, H, F, w_down, nullptr, y_perm, s);
        return true;
    }
    if (variant == 0) {
        // tuned default (Mixtral-8x22B layer shape on MI355X): the persistent 8-wave
        // kernel for both GEMMs; layers too shallow for its k stream fall back to the
        // kernels with three activation stages (8 waves gate/up, 4 waves down)
        if (launch_persist_ffn(x_perm, offsets, r_max, H, F, E, w_gate, w_up, w_down, h, y_perm, 41, phase, s))
            return true;
        bool ok = true;
        if (phase & 1) ok = ok && launch_pipe3_ffn(x_perm, offsets, r_max, H, F, E, w_gate, w_up, w_down, h, y_perm, 31, 1, s);
        if (phase & 2) ok = ok && launch_pipe3_ffn(x_perm, offsets, r_max, H, F, E, w_gate, w_up, w_down, h, y_perm, 30, 2, s);
        return ok;
    }
    if (variant >= 40 && launch_persist_ffn(x_perm, offsets, r_max, H, F, E, w_gate, w_up, w_down, h, y_perm, variant, phase, s))
        return true;
    if (variant >= 30 && launch_pipe3_ffn(x_perm, offsets, r_max, H, F, E, w_gate, w_up, w_down, h, y_perm, variant, phase, s))
        return true;
    // baseline kernel: two LDS stages, one workgroup per tile
    switch (variant) {
        default:
        case 1: run_pair<256, 256, 64, 2, 2, false>(x_perm, offsets, r_max, H, F, E, w_gate, w_up, w_down, h, y_perm, phase, s); break;
        case 2: run_pair<256, 256, 64, 2, 2, true>(x_perm, offsets, r_max, H, F, E, w_gate, w_up, w_down, h, y_perm, phase, s); break;
        case 5: run_pair<128, 256, 64, 2, 2, false>(x_perm, offsets, r_max, H, F, E, w_gate, w_up, w_down, h, y_perm, phase, s); break;
        case 7: run_pair<128, 128, 64, 2, 2, false>(x_perm, offsets, r_max, H, F, E, w_gate, w_up, w_down, h, y_perm, phase, s); break;
    }
    return true;
}

}  // namespace moe
