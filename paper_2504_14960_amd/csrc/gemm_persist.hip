// Grouped expert GEMM (a3), persistent kernel: one workgroup per compute unit
// walks a static list of output tiles and treats their k-tiles as ONE stream.
//
// Same tile engine as gemm_pipe3.hip (256 x 256 x 64 tiles, three LDS stages
// for the activation tile and two for the weight tile, direct global->LDS
// loads spread in source order between the MFMA groups, one barrier per
// k-tile).  What changes is what happens at a tile boundary:
//
//  * the loads issued during the last two k-tiles of a tile already fetch the
//    first two k-tiles of the workgroup's NEXT tile, so the pipeline never
//    drains and there is no per-tile prologue;
//  * the tile scheduler (prefix of per-expert M-tile counts) lives in registers
//    of every wave and is evaluated with wave-level operations only: no LDS, no
//    barrier, no memory access per tile;
//  * the epilogue goes through the one LDS stage that is idle at that moment:
//    every wave transposes its accumulators through a private, XOR-swizzled
//    patch of it and writes whole 16-byte-per-lane row segments, instead of
//    8-byte pieces scattered over 32 rows per store instruction.
//
// The workgroups never wait for one another, so any number of them may be
// resident; the launcher asks for one per compute unit.
#include <type_traits>

#include "gemm_persist.h"


namespace moe {

static int g_persist_workgroups = 0;  // 0: one per compute unit
static int g_persist_idle_skip = -1;  // -1: chosen from the expert count; 0 / 1: forced
static unsigned long long* g_persist_ticks = nullptr;  // device cell pair of the clock sample, or none

int persist_grid() {
    // every one of the 8 tile shares needs a workgroup with its residue mod 8
    if (g_persist_workgroups > 0) return g_persist_workgroups < 8 ? 8 : g_persist_workgroups;
    static int cus = 0;
    if (!cus) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess)
            cus = prop.multiProcessorCount;
        if (cus < 8) cus = 256;
    }
    return cus;
}

namespace {

// Epilogue through LDS.  For fragment row block i the wave writes its 32 x
// (32*FO) bf16 outputs (8 bytes per lane per store: row l%32, 4 consecutive
// columns) into a private patch of W = 64*FO bytes per row, 16-byte granules
// XOR-swizzled by the row so that neither side has bank conflicts, reads them
// back as whole 16-byte granules along the rows and stores those.
//
// MODE 0: C = acc.  MODE 1: C = silu(gate) * up, the gate in the first half of
// the fragments and the up projection in the second.  MODE 2: as 1, and the
// two pre-activations themselves go to GU [rows, 2N] (gate in columns
// [0, N), up in [N, 2N)) for a backward pass that does not recompute them.
template <int FM, int FN, int WM, int MODE, bool ACC_IN_AGPR>
__device__ __forceinline__ void store_tile_staged(f32x16 (&acc)[FM][FN], int t_row0, int t_rows, int t_n0,
                                                  bf16_t* __restrict__ C, bf16_t* __restrict__ GU, int N, int wm,
                                                  int wn, int lane, uint8_t* stage) {
    constexpr bool SWIGLU = MODE == 1 || MODE == 2;
    constexpr int FO = SWIGLU ? FN / 2 : FN;
    constexpr int W = FO * 64;        // bytes per staged row
    constexpr int GPR = W / 16;       // granules per row
    constexpr int RP256 = 256 / W;    // rows per 256 bytes (one pass over all banks)
    constexpr int RPI = 1024 / W;     // rows per 64-lane read
    static_assert(W <= 256 && 256 % W == 0, "staged row must divide the bank window");
    // the lane-dependent addresses below are cheap to recompute per tile; hiding
    // the lane id keeps them from being hoisted out of the tile loop, where they
    // would occupy registers across the whole k loop
    asm volatile("" : "+v"(lane));
    const int fr = lane & 31, fk = lane >> 5;
    const int xw = (fr / RP256) & (GPR - 1);
    uint8_t* wrow = stage + fr * W + 8 * fk;
    const int rl = lane / GPR, gl = lane % GPR;
    const int col = t_n0 + wn * (FO * 32) + gl * 8;
#pragma unroll
    for (int i = 0; i < FM; ++i) {
        // one row block at a time.  With 256 accumulators per lane they live in
        // the accumulation registers; naming them there once more per block keeps
        // the copies into ordinary registers from being made all at once, which
        // would push the loop's long-lived values out to scratch memory
        __builtin_amdgcn_sched_barrier(0);
        if (ACC_IN_AGPR) {
#pragma unroll
            for (int j = 0; j < FN; ++j) asm volatile("" : "+a"(acc[i][j]));
        }
        if (MODE == 2) {
            // the pre-activations first: gate half, then up half, each through the same patch
#pragma unroll
            for (int half = 0; half < 2; ++half) {
#pragma unroll
                for (int j = 0; j < FO; ++j) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const f32x16& a = acc[i][j + half * FO];
                        u32x2 o;
                        o[0] = pack2_bf16(a[4 * q], a[4 * q + 1]);
                        o[1] = pack2_bf16(a[4 * q + 2], a[4 * q + 3]);
                        *reinterpret_cast<u32x2*>(wrow + (((4 * j + q) ^ xw) << 4)) = o;
                    }
                }
#pragma unroll
                for (int it = 0; it < 32 / RPI; ++it) {
                    const int row = it * RPI + rl;
                    const int xr = (row / RP256) & (GPR - 1);
                    const u32x4 v = *reinterpret_cast<const u32x4*>(stage + row * W + ((gl ^ xr) << 4));
                    const int grow = wm * WM + i * 32 + row;
                    if (grow < t_rows && col < N)
                        *reinterpret_cast<u32x4*>(GU + (size_t)(t_row0 + grow) * (2 * N) + half * N + col) = v;
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
#pragma unroll
        for (int j = 0; j < FO; ++j) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float v[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    if (SWIGLU) {
                        const float g = acc[i][j][4 * q + u];
                        const float up = acc[i][j + FO][4 * q + u];
                        v[u] = g * __builtin_amdgcn_rcpf(1.f + __expf(-g)) * up;  // silu(g) * up
                    } else {
                        v[u] = acc[i][j][4 * q + u];
                    }
                }
                u32x2 o;
                o[0] = pack2_bf16(v[0], v[1]);
                o[1] = pack2_bf16(v[2], v[3]);
                *reinterpret_cast<u32x2*>(wrow + (((4 * j + q) ^ xw) << 4)) = o;
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        if (MODE == 3) {
            // the saved pre-activations of this row block first (their addresses do not depend on the staging)
            u32x4 gv[32 / RPI], uv[32 / RPI];
#pragma unroll
            for (int it = 0; it < 32 / RPI; ++it) {
                const int grow = wm * WM + i * 32 + it * RPI + rl;
                gv[it] = u32x4{0u, 0u, 0u, 0u};
                uv[it] = u32x4{0u, 0u, 0u, 0u};
                if (grow < t_rows && col < N) {
                    const bf16_t* src = GU + (size_t)(t_row0 + grow) * (2 * N) + col;
                    gv[it] = *reinterpret_cast<const u32x4*>(src);
                    uv[it] = *reinterpret_cast<const u32x4*>(src + N);
                }
            }
#pragma unroll
            for (int it = 0; it < 32 / RPI; ++it) {
                const int row = it * RPI + rl;
                const int xr = (row / RP256) & (GPR - 1);
                const u32x4 v = *reinterpret_cast<const u32x4*>(stage + row * W + ((gl ^ xr) << 4));
                const int grow = wm * WM + i * 32 + row;
                u32x4 og, ou;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    float dgv[2], duv[2];
#pragma unroll
                    for (int hlf = 0; hlf < 2; ++hlf) {
                        const float dh = __uint_as_float(hlf ? (v[j] & 0xffff0000u) : (v[j] << 16));
                        const float g = __uint_as_float(hlf ? (gv[it][j] & 0xffff0000u) : (gv[it][j] << 16));
                        const float up = __uint_as_float(hlf ? (uv[it][j] & 0xffff0000u) : (uv[it][j] << 16));
                        const float sg = __builtin_amdgcn_rcpf(1.f + __expf(-g));
                        duv[hlf] = dh * g * sg;
                        dgv[hlf] = dh * up * sg * (1.f + g * (1.f - sg));
                    }
                    og[j] = pack2_bf16(dgv[0], dgv[1]);
                    ou[j] = pack2_bf16(duv[0], duv[1]);
                }
                if (grow < t_rows && col < N) {
                    bf16_t* dst = C + (size_t)(t_row0 + grow) * (2 * N) + col;
                    *reinterpret_cast<u32x4*>(dst) = og;
                    *reinterpret_cast<u32x4*>(dst + N) = ou;
                }
            }
        } else {
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
}

// GROUPK (MODE 0 only): the weight-gradient form C [E, M, N]; A and B0 are the
// transposed operands [M, K] and [N, K] with K = elements per row, every expert
// contracting over its own zero-padded column segment (see WgradSched); `ntn`
// carries M.  Experts without rows get no tiles here (their gradient is zeroed
// by wgrad_zero_empty_kernel).
//
// KMAJ (with GROUPK): the same product on the activations AS THE LAYER HOLDS THEM, A [rows, lda] and B0 [rows,
// ldb] row-major (K carries lda), no transposed copies.  A k-tile is then 64 rows x 256 features (512-byte LDS
// rows, 16-byte pieces XOR-swizzled by the row), and a fragment's eight contraction values per lane come from two
// transposing LDS loads (ds_read_b64_tr_b16: the 16 lanes of a group address a 4 x 16 block, four consecutive
// features each, and lane i receives feature i of the four rows).  Both operands are read the same way, so they
// agree on the order of the contraction values.  Rows past the expert's last one are fetched from the zero row
// that GU points at (512 bytes of zeros).
//
// DEEP_B: which operand gets the three LDS stages.  false: the activation tile (three stages, fetched two k-tiles
// ahead) and two stages for the weight tile; true: the other way round -- the weights are what streams in from
// HBM (every weight byte is used by one M-group only), the activation panels are re-read from the caches.
template <int BM, int BN, int WGM, int WGN, int MODE, bool GROUPK = false, bool KMAJ = false, bool IDLE_SKIP = false,
          bool DEEP_B = false, bool BY_ROUND = true>
__global__ __launch_bounds__(WGM* WGN * 64) void gemm_bf16_persist_kernel(
    const bf16_t* __restrict__ A, const int32_t* __restrict__ offsets, int E, int N, int K,
    const bf16_t* __restrict__ B0, const bf16_t* __restrict__ B1, bf16_t* __restrict__ C, bf16_t* __restrict__ GU,
    int ntn, int ldb, unsigned long long* __restrict__ ticks) {
    static_assert(!GROUPK || MODE == 0, "the weight-gradient form has a plain epilogue");
    static_assert(!KMAJ || (GROUPK && BM == 256 && BN == 256 && WGM * WGN == 8), "row-major form: 256 x 256 tiles, 8 waves");
    static_assert(!(KMAJ && DEEP_B), "the row-major form keeps three activation stages");
    constexpr bool SWIGLU = MODE == 1 || MODE == 2;
    constexpr int BK = 64;
    constexpr int NW = WGM * WGN;
    constexpr int NT = NW * 64;
    constexpr int WM = BM / WGM, WN = BN / WGN;
    constexpr int FM = WM / 32, FN = WN / 32;
    constexpr int CPR = BK / 8;
    constexpr int RPP = NT / CPR;               // tile rows fetched per pass of the workgroup
    constexpr int PA = BM / RPP, PB = BN / RPP;
    constexpr int ROWB = BK * 2;
    constexpr int A_BYTES = BM * ROWB, B_BYTES = BN * ROWB;
    constexpr int B_REGION = (DEEP_B ? 2 : 3) * A_BYTES;   // the activation slots, then the weight slots
    // "early" operand: two slots, fetched one k-tile ahead, issued first in a period; "late" operand: three
    // slots, fetched two k-tiles ahead
    constexpr int PE = DEEP_B ? PA : PB, PL = DEEP_B ? PB : PA;
    constexpr int OUTN = SWIGLU ? BN / 2 : BN;
    constexpr int NLOAD = PA + PB;              // direct loads per thread per k-tile (early operand first)
    constexpr int NREAD = FM + FN;
    constexpr int NMFMA = FM * FN;
    constexpr int NSLOT = NREAD;
    constexpr int MPS = NMFMA / NSLOT;
    // a period's loads are spread over the k-steps 3 (of the previous k-tile), 0 and 1
    constexpr int LA = NLOAD / 3;
    constexpr int LB = LA + (NLOAD - LA + 1) / 2;
    constexpr int LC = NLOAD;
    // fragment reads per slot of a k-step: one (spread over the whole k-step) with eight waves, whose LDS pipe is
    // as busy as the matrix pipe; two with four waves
    constexpr int RDPS = NW == 8 ? 1 : 2;
    constexpr int FO = SWIGLU ? FN / 2 : FN;
    static_assert(BM % RPP == 0 && BN % RPP == 0 && RPP % 8 == 0, "tile rows must divide into fetch passes");
    static_assert(!SWIGLU || ((BN / 2) % RPP == 0 && FN % 2 == 0), "gate/up halves must be pass- and fragment-aligned");
    static_assert(LA <= PE, "only loads of the early operand may be issued under k-step 3");
    static_assert(LB - LA <= NSLOT && LC - LB <= NSLOT && LA <= NSLOT, "not enough slots for the loads");
    static_assert(PL < 64, "vmcnt holds 6 bits");
    static_assert(3 * A_BYTES + 2 * B_BYTES <= 160 * 1024, "tile stages exceed the 160 KiB of LDS");
    static_assert(NW * 32 * FO * 64 <= (DEEP_B ? B_BYTES : A_BYTES), "epilogue patches must fit into one slot of the late operand");

    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
    // clock sample (ticks != NULL): shader-clock and 100 MHz reference ticks workgroup 0 spends in the kernel
    const bool sample = ticks != nullptr && blockIdx.x == 0;
    unsigned long long tk_entry = 0, rt_entry = 0;
    if (sample) {
        tk_entry = __builtin_amdgcn_s_memtime();
        rt_entry = __builtin_amdgcn_s_memrealtime();
    }

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WGN, wn = wave % WGN;

    const uint8_t* const Ab = reinterpret_cast<const uint8_t*>(A);
    const uint8_t* const B0b = reinterpret_cast<const uint8_t*>(B0);
    const uint8_t* const B1b = SWIGLU ? reinterpret_cast<const uint8_t*>(B1) : B0b;

    // tiles are dealt to the XCDs round by round, except in the many-expert instantiations (measured: there the
    // gate/up GEMM loses 1 %, and the two GEMMs of a layer must walk the rows in the same order)
    typename std::conditional<KMAJ, WgradSchedKM<BM, BN>,
                              typename std::conditional<GROUPK, WgradSched<BM, BN>, TileSched<BM, BY_ROUND>>::type>::type sched;
    if constexpr (GROUPK)
        sched.init(offsets, E, ntn, N, lane);
    else
        sched.init(offsets, E, ntn, lane);
    auto get_tile = [&](int i) -> PTile {
        if constexpr (KMAJ)
            return sched.get(i, Ab, B0b, ntn, N, K, ldb);
        else if constexpr (GROUPK)
            return sched.get(i, Ab, B0b, ntn, N, K);
        else
            return sched.get(i, Ab, B0b, B1b, N, (size_t)K * 2, OUTN);
    };
    // current and next tile of this workgroup, as plain wave-uniform scalars
    int ti = 0;
    const uint8_t *c_a, *c_b0, *c_b1, *n_a, *n_b0, *n_b1;
    uint32_t c_alim, c_blim, n_alim, n_blim;
    int c_row0, c_rows, c_n0, n_row0, n_rows, n_n0;
    int c_kt = K / BK, n_kt = K / BK;   // k-tiles per output tile: per tile in the weight-gradient form
    int c_krows = 0, n_krows = 0;       // row-major form: rows of the tile's expert
    bool n_valid;
    {
        const PTile t = get_tile(0);
        if (!t.valid) return;
        c_a = t.a; c_b0 = t.b0; c_b1 = t.b1; c_alim = t.a_lim; c_blim = t.b_lim;
        c_row0 = t.row0; c_rows = t.rows; c_n0 = t.n0;
        if (GROUPK) c_kt = t.kt;
        if (KMAJ) c_krows = t.krows;
    }
    auto fetch_next_tile = [&](int i) {
        const PTile t = get_tile(i);
        n_a = t.a; n_b0 = t.b0; n_b1 = t.b1; n_alim = t.a_lim; n_blim = t.b_lim;
        n_row0 = t.row0; n_rows = t.rows; n_n0 = t.n0; n_valid = t.valid;
        if (GROUPK) n_kt = t.kt;
        if (KMAJ) n_krows = t.krows;
    };
    fetch_next_tile(1);

    // global side of the direct loads: thread (frow, fchunk) of a pass fetches
    // 16 bytes of tile row p*RPP + frow; the chunk it asks for is XOR-swizzled
    // so that the LDS side can stay linear (lane * 16 bytes)
    const int frow = tid / CPR, fchunk = tid % CPR;
    const uint32_t k2 = (uint32_t)K * 2u;
    const uint32_t vrow = (uint32_t)frow * k2;
    const uint32_t vswz = (uint32_t)((fchunk ^ lds_swizzle(frow)) * 16);   // every pass starts at a multiple of 16 rows
    const uint32_t step = (uint32_t)RPP * k2;
    const int wbase = (wave * 64 / CPR) * ROWB;

    // row-major form: a pass covers 16 rows of 512 bytes; thread = (row tid / 32, piece tid % 32); the piece it asks
    // for is XOR-swizzled by the row in units of 32 bytes: a 16-lane group of a transposing read touches 32 bytes
    // of four consecutive rows, which then lie in the four different quarters of the 128-byte bank window
    const int km_row = tid >> 5;
    const uint32_t km_piece = (uint32_t)(((tid & 31) ^ (2 * (km_row & 3))) * 16);
    const uint8_t* const zero_row = reinterpret_cast<const uint8_t*>(GU) + (tid & 31) * 16;
    auto fetch_km = [&](int p, const uint8_t* base, uint32_t ld2, uint32_t lim, int rows_left, uint8_t* st) {
        const int krow = 16 * p + km_row;
        const uint8_t* src = base + (uint32_t)krow * ld2 + min(km_piece, lim);
        if (krow >= rows_left) src = zero_row;   // past the expert's last row: contributes nothing
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                         (__attribute__((address_space(3))) void*)(st + p * RPP * ROWB + wbase), 16,
                                         0, 0);
    };
    auto fetch_a = [&](int p, const uint8_t* base, uint32_t lim, uint8_t* st) {
        const uint32_t off = min(vrow + (uint32_t)p * step, lim) + vswz;  // ragged tail: a valid row again
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
    // where k-tile kk of the stream that starts at cur's k-tile 0 comes from
    struct Src {
        const uint8_t* a;
        const uint8_t* b0;
        const uint8_t* b1;
        uint32_t a_lim, b_lim;
        int rows_left;   // row-major form: valid rows from this k-tile's first row on
    };
    // every tile has at least two k-tiles, so k-tile KT + 1 of the stream is the next tile's second
    auto src = [&](int kk) -> Src {
        const int KT = c_kt;
        const bool in_cur = kk < KT;
        const bool use_cur = in_cur || !n_valid;  // past the last tile: its last k-tile again, never used
        const int k = in_cur ? kk : (n_valid ? kk - KT : KT - 1);
        // a k-tile is 64 elements along the rows, or (row-major form) 64 rows
        const size_t kbyte_a = KMAJ ? (size_t)k * 64 * ((size_t)K * 2) : (size_t)k * (BK * 2);
        const size_t kbyte_b = KMAJ ? (size_t)k * 64 * ((size_t)ldb * 2) : (size_t)k * (BK * 2);
        Src s;
        s.a = (use_cur ? c_a : n_a) + kbyte_a;
        s.b0 = (use_cur ? c_b0 : n_b0) + kbyte_b;
        s.b1 = (use_cur ? c_b1 : n_b1) + kbyte_b;
        s.a_lim = use_cur ? c_alim : n_alim;
        s.b_lim = use_cur ? c_blim : n_blim;
        s.rows_left = KMAJ ? (use_cur ? c_krows : n_krows) - k * 64 : 0;
        return s;
    };
    // load i of a period: i < PE -> pass i of the early operand's tile (source se), else pass i - PE of the late
    // operand's (source sl); ld_b / ld_a: the weight / activation slot being filled
    auto fetch_one = [&](int i, const Src& se, const Src& sl, uint8_t* ld_b, uint8_t* ld_a) {
        if constexpr (KMAJ) {
            if (i < PB)
                fetch_km(i, se.b0, (uint32_t)ldb * 2u, se.b_lim, se.rows_left, ld_b);
            else
                fetch_km(i - PB, sl.a, k2, sl.a_lim, sl.rows_left, ld_a);
        } else if constexpr (DEEP_B) {
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
    const int f_sw = lds_swizzle(fr);  // fragments start at multiples of 32 rows
    if constexpr (KMAJ) {
        // lane (group g = lane / 16, s = lane % 16) addresses row 4 (g / 2) + s / 4 of an 8-row block, features
        // 16 (g % 2) + 4 (s % 4) .. + 3 of the fragment's 32; its row decides the swizzle of the 64-byte unit
        const int g = lane >> 4, sl = lane & 15;
        const int r8 = 4 * (g >> 1) + (sl >> 2);
        const int piece_in = 2 * (g & 1) + ((sl & 3) >> 1);   // 16-byte piece inside the fragment's 64 bytes
        const int byte_in = 8 * (sl & 1);
#pragma unroll
        for (int i = 0; i < FM; ++i)
            a_off[i] = r8 * 512 + ((((wm * WM + i * 32) >> 3) + piece_in) ^ (2 * (r8 & 3))) * 16 + byte_in;
#pragma unroll
        for (int j = 0; j < FN; ++j)
            b_off[j] = r8 * 512 + ((((wn * WN + j * 32) >> 3) + piece_in) ^ (2 * (r8 & 3))) * 16 + byte_in;
    } else {
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
        if constexpr (KMAJ) {
            // k-step s = rows 16 s .. 16 s + 15: one transposing load for its first 8 rows, one for the last 8
            typedef __attribute__((ext_vector_type(4))) short s16x4;
            typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
            const uint8_t* p = (q < FM ? sa + a_off[q] : sb + b_off[q - FM]) + s * (16 * 512);
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p));
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 8 * 512));
            typedef __attribute__((ext_vector_type(8))) short s16x8;
            const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            if (q < FM)
                af[buf][q] = __builtin_bit_cast(bf16x8, v);
            else
                bfg[buf][q - FM] = __builtin_bit_cast(bf16x8, v);
            return;
        }
        const int c = ((2 * s + fk) ^ f_sw) << 4;
        if (q < FM)
            af[buf][q] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(sa + a_off[q] + c));
        else
            bfg[buf][q - FM] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(sb + b_off[q - FM] + c));
    };
    auto mfma_one = [&](int buf, int m) {
        // boustrophedon over the wave's blocks: successive MFMAs share one operand fragment
        const int i = m / FN, j = (i & 1) ? FN - 1 - m % FN : m % FN;
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfg[buf][j], af[buf][i], acc[i][j], 0, 0, 0);
    };
    // one k-step in issue order: NSLOT slots of {MPS MFMAs on set mf_buf; up to
    // 2 fragment reads of k-step rd_s into the other set; one direct load}
    // `aside`: scalar bookkeeping run under the MFMAs of slot 1 (the next period's load sources), so that it does
    // not sit between two k-tiles with the matrix pipe empty
    auto kstep = [&](int mf_buf, const uint8_t* rd_a, const uint8_t* rd_b, int rd_s, int ld_begin, int ld_end,
                     const Src& se, const Src& sl, uint8_t* ld_b, uint8_t* ld_a, auto&& aside) {
        int m = 0, rd = 0, ld = ld_begin;
#pragma unroll
        for (int slot = 0; slot < NSLOT; ++slot) {
#pragma unroll
            for (int q = 0; q < MPS; ++q) {
                mfma_one(mf_buf, m);
                ++m;
            }
            if (slot == 1) aside();
            // the k-step's first MFMA waits (lgkmcnt) for the fragments read during the previous k-step; keep
            // this k-step's reads behind it, or the compiler hoists them and that wait also covers reads issued
            // a moment ago (a full LDS round trip in front of every k-step)
            if (slot == 0) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int q = 0; q < RDPS; ++q)
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
#pragma unroll
        for (int mm = NSLOT * MPS; mm < NMFMA; ++mm) mfma_one(mf_buf, mm);
        __builtin_amdgcn_sched_barrier(0);
    };

    uint8_t* const a_region = smem;
    uint8_t* const b_region = smem + B_REGION;

    // prologue (first tile of this workgroup only): late(0), early(0), then late(1); only the first two must have
    // landed before the first fragment reads
    {
        const Src s0 = src(0), s1 = src(1);
#pragma unroll
        for (int i = PE; i < NLOAD; ++i) fetch_one(i, s0, s0, b_region, a_region);
#pragma unroll
        for (int i = 0; i < PE; ++i) fetch_one(i, s0, s0, b_region, a_region);
#pragma unroll
        for (int i = PE; i < NLOAD; ++i)
            fetch_one(i, s1, s1, b_region + (DEEP_B ? B_BYTES : 0), a_region + (DEEP_B ? 0 : A_BYTES));
        __builtin_amdgcn_s_waitcnt(0x0F70 | (PL & 0xF) | ((PL >> 4) << 14));  // vmcnt(PL)
        __builtin_amdgcn_s_barrier();
#pragma unroll
        for (int q = 0; q < NREAD; ++q) read_one(a_region, b_region, 0, 0, q);
        // head of early(1) into the early operand's slot 1
#pragma unroll
        for (int i = 0; i < LA; ++i) fetch_one(i, s1, s1, b_region + B_BYTES, a_region + A_BYTES);
    }

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
        // (IDLE_SKIP instantiations, chosen for launches with many experts, i.e. many ragged tails; the test costs
        // the plain kernel half a per cent.)  A wave whose rows of the tile all lie past the tile's last valid row
        // (ragged tail of an expert) has nothing to multiply: it keeps issuing its share of the loads and meeting the barriers, and leaves the
        // matrix pipe and the LDS reads alone (under a power cap that is clock for the other workgroups).
        const bool wave_idle = IDLE_SKIP && wm * WM >= c_rows;   // wave-uniform
        if (!wave_idle) {
        // sources of the loads of k-tiles kt+1 and kt+2.  With one wave per SIMD (four waves) nothing covers the
        // scalar arithmetic that forms them if it sits between two k-tiles (some fifty instructions with the
        // matrix pipe empty), so there they are carried from period to period: the pair a period needs is the
        // previous period's second source and one computed under the MFMAs of the previous period's k-step 2 (a
        // tile's first period forms its own: the next tile's third k-tile need not exist).  With two waves per
        // SIMD the other wave covers it, and the carried form measured 1.7 % slower; there only the first of the
        // pair is carried and the second is formed at the top of the period.
        constexpr bool CARRY = NW == 4;
        Src s1 = src(1), s2 = src(2), s3 = s2;
        auto nothing = [] {};
        for (int kt = 0; kt < c_kt; ++kt) {
            if constexpr (!CARRY) {
                // the source of k-tile kt+1 is last period's second source; only the new one is formed here
                if (kt > 0) s1 = s2;
                s2 = src(kt + 2);
            }
            const uint8_t* ca = a_region + a0;
            const uint8_t* cb = b_region + b0;
            // this period fills early(kt+1) and late(kt+2)
            uint8_t* lb = b_region + (DEEP_B ? b2 : b1);
            uint8_t* la = a_region + (DEEP_B ? a1 : a2);
            __builtin_amdgcn_sched_barrier(0);
            kstep(0, ca, cb, 1, LA, LB, s1, s2, lb, la, nothing);  // k-step 0
            kstep(1, ca, cb, 2, LB, LC, s1, s2, lb, la, nothing);  // k-step 1
            if constexpr (CARRY)
                kstep(0, ca, cb, 3, LC, LC, s1, s2, lb, la, [&] { s3 = src(kt + 3); });  // k-step 2
            else
                kstep(0, ca, cb, 3, LC, LC, s1, s2, lb, la, nothing);
            // early(kt+1) was issued before late(kt+2) in this period and late(kt+1) a period
            // ago: all but the PL youngest loads must have landed; this wave's
            // fragment reads of k-tile kt are in registers (lgkmcnt(0))
            __builtin_amdgcn_s_waitcnt((PL & 0xF) | ((PL >> 4) << 14));
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);
            // k-step 3: first fragments of k-tile kt+1; the early operand's slot of k-tile
            // kt is free, the head of early(kt+2) goes into it
            kstep(1, a_region + a1, b_region + b1, 0, 0, LA, s2, s2, b_region + b0, a_region + a0, nothing);
            rotate();
            if constexpr (CARRY) {
                s1 = s2;
                s2 = s3;
            }
        }
        } else {
            for (int kt = 0; kt < c_kt; ++kt) {
                const Src s1 = src(kt + 1), s2 = src(kt + 2);
                uint8_t* lb = b_region + (DEEP_B ? b2 : b1);
                uint8_t* la = a_region + (DEEP_B ? a1 : a2);
#pragma unroll
                for (int i = LA; i < LC; ++i) fetch_one(i, s1, s2, lb, la);
                __builtin_amdgcn_s_waitcnt((PL & 0xF) | ((PL >> 4) << 14));
                __builtin_amdgcn_s_barrier();
#pragma unroll
                for (int i = 0; i < LA; ++i) fetch_one(i, s2, s2, b_region + b0, a_region + a0);
                rotate();
            }
            // the next tile may have rows for this wave: its first fragments, as the last k-step would have read them
            if (n_valid) {
#pragma unroll
                for (int q = 0; q < NREAD; ++q) read_one(a_region + a0, b_region + b0, 0, 0, q);
            }
        }
        // Epilogue.  The late operand's slot that held the last k-tile (now its third) is
        // idle: every wave finished reading it before the last barrier, and the
        // next loads into it are issued only after the barrier below.
        store_tile_staged<FM, FN, WM, MODE, (FM * FN * 16 > 128)>(acc, c_row0, c_rows, c_n0, C, GU, N, wm, wn, lane,
                                              (DEEP_B ? b_region + b2 : a_region + a2) + wave * (32 * FO * 64));
        if (!n_valid) break;
        c_a = n_a; c_b0 = n_b0; c_b1 = n_b1; c_alim = n_alim; c_blim = n_blim;
        c_row0 = n_row0; c_rows = n_rows; c_n0 = n_n0;
        if (GROUPK) c_kt = n_kt;
        if (KMAJ) c_krows = n_krows;
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
    if (sample && tid == 0) {
        ticks[0] = __builtin_amdgcn_s_memtime() - tk_entry;
        ticks[1] = __builtin_amdgcn_s_memrealtime() - rt_entry;
    }
}

template <int BM, int BN, int WGM, int WGN, int MODE, bool DEEP_B = false>
void launch_persist(const void* A, const int32_t* offsets, int r_max, int E, int N, int K, const void* B0,
                    const void* B1, void* C, void* GU, hipStream_t s) {
    constexpr int OUTN = (MODE == 1 || MODE == 2) ? BN / 2 : BN;
    constexpr size_t smem = (size_t)(3 * BM + 2 * BN) * 64 * 2;
    const int ntn = (N + OUTN - 1) / OUTN;
    // many experts = many ragged tail tiles: the instantiation whose idle waves skip the multiplication
    const bool idle_skip = MODE != 3 && persist_idle_skip(E);
    // few experts: whole rounds of tiles are dealt to the XCDs round by round; many: contiguous shares (measured)
    const bool by_round = MODE == 3 || E < 16;
    auto kern = idle_skip ? (by_round ? gemm_bf16_persist_kernel<BM, BN, WGM, WGN, MODE, false, false, (MODE != 3), DEEP_B, true>
                                      : gemm_bf16_persist_kernel<BM, BN, WGM, WGN, MODE, false, false, (MODE != 3), DEEP_B, false>)
                          : (by_round ? gemm_bf16_persist_kernel<BM, BN, WGM, WGN, MODE, false, false, false, DEEP_B, true>
                                      : gemm_bf16_persist_kernel<BM, BN, WGM, WGN, MODE, false, false, false, DEEP_B, false>);
    static bool attr_set[2][2] = {{false, false}, {false, false}};
    if (!attr_set[idle_skip][by_round]) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  (int)smem);
        attr_set[idle_skip][by_round] = true;
    }
    // never more workgroups than the static bound on the tile count
    const int grid = min(persist_grid(), grid_for(r_max, E, BM, ntn));
    hipLaunchKernelGGL(kern, dim3(grid), dim3(WGM * WGN * 64), smem, s, static_cast<const bf16_t*>(A), offsets, E, N,
                       K, static_cast<const bf16_t*>(B0), static_cast<const bf16_t*>(B1), static_cast<bf16_t*>(C),
                       static_cast<bf16_t*>(GU), ntn, 0, g_persist_ticks);
}

// dw[e] = 0 for every expert without rows (the persistent weight-gradient kernel gives them no tiles)
__global__ __launch_bounds__(256) void wgrad_zero_empty_kernel(const int32_t* __restrict__ offsets, size_t per_expert,
                                                               bf16_t* __restrict__ dw) {
    const int e = blockIdx.y;
    if (offsets[e + 1] - offsets[e] > 0) return;
    u32x4* dst = reinterpret_cast<u32x4*>(dw + (size_t)e * per_expert);   // per_expert is a multiple of 8
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < per_expert / 8; i += (size_t)gridDim.x * 256)
        dst[i] = u32x4{0u, 0u, 0u, 0u};
}

template <int BM, int BN, int WGM, int WGN>
void launch_persist_groupk(const void* A, const void* B, const int32_t* offsets, int E, int M, int N, int ld,
                           void* C, hipStream_t s) {
    constexpr size_t smem = (size_t)(3 * BM + 2 * BN) * 64 * 2;
    auto kern = gemm_bf16_persist_kernel<BM, BN, WGM, WGN, 0, true>;
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  (int)smem);
        attr_set = true;
    }
    hipLaunchKernelGGL(wgrad_zero_empty_kernel, dim3(64, E), dim3(256), 0, s, offsets, (size_t)M * N,
                       static_cast<bf16_t*>(C));
    const long long tiles = (long long)E * ((M + BM - 1) / BM) * ((N + BN - 1) / BN);
    const int grid = (int)min((long long)persist_grid(), (tiles + 7) / 8 * 8);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(WGM * WGN * 64), smem, s, static_cast<const bf16_t*>(A), offsets, E, N,
                       ld, static_cast<const bf16_t*>(B), static_cast<const bf16_t*>(B), static_cast<bf16_t*>(C),
                       static_cast<bf16_t*>(nullptr), M, 0, g_persist_ticks);
}

// weight gradients straight from the row-major activations (no transposed copies): see the kernel's KMAJ form
template <int BM, int BN, int WGM, int WGN>
void launch_persist_groupk_rowmajor(const void* A, int lda, const void* B, int ldb, const int32_t* offsets, int E,
                                    int M, int N, const void* zero_row, void* C, hipStream_t s) {
    constexpr size_t smem = (size_t)(3 * BM + 2 * BN) * 64 * 2;
    auto kern = gemm_bf16_persist_kernel<BM, BN, WGM, WGN, 0, true, true>;
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  (int)smem);
        attr_set = true;
    }
    hipLaunchKernelGGL(wgrad_zero_empty_kernel, dim3(64, E), dim3(256), 0, s, offsets, (size_t)M * N,
                       static_cast<bf16_t*>(C));
    const long long tiles = (long long)E * ((M + BM - 1) / BM) * ((N + BN - 1) / BN);
    const int grid = (int)min((long long)persist_grid(), (tiles + 7) / 8 * 8);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(WGM * WGN * 64), smem, s, static_cast<const bf16_t*>(A), offsets, E, N,
                       lda, static_cast<const bf16_t*>(B), static_cast<const bf16_t*>(B), static_cast<bf16_t*>(C),
                       static_cast<bf16_t*>(const_cast<void*>(zero_row)), M, ldb, g_persist_ticks);
}

template <int BM, int BN, int WGM, int WGN, bool DEEP_B = false>
void run_persist_pair(const void* x_perm, const int32_t* offsets, int r_max, int H, int F, int E,
                      const void* w_gate, const void* w_up, const void* w_down, void* h, void* y_perm, int phase,
                      hipStream_t s) {
    if (phase & 1) launch_persist<BM, BN, WGM, WGN, 1, DEEP_B>(x_perm, offsets, r_max, E, F, H, w_gate, w_up, h, nullptr, s);
    if (phase & 2) launch_persist<BM, BN, WGM, WGN, 0, DEEP_B>(h, offsets, r_max, E, H, F, w_down, nullptr, y_perm, nullptr, s);
}

}  // namespace

void set_persist_workgroups(int n) { g_persist_workgroups = n; }
void set_persist_idle_skip(int v) { g_persist_idle_skip = v; }
void set_persist_clock_sample(unsigned long long* ticks) { g_persist_ticks = ticks; }
bool persist_idle_skip(int E) { return g_persist_idle_skip < 0 ? E >= 16 : g_persist_idle_skip != 0; }

// C [rows, N] = A [rows, K] . B[e]^T with B [E, N, K], rows grouped by expert (bf16): the
// down-projection form of the persistent kernel, for any operands of that shape
bool launch_grouped_nt(const void* A, const int32_t* offsets, int r_max, int E, int N, int K, const void* B,
                       void* C, hipStream_t s) {
    if (K < 128 || K % 64 || N % 8) return false;
    launch_persist<256, 256, 2, 4, 0, true>(A, offsets, r_max, E, N, K, B, nullptr, C, nullptr, s);
    return true;
}

// dw [E, M, N] = per expert a_t[:, seg_e] . b_t[:, seg_e]^T (see WgradSched); M, N multiples of 8, ld of 64
void launch_persist_wgrad(const void* a_t, const void* b_t, const int32_t* offsets, int E, int M, int N, int ld,
                          void* dw, hipStream_t s) {
    launch_persist_groupk<256, 256, 2, 4>(a_t, b_t, offsets, E, M, N, ld, dw, s);
}

// dw [E, M, N] = per expert A[rows_e, 0:M]^T . B[rows_e, 0:N], A [rows, lda] and B [rows, ldb] row-major; M, N
// multiples of 8 and lda, ldb multiples of 8; zero_row: 512 bytes of zeros
void launch_persist_wgrad_rowmajor(const void* a, int lda, const void* b, int ldb, const int32_t* offsets, int E,
                                   int M, int N, const void* zero_row, void* dw, hipStream_t s) {
    launch_persist_groupk_rowmajor<256, 256, 2, 4>(a, lda, b, ldb, offsets, E, M, N, zero_row, dw, s);
}

// dg | du [rows, 2N] from dh = A . B[e]^T (never stored) and the saved pre-activations gu [rows, 2N]
bool launch_grouped_nt_swiglu_bwd(const void* A, const int32_t* offsets, int r_max, int E, int N, int K,
                                  const void* B, const void* gu, void* dgdu, hipStream_t s) {
    if (K < 128 || K % 64 || N % 8) return false;
    launch_persist<256, 256, 2, 4, 3, true>(A, offsets, r_max, E, N, K, B, nullptr, dgdu, const_cast<void*>(gu), s);
    return true;
}

// h = silu(x W_gate^T) * (x W_up^T) as in the forward, and the two pre-activations to gu [rows, 2F]
bool launch_gate_up_saving(const void* x_perm, const int32_t* offsets, int r_max, int H, int F, int E,
                           const void* w_gate, const void* w_up, void* h, void* gu, hipStream_t s) {
    if (H < 128 || H % 64 || F % 8) return false;
    launch_persist<256, 256, 2, 4, 2, true>(x_perm, offsets, r_max, E, F, H, w_gate, w_up, h, gu, s);
    return true;
}

bool launch_persist_ffn(const void* x_perm, const int32_t* offsets, int r_max, int H, int F, int E,
                        const void* w_gate, const void* w_up, const void* w_down, void* h, void* y_perm,
                        int variant, int phase, hipStream_t s) {
    if (H < 128 || F < 128) return false;  // the k stream needs at least two k-tiles per output tile
    switch (variant) {
        case 40: run_persist_pair<256, 256, 2, 2>(x_perm, offsets, r_max, H, F, E, w_gate, w_up, w_down, h, y_perm, phase, s); return true;
        case 41: run_persist_pair<256, 256, 2, 4>(x_perm, offsets, r_max, H, F, E, w_gate, w_up, w_down, h, y_perm, phase, s); return true;
        case 42: run_persist_pair<256, 256, 2, 2, true>(x_perm, offsets, r_max, H, F, E, w_gate, w_up, w_down, h, y_perm, phase, s); return true;
        case 43: run_persist_pair<256, 256, 2, 4, true>(x_perm, offsets, r_max, H, F, E, w_gate, w_up, w_down, h, y_perm, phase, s); return true;
        default: return false;
    }
}

}  // namespace moe
