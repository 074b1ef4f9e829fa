// a3. Grouped SwiGLU expert FFN (Section 3.1.2 "Expert Computation"; f_e of
// Eq. 1): for every expert e, over its contiguous rows,
//     h = silu(X_e W_gate,e^T) * (X_e W_up,e^T),   Y_e = h W_down,e^T.
//
// Both products are "NT" GEMMs (activations [rows, K] and weights [N, K] are
// both contiguous along the contraction index), which is exactly the operand
// order the gfx950 bf16 MFMA wants: each lane feeds 8 consecutive-K values.
//
// This file holds the dispatch and the plain kernel for fp32 layers and odd
// shapes.  The MFMA kernels live in gemm_persist.hip (default: one persistent
// workgroup per compute unit walking a device-side tile list) and
// gemm_pipe3.hip (one workgroup per tile; taken when the contraction is too
// shallow for the persistent kernel's k stream).  For the first GEMM a weight
// tile holds 128 gate rows and the 128 matching up rows and every wave owns the
// same feature range of both, so silu(g)*u happens in registers and only h is
// written.
//
// Ragged scheduling: the per-expert row offsets live in device memory; the
// kernels derive the real tile list from them, no host round trip.
#include "gemm_tile.h"

namespace moe {

namespace {

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

template <typename TIn, bool SWIGLU>
void launch_simple_gemm(const void* A, const int32_t* offsets, int r_max, int E, int N, int K,
                        const void* B0, const void* B1, void* C, hipStream_t s) {
    const int ntn = (N + 63) / 64;
    const int grid = grid_for(r_max, E, 64, ntn);
    hipLaunchKernelGGL((gemm_simple_kernel<TIn, SWIGLU>), dim3(grid), dim3(256), 0, s,
                       static_cast<const TIn*>(A), offsets, E, N, K, static_cast<const TIn*>(B0),
                       static_cast<const TIn*>(B1), static_cast<TIn*>(C), ntn);
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
        // tuned default (measured on MI355X at the benchmark shapes): the persistent 8-wave kernel with three LDS
        // stages for the weight tile; layers too shallow for its k stream fall back to the
        // one-workgroup-per-tile kernels (8 waves gate/up, 4 waves down)
        if (launch_persist_ffn(x_perm, offsets, r_max, H, F, E, w_gate, w_up, w_down, h, y_perm, 43, phase, s))
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
    return false;   // unknown variant
}

}  // namespace moe
