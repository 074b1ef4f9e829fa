// Helpers of the expert FFN's backward (Section 3.3: the backward workflow
// mirrors the forward; f_e of Eq. 1 by the chain rule).  The grouped GEMM
// kernels of this library multiply operands that are both contiguous along the
// contraction index ("NT").  The backward needs the other layouts, so operands
// are re-laid once and the same GEMM engine is reused:
//
//   transpose_batched_kernel   weights [B, R, C] -> [B, C, ld] (at a column
//                              offset, so W_gate^T and W_up^T can sit side by
//                              side for the input-gradient GEMM)
//   ragged_transpose_kernel    activations [rows, C] -> [C, Rp]: the rows of
//                              expert e become columns poff_e .. poff_e + n_e,
//                              every expert's segment padded with zeros to a
//                              multiple of 64 (at least 128) columns, so the
//                              weight-gradient GEMMs contract over whole k-tiles
//   swiglu_backward_kernel     (dh, g, u) -> dg | du side by side
//
// All bf16, 64 x 64 tiles through LDS for the transposes.
#include "common.h"

namespace moe {

namespace {

constexpr int TT = 64;  // transpose tile

// Load a TT x TT tile of 16-bit elements (rows r0.., cols c0..) into LDS, rows
// beyond `rows` / cols beyond `cols` as zero.  256 threads: 8 lanes x 16 bytes
// per row, 32 rows per pass.
__device__ __forceinline__ void load_tile(const uint16_t* __restrict__ src, size_t ld, int r0, int c0, int rows,
                                          int cols, uint16_t (*tile)[TT + 2]) {
    const int tid = threadIdx.x;
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        const int r = p * 32 + tid / 8, c = (tid % 8) * 8;
        u32x4 v = u32x4{0u, 0u, 0u, 0u};
        if (r0 + r < rows && c0 + c < cols)   // cols is a multiple of 8
            v = *reinterpret_cast<const u32x4*>(src + (size_t)(r0 + r) * ld + c0 + c);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            tile[r][c + 2 * j] = (uint16_t)(v[j] & 0xffffu);
            tile[r][c + 2 * j + 1] = (uint16_t)(v[j] >> 16);
        }
    }
}

// Store the transpose of the tile: output row c0 + c gets 8 consecutive source
// rows per lane (16 bytes), i.e. dst[(c0 + c) * ldo + o0 + r .. + 7].
__device__ __forceinline__ void store_tile_t(uint16_t* __restrict__ dst, size_t ldo, int c0, int cols, size_t o0,
                                             int n_out, const uint16_t (*tile)[TT + 2]) {
    const int tid = threadIdx.x;
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        const int c = p * 32 + tid / 8, r = (tid % 8) * 8;
        if (c0 + c >= cols || r >= n_out) continue;   // n_out is a multiple of 8
        u32x4 v;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            v[j] = (uint32_t)tile[r + 2 * j][c] | ((uint32_t)tile[r + 2 * j + 1][c] << 16);
        *reinterpret_cast<u32x4*>(dst + (size_t)(c0 + c) * ldo + o0 + r) = v;
    }
}

// dst[b][c][col0 + r] = src[b][r][c];  R, C multiples of 8.
__global__ __launch_bounds__(256) void transpose_batched_kernel(const uint16_t* __restrict__ src, int R, int C,
                                                                uint16_t* __restrict__ dst, size_t ldo, int col0) {
    __shared__ uint16_t tile[TT][TT + 2];
    const int b = blockIdx.z, r0 = blockIdx.y * TT, c0 = blockIdx.x * TT;
    load_tile(src + (size_t)b * R * C, (size_t)C, r0, c0, R, C, tile);
    __syncthreads();
    const int n_out = min(TT, R - r0);
    store_tile_t(dst + (size_t)b * C * ldo, ldo, c0, C, (size_t)col0 + r0, n_out, tile);
}

// padded length of an expert's column segment in the transposed activations
__device__ __forceinline__ int padded_rows(int n) { return n <= 0 ? 0 : max(128, (n + 63) & ~63); }

// poff[e] = first column of expert e's zero-padded segment (exclusive prefix of the padded row counts), e = 0..E.
// One workgroup of 256 threads; E <= 256.
__global__ __launch_bounds__(256) void ragged_offsets_kernel(const int32_t* __restrict__ offsets, int E,
                                                             int32_t* __restrict__ poff) {
    __shared__ int scan[2][256];
    const int tid = threadIdx.x;
    const int pn = (tid < E) ? padded_rows(offsets[tid + 1] - offsets[tid]) : 0;
    scan[0][tid] = pn;
    __syncthreads();
    int cur = 0;
    for (int d = 1; d < 256; d <<= 1) {
        scan[cur ^ 1][tid] = scan[cur][tid] + ((tid >= d) ? scan[cur][tid - d] : 0);
        cur ^= 1;
        __syncthreads();
    }
    if (tid < E) poff[tid + 1] = scan[cur][tid];
    if (tid == 0) poff[0] = 0;
}

// dst[c][poff_e + (r - lo_e)] = src[r][c] for the rows r of expert e; the pad up to
// padded_rows(n_e) is zero.  One workgroup per (64-column block, 64-row block of the
// padded axis); the expert of a padded position is the one whose segment [poff_e,
// poff_e+1) holds it (segments are multiples of 64, so a block never straddles two).
__global__ __launch_bounds__(256) void ragged_transpose_kernel(const uint16_t* __restrict__ src,
                                                               const int32_t* __restrict__ offsets,
                                                               const int32_t* __restrict__ poff, int E, int C,
                                                               uint16_t* __restrict__ dst, size_t ldo) {
    __shared__ uint16_t tile[TT][TT + 2];
    __shared__ int seg[3];   // first source row of this block, valid rows from there on, found flag
    const int p0 = blockIdx.y * TT, c0 = blockIdx.x * TT;
    if (threadIdx.x == 0) seg[2] = 0;
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += 256) {
        const int lo_p = poff[e], hi_p = poff[e + 1];
        if (lo_p <= p0 && p0 < hi_p) {   // at most one expert
            const int lo = offsets[e], n = offsets[e + 1] - lo;
            seg[0] = lo + (p0 - lo_p);
            seg[1] = n - (p0 - lo_p);   // may be <= 0: a block of pure padding
            seg[2] = 1;
        }
    }
    __syncthreads();
    if (!seg[2]) return;   // past the last expert's padding: nothing to write
    const int r_first = seg[0];
    const int n_valid = max(0, min(TT, seg[1]));
    // rows r_first .. r_first + n_valid of src; the rest of the 64 positions are padding (zeros)
    load_tile(src, (size_t)C, r_first, c0, r_first + n_valid, C, tile);
    __syncthreads();
    store_tile_t(dst, ldo, c0, C, (size_t)p0, TT, tile);
}

// dg | du from dh [rows, F] and g, u (bf16, rows ld_gu elements apart; out [rows, 2F]): with s = 1/(1+e^-g),
//   du = dh * g * s,   dg = dh * u * s * (1 + g * (1 - s)).
// Only rows below *n_rows (device: the kept-row count) are processed.
__global__ __launch_bounds__(256) void swiglu_backward_kernel(const uint16_t* __restrict__ dh,
                                                              const uint16_t* __restrict__ g,
                                                              const uint16_t* __restrict__ u, size_t ld_gu,
                                                              const int32_t* __restrict__ n_rows, int F,
                                                              uint16_t* __restrict__ out) {
    const int rows = *n_rows;
    const int vpr = F / 8;  // 16-byte vectors per row
    const size_t nvec = (size_t)rows * vpr;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < nvec; i += (size_t)gridDim.x * 256) {
        const size_t r = i / vpr;
        const int c = (int)(i - r * vpr) * 8;
        const u32x4 a = *reinterpret_cast<const u32x4*>(dh + r * F + c);
        const u32x4 b = *reinterpret_cast<const u32x4*>(g + r * ld_gu + c);
        const u32x4 d = *reinterpret_cast<const u32x4*>(u + r * ld_gu + c);
        u32x4 og, ou;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float dgv[2], duv[2];
#pragma unroll
            for (int hlf = 0; hlf < 2; ++hlf) {
                const float dhv = __uint_as_float(hlf ? (a[j] & 0xffff0000u) : (a[j] << 16));
                const float gv = __uint_as_float(hlf ? (b[j] & 0xffff0000u) : (b[j] << 16));
                const float uv = __uint_as_float(hlf ? (d[j] & 0xffff0000u) : (d[j] << 16));
                const float s = __builtin_amdgcn_rcpf(1.f + __expf(-gv));
                duv[hlf] = dhv * gv * s;
                dgv[hlf] = dhv * uv * s * (1.f + gv * (1.f - s));
            }
            og[j] = pack2_bf16(dgv[0], dgv[1]);
            ou[j] = pack2_bf16(duv[0], duv[1]);
        }
        *reinterpret_cast<u32x4*>(out + r * 2 * F + c) = og;
        *reinterpret_cast<u32x4*>(out + r * 2 * F + F + c) = ou;
    }
}

}  // namespace

void launch_transpose_batched(const void* src, int B, int R, int C, void* dst, size_t ldo, int col0, hipStream_t s) {
    if (B <= 0 || R <= 0 || C <= 0) return;
    hipLaunchKernelGGL(transpose_batched_kernel, dim3((C + TT - 1) / TT, (R + TT - 1) / TT, B), dim3(256), 0, s,
                       static_cast<const uint16_t*>(src), R, C, static_cast<uint16_t*>(dst), ldo, col0);
}

void launch_ragged_offsets(const int32_t* offsets, int E, int32_t* poff, hipStream_t s) {
    hipLaunchKernelGGL(ragged_offsets_kernel, dim3(1), dim3(256), 0, s, offsets, E, poff);
}

// rp_max: the static bound on the padded axis (a multiple of 64); blocks past the real padded length exit.
// poff: the E + 1 segment starts written by launch_ragged_offsets
void launch_ragged_transpose(const void* src, const int32_t* offsets, const int32_t* poff, int E, int C, int rp_max,
                             void* dst, hipStream_t s) {
    if (rp_max <= 0 || C <= 0) return;
    hipLaunchKernelGGL(ragged_transpose_kernel, dim3((C + TT - 1) / TT, rp_max / TT), dim3(256), 0, s,
                       static_cast<const uint16_t*>(src), offsets, poff, E, C, static_cast<uint16_t*>(dst),
                       (size_t)rp_max);
}

void launch_swiglu_backward(const void* dh, const void* g, const void* u, size_t ld_gu, const int32_t* n_rows,
                            int r_max, int F, void* out, hipStream_t s) {
    if (r_max <= 0) return;
    size_t blocks = ((size_t)r_max * (F / 8) + 255) / 256;
    if (blocks > 256 * 16) blocks = 256 * 16;
    hipLaunchKernelGGL(swiglu_backward_kernel, dim3((unsigned)blocks), dim3(256), 0, s,
                       static_cast<const uint16_t*>(dh), static_cast<const uint16_t*>(g),
                       static_cast<const uint16_t*>(u), ld_gu, n_rows, F, static_cast<uint16_t*>(out));
}

}  // namespace moe
