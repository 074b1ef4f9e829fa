// Shared declarations of the HIP side of the MoE hot path (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/moe.h"

namespace moe {

typedef uint16_t bf16_t;  // raw bf16 bit pattern in memory

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr int kWave = 64;
constexpr int kMaxExperts = 256;
constexpr int kMaxTopK = 64;

__device__ __forceinline__ float bf16_to_f32(bf16_t v) {
    return __uint_as_float(static_cast<uint32_t>(v) << 16);
}

// round-to-nearest-even; gfx950 has a native conversion for it
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
    __bf16 b = static_cast<__bf16>(f);
    return __builtin_bit_cast(bf16_t, b);
}

// two roundings in one instruction (v_cvt_pk_bf16_f32): lo in bits 0..15, hi in bits 16..31
__device__ __forceinline__ uint32_t pack2_bf16(float lo, float hi) {
    typedef __attribute__((ext_vector_type(2))) float f32x2_t;
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
    const f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// XOR term of the GEMM kernels' LDS tiles.  A tile row is 128 bytes = eight 16-byte pieces; piece c of row r lives
// at piece position c ^ lds_swizzle(r).  The LDS has 64 banks of 4 bytes, so one pass over all banks covers 256
// bytes = TWO tile rows, and a 16-byte-per-lane read is served 16 lanes at a time.  A fragment read has 16
// consecutive rows ask for the same logical piece, so those must land in 16 different 16-byte slots of the 256-byte
// window: slot = 8 (r mod 2) + (c ^ swizzle(r)) needs a swizzle that takes all eight values over eight consecutive
// even (and odd) rows.  (r / 2) mod 8 does; r mod 8, the choice for a 32-bank LDS, pairs rows r and r + 8 and
// halves the read rate (measured: 128 against 205 bytes per clock and CU with four waves reading).
__host__ __device__ __forceinline__ constexpr int lds_swizzle(int row) { return (row >> 1) & 7; }

// host-side error reporting (api.hip)
moe_status_t fail(moe_status_t st, const char* fmt, ...);
moe_status_t check_launch(const char* what);

// ---- kernel launchers (one per source file); all enqueue on `s` and return ----
void launch_router(const void* x, const void* w, const float* bias, float* logits, int T, int H,
                   int E, int K, int renorm, moe_dtype_t dt, int32_t* idx, float* gate,
                   hipStream_t s);

// backward of the router: dlogits always; dx, dw, dbias where non-NULL; ws of router_backward_workspace_bytes
size_t router_backward_workspace_bytes(int T, int H, int E);
void launch_router_backward(const void* x, const void* w, const float* logits, const int32_t* idx, const float* dgate,
                            int T, int H, int E, int K, int renorm, moe_dtype_t dt, float* dlogits, void* dx,
                            float* dw, float* dbias, void* ws, hipStream_t s);

// router: 16-token blocks per workgroup (1, 2 or 4); 0 = chosen from T and E
void set_router_tile(int mb);

size_t permute_workspace_bytes(int T, int K, int E);
void set_permute_fused(int v);   // 1 (default): small index arrays take the one-launch dispatch; 0: never
void launch_permute(const void* x, const int32_t* idx, int T, int H, int E, int K, int capacity,
                    int r_max, moe_dtype_t dt, void* x_perm, int32_t* counts, int32_t* offsets,
                    int32_t* row_of_assign, int32_t* assign_of_row, void* ws, hipStream_t s);

// the library's own scratch for moe_permute_noalloc: its size, and its address on the current device
size_t permute_scratch_bytes();
int32_t* permute_scratch(hipError_t* err);

void launch_combine(const void* y_perm, const int32_t* row_of_assign, const float* gate,
                    const void* addend, int T, int H, int K, int r_max, moe_dtype_t dt, void* y,
                    hipStream_t s);

void launch_combine_backward(const void* dy, const void* y_perm, const int32_t* row_of_assign, const float* gate,
                             int T, int H, int K, int r_max, moe_dtype_t dt, void* dy_perm, float* dgate,
                             hipStream_t s);

// persistent grouped-GEMM kernels: workgroups per launch, 0 = one per compute unit
void set_persist_workgroups(int n);
void set_persist_idle_skip(int v);   // -1 auto, 0 off, 1 on
// device cells {shader-clock ticks, 100 MHz ticks} that workgroup 0 of every later persistent bf16 GEMM launch fills
void set_persist_clock_sample(unsigned long long* ticks);

// grouped NT GEMMs of the expert FFN.  phase bit 0: gate/up + SwiGLU (x_perm ->
// h); bit 1: down projection (h -> y_perm).  Returns false if unsupported.
bool launch_expert_ffn(const void* x_perm, const int32_t* offsets, int r_max, int H, int F, int E,
                       const void* w_gate, const void* w_up, const void* w_down, moe_dtype_t dt,
                       void* h, void* y_perm, int variant, int phase, hipStream_t s);

inline size_t up256(size_t v) { return (v + 255) & ~size_t(255); }

size_t permute_variant_workspace_bytes(int T, int K, int E);
void launch_permute_variant(const void* x, const int32_t* idx, const float* scores, int T, int H, int E, int K,
                            int capacity, int by_score, int pad, int r_max, moe_dtype_t dt, void* x_perm,
                            int32_t* counts, int32_t* offsets, int32_t* row_of_assign, int32_t* assign_of_row,
                            void* ws, hipStream_t s);

// zero the rows r < rows of x_perm with assign_of_row[r] < 0
void launch_permute_zero_rows(const int32_t* assign_of_row, void* x_perm, int rows, int row_bytes, hipStream_t s);

void launch_fill_i32(int32_t* p, int n, int32_t v0, int32_t step, hipStream_t s);

// gather of ragged row chunks (expert-parallel share of one GPU): dst = src chunks order[0], order[1], ...
int sort_chunks_max_chunks();
size_t sort_chunks_workspace_bytes(int n_dst);
void launch_sort_chunks(const void* src, int r_src, const int32_t* chunk_rows, int n_src, const int32_t* order,
                        int n_dst, int group, int row_bytes, void* dst, int r_dst, int32_t* chunk_rows_out,
                        int32_t* group_offsets, void* ws, hipStream_t s);

// ---- pieces of the expert FFN's backward (bf16) ----
// C [rows, N] = A [rows, K] . B[e]^T, B [E, N, K], rows grouped by expert; false if the shape is not covered
bool launch_grouped_nt(const void* A, const int32_t* offsets, int r_max, int E, int N, int K, const void* B,
                       void* C, hipStream_t s);
// dst[b][c][col0 + r] = src[b][r][c], dst rows ld_out elements long
void launch_transpose_batched(const void* src, int B, int R, int C, void* dst, size_t ld_out, int col0, hipStream_t s);
// dst [C, rp_max]: rows of expert e of src [rows, C] become the columns of its zero-padded segment
void launch_ragged_offsets(const int32_t* offsets, int E, int32_t* poff, hipStream_t s);   // poff [E + 1]
void launch_ragged_transpose(const void* src, const int32_t* offsets, const int32_t* poff, int E, int C, int rp_max,
                             void* dst, hipStream_t s);
// out [rows, 2F] = dg | du from dh [rows, F] and g, u (rows ld_gu elements apart); rows = *n_rows (device)
void launch_swiglu_backward(const void* dh, const void* g, const void* u, size_t ld_gu, const int32_t* n_rows,
                            int r_max, int F, void* out, hipStream_t s);
// dh = A . B[e]^T fused with the SwiGLU derivative: writes dg | du [rows, 2N] from the saved gu [rows, 2N]
bool launch_grouped_nt_swiglu_bwd(const void* A, const int32_t* offsets, int r_max, int E, int N, int K,
                                  const void* B, const void* gu, void* dgdu, hipStream_t s);
// the forward's gate/up GEMM that also stores the pre-activations g | u to gu [rows, 2F]; false if not covered
bool launch_gate_up_saving(const void* x_perm, const int32_t* offsets, int r_max, int H, int F, int E,
                           const void* w_gate, const void* w_up, void* h, void* gu, hipStream_t s);
// dw [E, M, N] = per expert a_t[:, seg_e] . b_t[:, seg_e]^T over the expert's padded column segment
// persistent: one workgroup per compute unit; pipe3: one workgroup per output tile
void launch_persist_wgrad(const void* a_t, const void* b_t, const int32_t* offsets, int E, int M, int N, int ld,
                          void* dw, hipStream_t s);
// the same product straight from the row-major activations a [rows, lda], b [rows, ldb] (no transposed copies)
void launch_persist_wgrad_rowmajor(const void* a, int lda, const void* b, int ldb, const int32_t* offsets, int E,
                                   int M, int N, const void* zero_row, void* dw, hipStream_t s);
void launch_pipe3_wgrad(const void* a_t, const void* b_t, const int32_t* offsets, int E, int M, int N, int ld,
                        void* dw, hipStream_t s);

// measurement probe: the bare bf16 MFMA + LDS-fragment loop over a 64 KiB operand image
void launch_probe_mfma_bf16(const void* image, int iters, int workgroups, float* sink, unsigned long long* ticks,
                            hipStream_t s);
void launch_probe_mfma_fp8(const void* image, int iters, int workgroups, float* sink, unsigned long long* ticks,
                           hipStream_t s);

// FP8 (E4M3) path of the expert FFN: per-tensor quantisation with amax, and the
// two grouped GEMMs on quantised operands (phase bits as above)
void launch_fp8_quantize(const void* src, moe_dtype_t dt, size_t n, float scale, void* dst, float* amax,
                         hipStream_t s);
bool fp8_ffn_supported(int H, int F);
void set_fp8_deep_b(int v);   // FP8 grouped GEMM: 1 (default) three LDS stages for the weight tile, 0 for the activation tile
void launch_permute_fp8(const void* x, const int32_t* idx, int T, int H, int E, int K, int capacity, int r_max,
                        float scale, void* x_perm_fp8, int32_t* counts, int32_t* offsets, int32_t* row_of_assign,
                        int32_t* assign_of_row, float* amax, void* ws, hipStream_t s);
void launch_expert_ffn_fp8(const void* x_perm, const int32_t* offsets, int r_max, int H, int F, int E,
                           const void* w_gate, const void* w_up, const void* w_down, float dq_gate, float dq_up,
                           float scale_h, float dq_down, void* h, float* amax_h, void* y_perm, int phase,
                           hipStream_t s);

}  // namespace moe
