/*
 * moe.h -- C ABI of the MI355X (gfx950) MoE-layer hot path: the forward of the
 * layer's four stages, their backward, the FP8 expert FFN and one GPU's step of
 * expert-parallel dispatch.
 *
 * The library computes, on one GPU with all experts local, the
 * Mixture-of-Experts layer of arXiv 2504.14960:
 *
 *     y = sum_e g_e(x) * f_e(x)                       (Eq. 1, Section 3.1.1)
 *
 * through the data path of the paper's token dispatcher (Section 3.3, forward
 * workflow, with EP = ETP = 1 so that every collective drops out):
 *
 *     router -> permute -> experts -> un-permute
 *
 * Notation: T tokens, H hidden size, E experts, K experts per token, F expert
 * FFN size, C capacity (rows per expert, 0 = dropless), R kept rows.
 *
 * Conventions common to every entry point
 *   - Every tensor pointer is DEVICE memory owned by the caller, row-major,
 *     innermost dimension contiguous, 16-byte aligned.  The library never
 *     allocates, frees or retains device memory; scratch comes in as
 *     `workspace`.  `moe_last_error` is the only pointer it hands out.
 *   - `stream` is a hipStream_t owned by the caller (NULL = the default
 *     stream).  All work is enqueued on it; nothing synchronises; outputs are
 *     valid in stream order.  No host<->device copies happen: per-expert row
 *     counts stay on the device.
 *   - Weights are [out_features, in_features] (the contraction index is the
 *     contiguous one for both operands).
 *   - dt is the storage type of x, the weights, x_perm, h, y_perm and y.
 *     Logits, gates and all accumulation are fp32 for both types.
 *   - Argument errors are detected on the host before anything is enqueued and
 *     returned as a status; `moe_last_error()` then holds a message.  Device
 *     data is never validated on the host: an expert index outside [0, E) is
 *     treated as a dropped assignment, never as an address.
 *   - T == 0 is legal (MOE_OK, nothing launched).  Experts with no rows are
 *     legal everywhere.
 *   - Same inputs give bit-identical outputs on every call (no floating-point
 *     atomics, no slot-claiming atomics).
 *   - Limits: 1 <= K <= min(E, 64), E <= 256, T*K < 2^31, H % 8 == 0 and
 *     F % 8 == 0 for MOE_BF16 (H % 4, F % 4 for MOE_F32).
 */
#ifndef MOE_H_
#define MOE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MOE_OK = 0,
    MOE_ERR_INVALID_ARG = 1, /* NULL where not allowed, bad size, misalignment */
    MOE_ERR_UNSUPPORTED = 2, /* a legal request outside the limits above */
    MOE_ERR_WORKSPACE = 3,   /* workspace NULL or too small */
    MOE_ERR_LAUNCH = 4       /* the HIP runtime refused a launch */
} moe_status_t;

typedef enum { MOE_F32 = 0, MOE_BF16 = 1 } moe_dtype_t;

typedef void* moe_stream_t;

/* Message of the last failed call on this host thread ("" if none).  Static
 * thread-local storage; never free it. */
const char* moe_last_error(void);

/* Library version string (static storage). */
const char* moe_version(void);

/* Eq. 4 (Section 3.1.1): capacity per expert = CF * L / E, with L = T*K
 * token-expert assignments, rounded up.  Host only, pure.  Returns 0 when
 * capacity_factor <= 0 (dropless). */
int moe_capacity_from_factor(double capacity_factor, int T, int K, int E);

/* Rows x_perm / y_perm / h / assign_of_row must have room for:
 * T*K when dropless (capacity <= 0), else min(T*K, E*capacity).  Host only. */
int moe_max_rows(int T, int K, int E, int capacity);

/* Bytes of scratch moe_permute needs.  Host only. */
size_t moe_permute_workspace_bytes(int T, int K, int E);

/*
 * a1. Router: Eq. 3 (s = softmax(W_g x)) and Eq. 2 (Top-K gating), Section
 * 3.1.1; "selecting the top-k ... based on their softmax probabilities",
 * Section 3.3.
 *
 *   logits[t,e] = sum_h x[t,h] * w_router[e,h] (+ logit_bias[e])     fp32
 *   the K experts with the largest logits are selected, slot order = logit
 *   descending, equal logits -> lower expert index first (-0 == +0, NaN ranks
 *   last); topk_gate[t,k] = softmax(logits[t,:])[topk_idx[t,k]], divided by
 *   the sum of the K selected gates when renormalize != 0.
 *
 * x [T,H] (dt), w_router [E,H] (dt), logit_bias [E] fp32 or NULL.
 * logits [T,E] fp32: OUTPUT when x != NULL.  When x == NULL the product is
 * skipped and `logits` is the INPUT the selection runs on (w_router,
 * logit_bias, H are then ignored).
 * topk_idx [T,K] int32, topk_gate [T,K] fp32: outputs.
 */
moe_status_t moe_router_topk(const void* x, const void* w_router, const float* logit_bias,
                             float* logits, int T, int H, int E, int K, int renormalize,
                             moe_dtype_t dt, int32_t* topk_idx, float* topk_gate,
                             moe_stream_t stream);

/*
 * a2. Permute: Section 3.1.2 "Token Dispatching" (tokens of one expert stored
 * contiguously) with the capacity rule of Eq. 4 / Section 3.3 (sub-sequence
 * dropping: only this call's tokens decide).
 *
 * Assignments a = t*K + k are ranked inside their expert in ascending a; an
 * assignment is kept iff capacity <= 0 or its rank < capacity.  Kept rows of
 * expert e occupy rows [expert_offsets[e], expert_offsets[e+1]) of x_perm in
 * rank order; x_perm[row,:] is a byte copy of x[t,:].
 *
 * x [T,H] (dt), topk_idx [T,K] int32 -> x_perm [R_max,H] (dt; rows >= R are
 * left untouched), expert_counts [E], expert_offsets [E+1], row_of_assign
 * [T*K] (-1 = dropped), assign_of_row [R_max] (-1 = unused), all int32, with
 * R_max = moe_max_rows(T,K,E,capacity).  workspace: at least
 * moe_permute_workspace_bytes(T,K,E) bytes, contents irrelevant on entry.
 * x and x_perm may both be NULL to compute the maps only.
 */
moe_status_t moe_permute(const void* x, const int32_t* topk_idx, int T, int H, int E, int K,
                         int capacity, moe_dtype_t dt, void* x_perm, int32_t* expert_counts,
                         int32_t* expert_offsets, int32_t* row_of_assign,
                         int32_t* assign_of_row, void* workspace, size_t workspace_bytes,
                         moe_stream_t stream);

/*
 * moe_permute for callers that cannot hand over (or allocate) a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid device
 * allocation.  Same arguments, outputs, limits and errors as moe_permute, minus
 * the workspace: the chunk histograms live in a 1 MiB array inside the library's
 * device image (one copy per GPU, held until the process ends).  Nothing is
 * allocated or freed, here or in anything this calls.  The call is refused with
 * MOE_ERR_UNSUPPORTED when moe_permute_workspace_bytes(T, K, E) exceeds 1 MiB
 * (ceil(T*K/1024) * E > 262144; every benchmark shape is far below).  The array
 * keeps the previous call's contents; nothing in it has to start at zero (every
 * cell that is read was written earlier in the same call).  All calls on one GPU
 * share the array: calls that overlap in time on one GPU (different streams)
 * race; calls on one stream, or ordered by events, are fine.  The first call on
 * a device looks the array's address up (not to be captured into a graph: make
 * one plain call first).
 */
moe_status_t moe_permute_noalloc(const void* x, const int32_t* topk_idx, int T, int H, int E, int K,
                                 int capacity, moe_dtype_t dt, void* x_perm, int32_t* expert_counts,
                                 int32_t* expert_offsets, int32_t* row_of_assign,
                                 int32_t* assign_of_row, moe_stream_t stream);

/*
 * Two variants of a2 that capacity-based MoE training uses next to the paper's
 * default (Eq. 4 fixes the capacity; Section 3.3 drops by position):
 *
 *   drop_by_score != 0: an expert with more than `capacity` assignments keeps
 *     those with the largest scores[t,k] (fp32, finite; compared as floats, -0 =
 *     +0; equal scores: the lower assignment index wins) instead of the first
 *     `capacity` in token order.  Typically scores = topk_gate.  Ignored when
 *     capacity <= 0.
 *   pad_to_capacity != 0: expert e owns rows [e*capacity, (e+1)*capacity):
 *     expert_offsets[e] = e*capacity (so the grouped GEMM sees equal groups),
 *     expert_counts[e] = rows really kept, the rest of each block is zero rows
 *     with assign_of_row = -1 (zero rows give zero FFN outputs and no assignment
 *     points at them).  Needs capacity > 0.
 *
 * In either variant the kept rows of an expert are in ascending assignment
 * index.  With both flags 0 the result is moe_permute's.  R_max = rows x_perm and
 * assign_of_row have room for: at least E*capacity (padded) or
 * moe_max_rows(T, K, E, capacity) (packed); rows not owned get assign_of_row = -1
 * and, in the packed layout, are left untouched in x_perm.  scores may be NULL
 * unless drop_by_score.  workspace: moe_permute_variant_workspace_bytes.
 */
size_t moe_permute_variant_workspace_bytes(int T, int K, int E);
moe_status_t moe_permute_variant(const void* x, const int32_t* topk_idx, const float* scores, int T,
                                 int H, int E, int K, int capacity, int drop_by_score,
                                 int pad_to_capacity, moe_dtype_t dt, void* x_perm,
                                 int32_t* expert_counts, int32_t* expert_offsets,
                                 int32_t* row_of_assign, int32_t* assign_of_row, int R_max,
                                 void* workspace, size_t workspace_bytes, moe_stream_t stream);

/*
 * One GPU's step of expert-parallel dispatch (Section 3.3, forward workflow:
 * permute, All-to-All-V over the EP group, expert computation, All-to-All-V
 * back, un-permute).  After the first All-to-All-V a GPU that owns several
 * experts holds, source rank by source rank, each source's rows for its local
 * experts in turn; the grouped GEMM needs all rows of an expert together, and
 * the second All-to-All-V needs the source order again.  Both are this gather
 * of row chunks (the paper does not name the operation; the collective itself
 * is not part of this library):
 *
 *   src [R_src,H] (dt) is a sequence of n_src chunks, chunk c having
 *   chunk_rows[c] rows (int32 [n_src], DEVICE memory; negative counts as 0).
 *   dst [R_dst,H] receives the chunks order[0], order[1], ..., order[n_dst-1]
 *   (int32 [n_dst], DEVICE memory) one after the other.  A chunk named twice is
 *   copied twice; an index outside [0, n_src) stands for an empty chunk.  A row
 *   is copied when it lies below R_src in src and below R_dst in dst; all other
 *   rows of dst are left untouched.  src and dst must not overlap; either may
 *   be NULL (then only the outputs below are written).
 *
 *   chunk_rows_out [n_dst] (optional): rows of every destination chunk, i.e. the
 *   chunk_rows of the way back.  group_offsets [ceil(n_dst/group) + 1]
 *   (optional, needs group > 0): first dst row of chunk g*group, and the total
 *   as last entry -- with the received chunks listed expert-major and group =
 *   number of source ranks this is the expert_offsets array of a3.
 *
 * For S source ranks and L local experts the received chunk (s, e) is chunk
 * s*L + e of src; order[e*S + s] = s*L + e gathers by expert, and on the way
 * back order[s*L + e] = e*S + s with chunk_rows = the first call's
 * chunk_rows_out.  n_src, n_dst <= 4096.  Rows are opaque: any payload with
 * H * sizeof(dt) bytes per row, a multiple of 16.  workspace:
 * moe_sort_chunks_workspace_bytes(n_dst) bytes of device memory.
 */
size_t moe_sort_chunks_workspace_bytes(int n_dst);
moe_status_t moe_sort_chunks(const void* src, int R_src, const int32_t* chunk_rows, int n_src,
                             const int32_t* order, int n_dst, int group, int H, moe_dtype_t dt,
                             void* dst, int R_dst, int32_t* chunk_rows_out, int32_t* group_offsets,
                             void* workspace, size_t workspace_bytes, moe_stream_t stream);

/*
 * a3. Experts: Section 3.1.2 "Expert Computation"; f_e of Eq. 1 as a bias-free
 * SwiGLU FFN (the paper leaves f_e open):
 *
 *   h[r,:]      = silu(x_perm[r,:] W_gate,e^T) * (x_perm[r,:] W_up,e^T)
 *   y_perm[r,:] = h[r,:] W_down,e^T          for r in expert e's row range
 *
 * x_perm [R_max,H] (dt); expert_offsets [E+1] int32 in DEVICE memory (rows of
 * expert e = [offsets[e], offsets[e+1]), offsets[E] <= R_max, non-decreasing);
 * w_gate, w_up [E,F,H]; w_down [E,H,F]; h_workspace [R_max,F] (dt, scratch and
 * output: h is rounded to dt once); y_perm [R_max,H] (dt).  Rows >= offsets[E]
 * of h and y_perm are left untouched.  Accumulation is fp32; silu(z) =
 * z / (1 + exp(-z)) in fp32.
 */
moe_status_t moe_grouped_gemm_swiglu(const void* x_perm, const int32_t* expert_offsets, int R_max,
                                     int H, int F, int E, const void* w_gate, const void* w_up,
                                     const void* w_down, moe_dtype_t dt, void* h_workspace,
                                     void* y_perm, moe_stream_t stream);

/* The two halves of a3 as separate calls (same kernels, same arguments), so
 * that a caller can time or overlap them:
 *   moe_expert_gate_up:  h = silu(x_perm W_gate^T) * (x_perm W_up^T)
 *   moe_expert_down:     y_perm = h W_down^T
 * moe_grouped_gemm_swiglu is exactly gate_up followed by down. */
moe_status_t moe_expert_gate_up(const void* x_perm, const int32_t* expert_offsets, int R_max, int H,
                                int F, int E, const void* w_gate, const void* w_up, moe_dtype_t dt,
                                void* h, moe_stream_t stream);
moe_status_t moe_expert_down(const void* h, const int32_t* expert_offsets, int R_max, int H, int F,
                             int E, const void* w_down, moe_dtype_t dt, void* y_perm,
                             moe_stream_t stream);

/*
 * a4. Un-permute + combine: Section 3.1.2 "Token Restore" and the weighted sum
 * of Eq. 1:
 *
 *   y[t,:] = sum_{k ascending, row_of_assign[t*K+k] >= 0}
 *                topk_gate[t,k] * y_perm[row_of_assign[t*K+k],:]  (+ addend[t,:])
 *
 * accumulated in fp32 and rounded to dt once.  A token whose assignments were
 * all dropped gets exactly 0 (+ addend).  y_perm [R_max,H] (dt), row_of_assign
 * [T*K] int32 (each entry < R_max or negative), topk_gate [T,K] fp32, addend
 * [T,H] (dt) or NULL, y [T,H] (dt).
 */
moe_status_t moe_unpermute_combine(const void* y_perm, const int32_t* row_of_assign,
                                   const float* topk_gate, const void* addend, int T, int H,
                                   int K, int R_max, moe_dtype_t dt, void* y, moe_stream_t stream);

/*
 * Backward of the dispatcher's two data movements (Section 3.3: the backward
 * workflow mirrors the forward one).
 *
 * moe_unpermute_combine_backward, for y = moe_unpermute_combine(y_perm, ...):
 *   dy_perm[row_of_assign[t*K+k],:] = topk_gate[t,k] * dy[t,:]      (rounded to dt once)
 *   dgate[t,k] = sum_n dy[t,n] * y_perm[row_of_assign[t*K+k],n]     (fp32; 0 if dropped)
 * dy [T,H], y_perm [R_max,H] (the forward's), dy_perm [R_max,H] (dt; only rows
 * some kept assignment points at are written), dgate [T,K] fp32.
 *
 * moe_permute_backward, for x_perm = moe_permute(x, ...):
 *   dx[t,:] = sum over kept k of dx_perm[row_of_assign[t*K+k],:]  (+ addend[t,:])
 * accumulated in fp32 and rounded to dt once; addend [T,H] (dt) or NULL carries
 * the gradient that reaches x along other paths (router, residual).
 *
 * Limits and errors as moe_unpermute_combine.
 */
moe_status_t moe_unpermute_combine_backward(const void* dy, const void* y_perm,
                                            const int32_t* row_of_assign, const float* topk_gate,
                                            int T, int H, int K, int R_max, moe_dtype_t dt,
                                            void* dy_perm, float* dgate, moe_stream_t stream);
moe_status_t moe_permute_backward(const void* dx_perm, const int32_t* row_of_assign,
                                  const void* addend, int T, int H, int K, int R_max,
                                  moe_dtype_t dt, void* dx, moe_stream_t stream);

/*
 * Backward of a1, the router (Eq. 2 + Eq. 3 by the chain rule).  The selection
 * is piecewise constant and has no gradient.  With p = softmax(logits[t,:]) and
 * S = sum_k p[idx_k]:
 *
 *   q_k = dgate[t,k]                                  (renormalize == 0)
 *   q_k = (dgate[t,k] - sum_j dgate[t,j] gate[t,j]) / S   (renormalize != 0)
 *   dlogits[t,e] = [e == idx_k] q_k p_e - p_e sum_k q_k p[idx_k]
 *   dx[t,:] = sum_e dlogits[t,e] w_router[e,:]         (dt; NULL to skip)
 *   dw_router[e,:] = sum_t dlogits[t,e] x[t,:]          (fp32 [E,H]; NULL to skip)
 *   dbias[e] = sum_t dlogits[t,e]                       (fp32 [E]; NULL to skip)
 *
 * logits [T,E] are the fp32 logits moe_router_topk wrote (bias included),
 * topk_idx [T,K] its selection (entries outside [0,E) get no gradient), dgate
 * [T,K] fp32.  dlogits [T,E] fp32 is always written.  Sums over tokens are taken
 * in a fixed order.  H a multiple of 8.  workspace: moe_router_backward_workspace_bytes
 * (needed only if dw_router is given).
 */
size_t moe_router_backward_workspace_bytes(int T, int H, int E);
moe_status_t moe_router_backward(const void* x, const void* w_router, const float* logits,
                                 const int32_t* topk_idx, const float* dgate, int T, int H, int E,
                                 int K, int renormalize, moe_dtype_t dt, float* dlogits, void* dx,
                                 float* dw_router, float* dbias, void* workspace,
                                 size_t workspace_bytes, moe_stream_t stream);

/*
 * Backward of a3, the grouped SwiGLU expert FFN (bf16 only; Section 3.3: the
 * backward workflow mirrors the forward; f_e of Eq. 1 by the chain rule).  With
 * g = x_perm W_gate^T, u = x_perm W_up^T, s = 1/(1+e^-g), h = g s u, for every
 * expert over its rows and dy_perm given:
 *
 *   dw_down[e] = dy_perm^T h               dh = dy_perm W_down[e]
 *   du = dh g s      dg = dh u s (1 + g (1 - s))
 *   dw_gate[e] = dg^T x_perm    dw_up[e] = du^T x_perm
 *   dx_perm = dg W_gate[e] + du W_up[e]
 *
 * Every intermediate (g, u, dh, dg, du) is bf16, rounded once; accumulation is
 * fp32; h is the forward's.  gu [R_max,2F] = (g | u) as written by
 * moe_expert_gate_up_saving, the forward's first GEMM with the two
 * pre-activations kept; gu == NULL makes the backward recompute g and u from
 * x_perm, w_gate and w_up (two more GEMMs, no saved tensor; w_gate and w_up are
 * read only then).  The GEMM kernels multiply operands that are contiguous along the
 * contraction index, so the weights are needed transposed:
 * moe_expert_weights_transpose writes wgu_t [E,H,2F] = (W_gate[e]^T | W_up[e]^T)
 * and wd_t [E,F,H] = W_down[e]^T; they stay valid until the weights change (all
 * micro-batches of a step).  Activations are re-laid inside the workspace.
 *
 * x_perm, dy_perm, dx_perm [R_max,H]; h [R_max,F]; dw_gate, dw_up [E,F,H],
 * dw_down [E,H,F] (bf16; experts without rows get zeros); rows in [R, R_max) of
 * dx_perm are not touched.  H and F multiples of 128, E <= 256; otherwise
 * MOE_ERR_UNSUPPORTED.  workspace: moe_expert_backward_workspace_bytes.
 */
size_t moe_expert_backward_workspace_bytes(int R_max, int H, int F, int E);
moe_status_t moe_expert_weights_transpose(const void* w_gate, const void* w_up, const void* w_down,
                                          int H, int F, int E, void* wgu_t, void* wd_t,
                                          moe_stream_t stream);
moe_status_t moe_expert_gate_up_saving(const void* x_perm, const int32_t* expert_offsets, int R_max,
                                       int H, int F, int E, const void* w_gate, const void* w_up,
                                       void* h, void* gu, moe_stream_t stream);
moe_status_t moe_grouped_gemm_swiglu_backward(const void* x_perm, const void* h, const void* gu,
                                              const void* dy_perm,
                                              const int32_t* expert_offsets, int R_max, int H, int F,
                                              int E, const void* w_gate, const void* w_up,
                                              const void* wgu_t, const void* wd_t, void* dx_perm,
                                              void* dw_gate, void* dw_up, void* dw_down,
                                              void* workspace, size_t workspace_bytes,
                                              moe_stream_t stream);

/* Bytes of workspace moe_layer_forward needs.  Fs = FFN size of the shared
 * expert (0 = none).  Host only. */
size_t moe_layer_workspace_bytes(int T, int H, int E, int K, int F, int Fs, int capacity,
                                 moe_dtype_t dt);
/* The same for a layer without a shared expert (Fs = 0): the forward workflow of
 * Section 3.3 as the paper states it. */
size_t moe_workspace_bytes(int T, int H, int E, int K, int F, int capacity, moe_dtype_t dt);

/*
 * The training step of the layer in two calls (bf16, no shared expert; Section
 * 3.3: the backward workflow mirrors the forward one).
 *
 * moe_layer_forward_train is moe_layer_forward with the first expert GEMM
 * keeping its pre-activations: gu [R_max, 2F] = (g | u) (caller-owned, R_max =
 * moe_max_rows(T, K, E, capacity)).  Same workspace size and layout as
 * moe_layer_forward with Fs = 0; the workspace must stay untouched until the
 * backward has run.
 *
 * moe_layer_backward takes dy [T,H] and that forward workspace and chains
 * moe_unpermute_combine_backward, moe_grouped_gemm_swiglu_backward,
 * moe_router_backward and moe_permute_backward (the router's input gradient
 * joins the experts' at the last step).  Outputs: dx [T,H] bf16; dw_router
 * [E,H] and dbias [E] fp32 (either may be NULL); dw_gate, dw_up [E,F,H],
 * dw_down [E,H,F] bf16.  wgu_t, wd_t: from moe_expert_weights_transpose.  gu
 * may be NULL (g and u are then recomputed).  H and F multiples of 128.
 * workspace: moe_layer_backward_workspace_bytes, separate from the forward's.
 */
moe_status_t moe_layer_forward_train(const void* x, const void* w_router, const float* logit_bias,
                                     const void* w_gate, const void* w_up, const void* w_down, int T,
                                     int H, int E, int K, int F, int renormalize, int capacity, void* y,
                                     void* gu, void* workspace, size_t workspace_bytes,
                                     moe_stream_t stream);
size_t moe_layer_backward_workspace_bytes(int T, int H, int E, int K, int F, int capacity);
moe_status_t moe_layer_backward(const void* x, const void* w_router, const void* w_gate,
                                const void* w_up, const void* wgu_t, const void* wd_t, const void* dy,
                                int T, int H, int E, int K, int F, int renormalize, int capacity,
                                const void* forward_workspace, const void* gu, void* dx,
                                float* dw_router, float* dbias, void* dw_gate, void* dw_up,
                                void* dw_down, void* workspace, size_t workspace_bytes,
                                moe_stream_t stream);

/* Where moe_layer_forward keeps its intermediates inside `workspace`, for
 * tests and profiling.  Writes 11 byte offsets into byte_offsets[0..10], in
 * this order: logits [T,E] f32, topk_idx [T,K] i32, topk_gate [T,K] f32,
 * expert_counts [E] i32, expert_offsets [E+1] i32, row_of_assign [T*K] i32,
 * assign_of_row [R_max] i32, x_perm [R_max,H] dt, h [R_max,F] dt,
 * y_perm [R_max,H] dt, shared-expert output [T,H] dt.  n = capacity of
 * byte_offsets (>= 11).  Host only. */
moe_status_t moe_layer_workspace_layout(int T, int H, int E, int K, int F, int Fs, int capacity,
                                        moe_dtype_t dt, size_t* byte_offsets, int n);

/*
 * The whole forward of Section 3.3 on one stream: a1 -> a2 -> a3 -> a4, plus an
 * optional always-on shared expert (ws_* non-NULL and Fs > 0) that is evaluated
 * on x directly and added, ungated, in a4.  The throughput metric times this
 * call.  y [T,H] (dt) is the only user-visible output; intermediates live in
 * `workspace` (layout private, see moe_layer_workspace_bytes).
 */
moe_status_t moe_layer_forward(const void* x, const void* w_router, const float* logit_bias,
                               const void* w_gate, const void* w_up, const void* w_down,
                               const void* ws_gate, const void* ws_up, const void* ws_down,
                               int T, int H, int E, int K, int F, int Fs, int renormalize,
                               int capacity, moe_dtype_t dt, void* y, void* workspace,
                               size_t workspace_bytes, moe_stream_t stream);

/*
 * FP8 variant of a3 with per-tensor delayed scaling (Section 4.5, "FP8 Training
 * Performance"; the paper names the recipe, the definitions here are this
 * library's reading of it).
 *
 * FP8 is the OCP E4M3 format (bias 7, largest finite value 448, no infinities).
 * A tensor t is held as codes q = e4m3(t * scale): round to nearest, ties to
 * even, magnitudes above 448 saturate, NaN stays NaN; the product is formed in
 * fp32.  "Delayed" scaling: the scale of a step is computed from the largest
 * |t| of EARLIER steps (moe_fp8_delayed_scale over a history of amax values the
 * caller keeps); the current step only records its own amax.
 */

/* Host only: 448 / (max(amax_history[0..len)) * 2^margin); non-finite entries
 * are ignored; 1.0 if nothing positive has been recorded yet. */
float moe_fp8_delayed_scale(const float* amax_history, int len, int margin);

/* dst[i] = e4m3(src[i] * scale) for i < n; src is dt (fp32 or bf16), dst n
 * bytes.  If amax is non-NULL, *amax (device, fp32) becomes max(*amax, max_i
 * |src[i]|): the caller zeroes it when a new step starts.  src and dst 16-byte
 * aligned. */
moe_status_t moe_fp8_quantize(const void* src, moe_dtype_t dt, size_t n, float scale, void* dst,
                              float* amax, moe_stream_t stream);

/*
 * a2 fused with the quantisation of its output: as moe_permute on a bf16 x, but
 * x_perm is written as E4M3 codes, x_perm_fp8[row,:] = e4m3(x[token,:] * scale)
 * ([R_max,H] bytes), and *amax (device, may be NULL, caller zeroes it) becomes
 * max(*amax, max |x[t,:]|) over the tokens with at least one kept assignment.
 * All other arguments, outputs, limits and errors as moe_permute; H must be a
 * multiple of 8.
 */
moe_status_t moe_permute_fp8(const void* x_bf16, const int32_t* topk_idx, int T, int H, int E, int K,
                             int capacity, float scale, void* x_perm_fp8, int32_t* expert_counts,
                             int32_t* expert_offsets, int32_t* row_of_assign, int32_t* assign_of_row,
                             float* amax, void* workspace, size_t workspace_bytes,
                             moe_stream_t stream);

/*
 * Grouped SwiGLU expert FFN on E4M3 operands.  x_perm [R_max,H], w_gate, w_up
 * [E,F,H], w_down [E,H,F] are E4M3 codes quantised with scales s_x, s_gate,
 * s_up, s_down.  For every expert over its rows:
 *
 *   g = dq_gate * (x_perm . w_gate^T)      dq_gate = 1 / (s_x * s_gate)
 *   u = dq_up   * (x_perm . w_up^T)        dq_up   = 1 / (s_x * s_up)
 *   h = silu(g) * u;  *amax_h = max(*amax_h, max |h|)   (amax_h may be NULL)
 *   h_fp8 = e4m3(h * scale_h)              [R_max,F] E4M3, workspace and output
 *   y_perm = dq_down * (h_fp8 . w_down^T)  dq_down = 1 / (scale_h * s_down), bf16
 *
 * with fp32 accumulation.  scale_h is this step's (delayed) scale of h.  H and
 * F must be multiples of 128 and at least 256, E <= 256; other shapes return
 * MOE_ERR_UNSUPPORTED.  Rows in [R, R_max) are not touched.
 */
moe_status_t moe_grouped_gemm_swiglu_fp8(const void* x_perm_fp8, const int32_t* expert_offsets,
                                         int R_max, int H, int F, int E, const void* w_gate_fp8,
                                         const void* w_up_fp8, const void* w_down_fp8, float dq_gate,
                                         float dq_up, float scale_h, float dq_down, void* h_fp8,
                                         float* amax_h, void* y_perm_bf16, moe_stream_t stream);

/* The two halves of moe_grouped_gemm_swiglu_fp8, for per-stage timing. */
moe_status_t moe_expert_gate_up_fp8(const void* x_perm_fp8, const int32_t* expert_offsets, int R_max,
                                    int H, int F, int E, const void* w_gate_fp8, const void* w_up_fp8,
                                    float dq_gate, float dq_up, float scale_h, void* h_fp8,
                                    float* amax_h, moe_stream_t stream);
moe_status_t moe_expert_down_fp8(const void* h_fp8, const int32_t* expert_offsets, int R_max, int H,
                                 int F, int E, const void* w_down_fp8, float dq_down,
                                 void* y_perm_bf16, moe_stream_t stream);

/*
 * Measurement probe (not a stage of the layer; for callers that cannot measure
 * the chip's sustained matrix rate otherwise, e.g. bench.py's roofline note).
 * Runs the bare inner loop of the bf16 grouped GEMM: `workgroups` workgroups of
 * four waves, each wave a 128 x 128 accumulator block, LDS fragment reads and
 * 32x32x16 bf16 MFMAs over a 64 KiB operand image, nothing else.  image: 65536
 * bytes, two blocks of [256 rows][64 bf16] (first operand, second operand).
 * One launch executes workgroups * iters * 8388608 FLOP.  sink: workgroups*256
 * floats (written, meaningless).  ticks (may be NULL): 2 x uint64, shader
 * clocks and 100 MHz reference clocks spent by workgroup 0 in its loop, i.e.
 * ticks[0] / ticks[1] * 100 = the shader clock in MHz under this load.
 * Enqueues one kernel; the caller times it.  1 <= iters, 1 <= workgroups <= 65536.
 */
moe_status_t moe_probe_mfma_bf16(const void* image, int iters, int workgroups, float* sink,
                                 uint64_t* ticks, moe_stream_t stream);
/* The same probe for the FP8 path: image = two blocks of [256 rows][128 E4M3
 * bytes], 32x32x64 FP8 MFMAs; one launch executes workgroups * iters * 16777216
 * FLOP. */
moe_status_t moe_probe_mfma_fp8(const void* image, int iters, int workgroups, float* sink,
                                uint64_t* ticks, moe_stream_t stream);

/*
 * Clock sample of the grouped bf16 GEMMs (measurement aid, like the probes
 * above).  ticks: DEVICE memory, 2 x uint64, or NULL to switch the sampling off
 * (the default).  While set, workgroup 0 of every grouped bf16 GEMM launch that
 * runs on the persistent kernel (forward, backward) writes ticks[0] = shader
 * clocks and ticks[1] = 100 MHz reference clocks it spent in the kernel, so
 * ticks[0] / ticks[1] * 100 is the shader clock in MHz the launch ran at.  The
 * pointer is process-wide host state read at launch time (not thread-safe); the
 * cells keep the last launch's values and stay untouched by a launch whose
 * workgroup 0 has no tile.  Always MOE_OK unless ticks is misaligned.
 */
moe_status_t moe_gemm_clock_sample(uint64_t* ticks);

/* Tuning knobs for experiments (process-wide, not thread-safe; defaults are
 * the tuned ones).  Unknown names return MOE_ERR_INVALID_ARG.  Names:
 * "gemm_variant" (bf16 expert FFN: 0 = auto = 43 with the one-workgroup-per-tile
 * kernel for layers whose H or F is below 128; 40 / 41 = persistent kernel with
 * three LDS stages for the activation tile, 4 / 8 waves; 42 / 43 = three stages
 * for the weight tile, 4 / 8 waves; 30 / 31 = one workgroup per tile, 4 / 8
 * waves; 99 = the plain LDS-tiled kernel of the fp32 and odd-shape layers;
 * any other value makes the expert calls return MOE_ERR_UNSUPPORTED);
 * "fp8_deep_weights" (FP8 expert GEMMs: 1, the default = three LDS stages for
 * the weight tile, 0 = for the activation tile); "gemm_workgroups" (workgroups launched by the
 * persistent grouped-GEMM kernels; 0 = one per compute unit, values below 8
 * are raised to 8); "router_tile" (16-token blocks per router workgroup: 1, 2
 * or 4; 0 = chosen from T and E); "wgrad_rowmajor" (1 = the expert FFN's backward
 * forms the weight gradients straight from the row-major activations with
 * transposing LDS loads instead of from transposed copies: about 1.8x slower
 * weight-gradient GEMMs, no ragged transposes; default 0); "permute_fused" (1, the default: layers with at most 8 experts and at most
 * 65532 assignments run moe_permute as ONE kernel in which every workgroup counts
 * the whole index array itself while its rows are on their way; 0: always the
 * three-kernel form; 2 / 3 force one / two tokens per wave); "gemm_idle_skip" (the
 * persistent GEMM kernels in which the waves that hold no valid row of a ragged
 * tile skip its multiplications: 1 = always, 0 = never, -1 = for E >= 16, the
 * default). */
moe_status_t moe_set_option(const char* name, int value);

#ifdef __cplusplus
}
#endif
#endif /* MOE_H_ */
