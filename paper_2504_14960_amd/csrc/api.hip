// C ABI of the MoE hot path: host-side argument validation and kernel launches.
// Nothing here touches device data, allocates, or synchronises.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <cmath>

#include "common.h"

namespace moe {

static thread_local char g_err[512] = "";
static int g_gemm_variant = 0;
static int g_wgrad_rowmajor = 0;   // 1: weight gradients straight from the row-major activations (slower, no transposed copies)

moe_status_t fail(moe_status_t st, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return st;
}

moe_status_t check_launch(const char* what) {
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(MOE_ERR_LAUNCH, "%s: %s", what, hipGetErrorString(e));
    return MOE_OK;
}

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

static moe_status_t check_dims(const char* fn, int T, int H, int E, int K, moe_dtype_t dt) {
    if (dt != MOE_F32 && dt != MOE_BF16) return fail(MOE_ERR_INVALID_ARG, "%s: unknown dtype %d", fn, (int)dt);
    if (T < 0 || H <= 0 || E <= 0 || K <= 0)
        return fail(MOE_ERR_INVALID_ARG, "%s: need T >= 0, H, E, K > 0 (T=%d H=%d E=%d K=%d)", fn, T, H, E, K);
    if (K > E) return fail(MOE_ERR_INVALID_ARG, "%s: K=%d exceeds E=%d", fn, K, E);
    if (E > kMaxExperts) return fail(MOE_ERR_UNSUPPORTED, "%s: E=%d exceeds the limit %d", fn, E, kMaxExperts);
    if (K > kMaxTopK) return fail(MOE_ERR_UNSUPPORTED, "%s: K=%d exceeds the limit %d", fn, K, kMaxTopK);
    if ((long long)T * K >= (1ll << 31)) return fail(MOE_ERR_UNSUPPORTED, "%s: T*K must be below 2^31", fn);
    const int vec = (dt == MOE_BF16) ? 8 : 4;
    if (H % vec != 0) return fail(MOE_ERR_UNSUPPORTED, "%s: H=%d must be a multiple of %d", fn, H, vec);
    return MOE_OK;
}

#define REQUIRE_PTR(fn, p)                                                                    \
    do {                                                                                      \
        if ((p) == nullptr) return fail(MOE_ERR_INVALID_ARG, "%s: %s is NULL", fn, #p);       \
        if (!aligned16(p)) return fail(MOE_ERR_INVALID_ARG, "%s: %s is not 16-byte aligned", fn, #p); \
    } while (0)

struct LayerLayout {
    size_t logits, idx, gate, counts, offsets, roa, aor, perm_ws, x_perm, h, y_perm;
    size_t s_offsets, s_h, s_y, total;
    int r_max;
};


static LayerLayout layer_layout(int T, int H, int E, int K, int F, int Fs, int capacity, moe_dtype_t dt) {
    LayerLayout L;
    const size_t es = (dt == MOE_BF16) ? 2 : 4;
    const size_t A = (size_t)T * K;
    L.r_max = moe_max_rows(T, K, E, capacity);
    const size_t R = (size_t)L.r_max;
    size_t o = 0;
    auto take = [&](size_t bytes) { const size_t at = o; o = up256(o + bytes); return at; };
    L.logits = take((size_t)T * E * 4);
    L.idx = take(A * 4);
    L.gate = take(A * 4);
    L.counts = take((size_t)E * 4);
    L.offsets = take((size_t)(E + 1) * 4);
    L.roa = take(A * 4);
    L.aor = take(R * 4);
    L.perm_ws = take(permute_workspace_bytes(T, K, E));
    L.x_perm = take(R * H * es);
    L.h = take(R * F * es);
    L.y_perm = take(R * H * es);
    L.s_offsets = take(2 * 4);
    L.s_h = take(Fs > 0 ? (size_t)T * Fs * es : 0);
    L.s_y = take(Fs > 0 ? (size_t)T * H * es : 0);
    L.total = o;
    return L;
}

}  // namespace moe

using namespace moe;

extern "C" {

const char* moe_last_error(void) { return g_err; }

const char* moe_version(void) { return "moe-hotpath-gfx950 0.1"; }

int moe_capacity_from_factor(double capacity_factor, int T, int K, int E) {
    if (!(capacity_factor > 0.0) || E <= 0) return 0;
    return (int)std::ceil(capacity_factor * (double)T * (double)K / (double)E);
}

int moe_max_rows(int T, int K, int E, int capacity) {
    const long long A = (long long)T * K;
    if (capacity <= 0) return (int)A;
    const long long cap = (long long)E * capacity;
    return (int)(A < cap ? A : cap);
}

size_t moe_permute_workspace_bytes(int T, int K, int E) {
    if (T < 0 || K <= 0 || E <= 0) return 0;
    return permute_workspace_bytes(T, K, E);
}

moe_status_t moe_router_topk(const void* x, const void* w_router, const float* logit_bias,
                             float* logits, int T, int H, int E, int K, int renormalize,
                             moe_dtype_t dt, int32_t* topk_idx, float* topk_gate,
                             moe_stream_t stream) {
    static const char* fn = "moe_router_topk";
    if (x == nullptr) H = (dt == MOE_BF16) ? 8 : 4;  // ignored, keep the shape check quiet
    if (moe_status_t st = check_dims(fn, T, H, E, K, dt)) return st;
    if (T == 0) return MOE_OK;
    REQUIRE_PTR(fn, logits);
    REQUIRE_PTR(fn, topk_idx);
    REQUIRE_PTR(fn, topk_gate);
    if (x != nullptr) {
        REQUIRE_PTR(fn, x);
        REQUIRE_PTR(fn, w_router);
        if (logit_bias && (reinterpret_cast<uintptr_t>(logit_bias) & 3u))
            return fail(MOE_ERR_INVALID_ARG, "%s: logit_bias is not 4-byte aligned", fn);
    }
    launch_router(x, w_router, x ? logit_bias : nullptr, logits, T, H, E, K, renormalize != 0, dt,
                  topk_idx, topk_gate, static_cast<hipStream_t>(stream));
    return check_launch(fn);
}

moe_status_t moe_permute(const void* x, const int32_t* topk_idx, int T, int H, int E, int K,
                         int capacity, moe_dtype_t dt, void* x_perm, int32_t* expert_counts,
                         int32_t* expert_offsets, int32_t* row_of_assign,
                         int32_t* assign_of_row, void* workspace, size_t workspace_bytes,
                         moe_stream_t stream) {
    static const char* fn = "moe_permute";
    if (moe_status_t st = check_dims(fn, T, H, E, K, dt)) return st;
    if ((x == nullptr) != (x_perm == nullptr))
        return fail(MOE_ERR_INVALID_ARG, "%s: x and x_perm must both be given or both be NULL", fn);
    REQUIRE_PTR(fn, expert_counts);
    REQUIRE_PTR(fn, expert_offsets);
    if (T == 0) {
        // nothing routed: all experts empty
        launch_fill_i32(expert_counts, E, 0, 0, static_cast<hipStream_t>(stream));
        launch_fill_i32(expert_offsets, E + 1, 0, 0, static_cast<hipStream_t>(stream));
        return check_launch(fn);
    }
    REQUIRE_PTR(fn, topk_idx);
    REQUIRE_PTR(fn, row_of_assign);
    REQUIRE_PTR(fn, assign_of_row);
    if (x) {
        REQUIRE_PTR(fn, x);
        REQUIRE_PTR(fn, x_perm);
    }
    const size_t need = permute_workspace_bytes(T, K, E);
    if (workspace == nullptr || workspace_bytes < need)
        return fail(MOE_ERR_WORKSPACE, "%s: workspace of %zu bytes needed, %zu given", fn, need,
                    workspace ? workspace_bytes : (size_t)0);
    REQUIRE_PTR(fn, workspace);
    const int r_max = moe_max_rows(T, K, E, capacity);
    launch_permute(x, topk_idx, T, H, E, K, capacity, r_max, dt, x_perm, expert_counts,
                   expert_offsets, row_of_assign, assign_of_row, workspace,
                   static_cast<hipStream_t>(stream));
    return check_launch(fn);
}

moe_status_t moe_permute_noalloc(const void* x, const int32_t* topk_idx, int T, int H, int E, int K,
                                 int capacity, moe_dtype_t dt, void* x_perm, int32_t* expert_counts,
                                 int32_t* expert_offsets, int32_t* row_of_assign,
                                 int32_t* assign_of_row, moe_stream_t stream) {
    static const char* fn = "moe_permute_noalloc";
    if (moe_status_t st = check_dims(fn, T, H, E, K, dt)) return st;
    // the size limit first: it needs no GPU
    const size_t need = permute_workspace_bytes(T, K, E);
    if (need > permute_scratch_bytes())
        return fail(MOE_ERR_UNSUPPORTED,
                    "%s: T*K=%lld assignments over E=%d experts need %zu bytes of scratch, the library holds %zu; "
                    "use moe_permute with a workspace",
                    fn, (long long)T * K, E, need, permute_scratch_bytes());
    if (T == 0)   // no scratch involved
        return moe_permute(x, topk_idx, T, H, E, K, capacity, dt, x_perm, expert_counts, expert_offsets,
                           row_of_assign, assign_of_row, nullptr, 0, stream);
    hipError_t err = hipSuccess;
    int32_t* ws = permute_scratch(&err);
    if (ws == nullptr) return fail(MOE_ERR_LAUNCH, "%s: no address for the scratch array: %s", fn, hipGetErrorString(err));
    return moe_permute(x, topk_idx, T, H, E, K, capacity, dt, x_perm, expert_counts, expert_offsets, row_of_assign,
                       assign_of_row, ws, permute_scratch_bytes(), stream);
}

size_t moe_permute_variant_workspace_bytes(int T, int K, int E) {
    if (T < 0 || K <= 0 || E <= 0) return 0;
    return permute_variant_workspace_bytes(T, K, E);
}

moe_status_t moe_permute_variant(const void* x, const int32_t* topk_idx, const float* scores, int T,
                                 int H, int E, int K, int capacity, int drop_by_score,
                                 int pad_to_capacity, moe_dtype_t dt, void* x_perm,
                                 int32_t* expert_counts, int32_t* expert_offsets,
                                 int32_t* row_of_assign, int32_t* assign_of_row, int R_max,
                                 void* workspace, size_t workspace_bytes, moe_stream_t stream) {
    static const char* fn = "moe_permute_variant";
    if (moe_status_t st = check_dims(fn, T, H, E, K, dt)) return st;
    if ((x == nullptr) != (x_perm == nullptr))
        return fail(MOE_ERR_INVALID_ARG, "%s: x and x_perm must both be given or both be NULL", fn);
    if (pad_to_capacity && capacity <= 0)
        return fail(MOE_ERR_INVALID_ARG, "%s: the padded layout needs capacity > 0", fn);
    if (capacity <= 0) drop_by_score = 0;   // nothing is dropped: the rule plays no part
    const long long need_rows = pad_to_capacity ? (long long)E * capacity : moe_max_rows(T, K, E, capacity);
    if (need_rows > INT32_MAX) return fail(MOE_ERR_UNSUPPORTED, "%s: E * capacity exceeds the int32 row index", fn);
    if (R_max < need_rows)
        return fail(MOE_ERR_INVALID_ARG, "%s: R_max=%d, but this dispatch can produce %lld rows", fn, R_max, need_rows);
    REQUIRE_PTR(fn, expert_counts);
    REQUIRE_PTR(fn, expert_offsets);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (T == 0) {
        launch_fill_i32(expert_counts, E, 0, 0, s);
        launch_fill_i32(expert_offsets, E + 1, 0, pad_to_capacity ? capacity : 0, s);
        if (R_max > 0) {
            REQUIRE_PTR(fn, assign_of_row);
            launch_fill_i32(assign_of_row, R_max, -1, 0, s);
            if (pad_to_capacity && x_perm)
                launch_permute_zero_rows(assign_of_row, x_perm, R_max, H * (dt == MOE_BF16 ? 2 : 4), s);
        }
        return check_launch(fn);
    }
    REQUIRE_PTR(fn, topk_idx);
    REQUIRE_PTR(fn, row_of_assign);
    REQUIRE_PTR(fn, assign_of_row);
    if (drop_by_score) REQUIRE_PTR(fn, scores);
    const size_t need = permute_variant_workspace_bytes(T, K, E);
    if (workspace == nullptr || workspace_bytes < need)
        return fail(MOE_ERR_WORKSPACE, "%s: workspace of %zu bytes needed, %zu given", fn, need,
                    workspace ? workspace_bytes : (size_t)0);
    REQUIRE_PTR(fn, workspace);
    launch_permute_variant(x, topk_idx, scores, T, H, E, K, capacity, drop_by_score, pad_to_capacity, R_max, dt,
                           x_perm, expert_counts, expert_offsets, row_of_assign, assign_of_row, workspace, s);
    return check_launch(fn);
}

size_t moe_sort_chunks_workspace_bytes(int n_dst) {
    if (n_dst < 0 || n_dst > sort_chunks_max_chunks()) return 0;
    return sort_chunks_workspace_bytes(n_dst);
}

moe_status_t moe_sort_chunks(const void* src, int R_src, const int32_t* chunk_rows, int n_src,
                             const int32_t* order, int n_dst, int group, int H, moe_dtype_t dt,
                             void* dst, int R_dst, int32_t* chunk_rows_out, int32_t* group_offsets,
                             void* workspace, size_t workspace_bytes, moe_stream_t stream) {
    static const char* fn = "moe_sort_chunks";
    if (dt != MOE_F32 && dt != MOE_BF16) return fail(MOE_ERR_INVALID_ARG, "%s: unknown dtype %d", fn, (int)dt);
    if (R_src < 0 || R_dst < 0 || n_src < 0 || n_dst < 0 || H <= 0 || group < 0)
        return fail(MOE_ERR_INVALID_ARG, "%s: need R_src, R_dst, n_src, n_dst, group >= 0 and H > 0", fn);
    if (n_src > sort_chunks_max_chunks() || n_dst > sort_chunks_max_chunks())
        return fail(MOE_ERR_UNSUPPORTED, "%s: n_src=%d, n_dst=%d exceed the limit %d", fn, n_src, n_dst,
                    sort_chunks_max_chunks());
    const long long row_bytes = (long long)H * (dt == MOE_BF16 ? 2 : 4);
    if (row_bytes % 16 || row_bytes > INT32_MAX)
        return fail(MOE_ERR_UNSUPPORTED, "%s: a row of %lld bytes is not a multiple of 16", fn, row_bytes);
    if (group_offsets != nullptr && group <= 0)
        return fail(MOE_ERR_INVALID_ARG, "%s: group_offsets needs group > 0", fn);
    if (n_src > 0) REQUIRE_PTR(fn, chunk_rows);
    if (n_dst > 0) REQUIRE_PTR(fn, order);
    if (src != nullptr && dst != nullptr && R_src > 0 && R_dst > 0) {
        const char* a = static_cast<const char*>(src);
        const char* b = static_cast<const char*>(dst);
        if (a < b + (size_t)R_dst * row_bytes && b < a + (size_t)R_src * row_bytes)
            return fail(MOE_ERR_INVALID_ARG, "%s: src and dst overlap", fn);
    }
    const size_t need = sort_chunks_workspace_bytes(n_dst);
    if (workspace == nullptr || workspace_bytes < need)
        return fail(MOE_ERR_WORKSPACE, "%s: workspace of %zu bytes needed, %zu given", fn, need,
                    workspace ? workspace_bytes : (size_t)0);
    launch_sort_chunks(src, R_src, chunk_rows, n_src, order, n_dst, group_offsets ? group : 0, (int)row_bytes, dst,
                       R_dst, chunk_rows_out, group_offsets, workspace, static_cast<hipStream_t>(stream));
    return check_launch(fn);
}

static moe_status_t expert_ffn(const char* fn, int phase, const void* x_perm,
                               const int32_t* expert_offsets, int R_max, int H, int F, int E,
                               const void* w_gate, const void* w_up, const void* w_down,
                               moe_dtype_t dt, void* h, void* y_perm, moe_stream_t stream) {
    if (dt != MOE_F32 && dt != MOE_BF16) return fail(MOE_ERR_INVALID_ARG, "%s: unknown dtype %d", fn, (int)dt);
    if (R_max < 0 || H <= 0 || F <= 0 || E <= 0)
        return fail(MOE_ERR_INVALID_ARG, "%s: need R_max >= 0 and H, F, E > 0", fn);
    if (E > kMaxExperts) return fail(MOE_ERR_UNSUPPORTED, "%s: E=%d exceeds the limit %d", fn, E, kMaxExperts);
    const int vec = (dt == MOE_BF16) ? 8 : 4;
    if (H % vec || F % vec)
        return fail(MOE_ERR_UNSUPPORTED, "%s: H=%d and F=%d must be multiples of %d", fn, H, F, vec);
    if (R_max == 0) return MOE_OK;
    REQUIRE_PTR(fn, expert_offsets);
    REQUIRE_PTR(fn, h);
    if (phase & 1) {
        REQUIRE_PTR(fn, x_perm);
        REQUIRE_PTR(fn, w_gate);
        REQUIRE_PTR(fn, w_up);
    }
    if (phase & 2) {
        REQUIRE_PTR(fn, w_down);
        REQUIRE_PTR(fn, y_perm);
    }
    if (!launch_expert_ffn(x_perm, expert_offsets, R_max, H, F, E, w_gate, w_up, w_down, dt, h, y_perm,
                           g_gemm_variant, phase, static_cast<hipStream_t>(stream)))
        return fail(MOE_ERR_UNSUPPORTED, "%s: no kernel for H=%d F=%d", fn, H, F);
    return check_launch(fn);
}

moe_status_t moe_grouped_gemm_swiglu(const void* x_perm, const int32_t* expert_offsets, int R_max,
                                     int H, int F, int E, const void* w_gate, const void* w_up,
                                     const void* w_down, moe_dtype_t dt, void* h_workspace,
                                     void* y_perm, moe_stream_t stream) {
    return expert_ffn("moe_grouped_gemm_swiglu", 3, x_perm, expert_offsets, R_max, H, F, E, w_gate, w_up,
                      w_down, dt, h_workspace, y_perm, stream);
}

moe_status_t moe_expert_gate_up(const void* x_perm, const int32_t* expert_offsets, int R_max, int H,
                                int F, int E, const void* w_gate, const void* w_up, moe_dtype_t dt,
                                void* h, moe_stream_t stream) {
    return expert_ffn("moe_expert_gate_up", 1, x_perm, expert_offsets, R_max, H, F, E, w_gate, w_up,
                      nullptr, dt, h, nullptr, stream);
}

moe_status_t moe_expert_down(const void* h, const int32_t* expert_offsets, int R_max, int H, int F,
                             int E, const void* w_down, moe_dtype_t dt, void* y_perm,
                             moe_stream_t stream) {
    return expert_ffn("moe_expert_down", 2, nullptr, expert_offsets, R_max, H, F, E, nullptr, nullptr,
                      w_down, dt, const_cast<void*>(h), y_perm, stream);
}

moe_status_t moe_unpermute_combine(const void* y_perm, const int32_t* row_of_assign,
                                   const float* topk_gate, const void* addend, int T, int H,
                                   int K, int R_max, moe_dtype_t dt, void* y, moe_stream_t stream) {
    static const char* fn = "moe_unpermute_combine";
    if (moe_status_t st = check_dims(fn, T, H, K, K, dt)) return st;  // E plays no part here
    if (R_max < 0) return fail(MOE_ERR_INVALID_ARG, "%s: R_max=%d is negative", fn, R_max);
    if (T == 0) return MOE_OK;
    REQUIRE_PTR(fn, row_of_assign);
    REQUIRE_PTR(fn, topk_gate);
    REQUIRE_PTR(fn, y);
    if (R_max > 0) REQUIRE_PTR(fn, y_perm);
    if (addend && !aligned16(addend)) return fail(MOE_ERR_INVALID_ARG, "%s: addend is not 16-byte aligned", fn);
    launch_combine(y_perm, row_of_assign, topk_gate, addend, T, H, K, R_max, dt, y,
                   static_cast<hipStream_t>(stream));
    return check_launch(fn);
}

moe_status_t moe_unpermute_combine_backward(const void* dy, const void* y_perm,
                                            const int32_t* row_of_assign, const float* topk_gate,
                                            int T, int H, int K, int R_max, moe_dtype_t dt,
                                            void* dy_perm, float* dgate, moe_stream_t stream) {
    static const char* fn = "moe_unpermute_combine_backward";
    if (moe_status_t st = check_dims(fn, T, H, K, K, dt)) return st;
    if (R_max < 0) return fail(MOE_ERR_INVALID_ARG, "%s: R_max=%d is negative", fn, R_max);
    if (T == 0) return MOE_OK;
    REQUIRE_PTR(fn, dy);
    REQUIRE_PTR(fn, row_of_assign);
    REQUIRE_PTR(fn, topk_gate);
    REQUIRE_PTR(fn, dgate);
    if (R_max > 0) {
        REQUIRE_PTR(fn, y_perm);
        REQUIRE_PTR(fn, dy_perm);
    }
    launch_combine_backward(dy, y_perm, row_of_assign, topk_gate, T, H, K, R_max, dt, dy_perm, dgate,
                            static_cast<hipStream_t>(stream));
    return check_launch(fn);
}

moe_status_t moe_permute_backward(const void* dx_perm, const int32_t* row_of_assign,
                                  const void* addend, int T, int H, int K, int R_max,
                                  moe_dtype_t dt, void* dx, moe_stream_t stream) {
    static const char* fn = "moe_permute_backward";
    if (moe_status_t st = check_dims(fn, T, H, K, K, dt)) return st;
    if (R_max < 0) return fail(MOE_ERR_INVALID_ARG, "%s: R_max=%d is negative", fn, R_max);
    if (T == 0) return MOE_OK;
    REQUIRE_PTR(fn, row_of_assign);
    REQUIRE_PTR(fn, dx);
    if (R_max > 0) REQUIRE_PTR(fn, dx_perm);
    if (addend && !aligned16(addend)) return fail(MOE_ERR_INVALID_ARG, "%s: addend is not 16-byte aligned", fn);
    // the sum of the kept rows of every token: the combine without gates
    launch_combine(dx_perm, row_of_assign, nullptr, addend, T, H, K, R_max, dt, dx, static_cast<hipStream_t>(stream));
    return check_launch(fn);
}

size_t moe_router_backward_workspace_bytes(int T, int H, int E) {
    if (T < 0 || H <= 0 || E <= 0) return 0;
    return router_backward_workspace_bytes(T, H, E);
}

moe_status_t moe_router_backward(const void* x, const void* w_router, const float* logits,
                                 const int32_t* topk_idx, const float* dgate, int T, int H, int E,
                                 int K, int renormalize, moe_dtype_t dt, float* dlogits, void* dx,
                                 float* dw_router, float* dbias, void* workspace,
                                 size_t workspace_bytes, moe_stream_t stream) {
    static const char* fn = "moe_router_backward";
    if (moe_status_t st = check_dims(fn, T, H, E, K, dt)) return st;
    if (H % 8) return fail(MOE_ERR_UNSUPPORTED, "%s: H=%d must be a multiple of 8", fn, H);
    if (T == 0) {
        // no tokens: the sums over tokens are zero
        if (dw_router) launch_fill_i32(reinterpret_cast<int32_t*>(dw_router), E * H, 0, 0, static_cast<hipStream_t>(stream));
        if (dbias) launch_fill_i32(reinterpret_cast<int32_t*>(dbias), E, 0, 0, static_cast<hipStream_t>(stream));
        return check_launch(fn);
    }
    REQUIRE_PTR(fn, logits);
    REQUIRE_PTR(fn, topk_idx);
    REQUIRE_PTR(fn, dgate);
    REQUIRE_PTR(fn, dlogits);
    if (dx) {
        REQUIRE_PTR(fn, dx);
        REQUIRE_PTR(fn, w_router);
    }
    if (dw_router) {
        REQUIRE_PTR(fn, dw_router);
        REQUIRE_PTR(fn, x);
        const size_t need = router_backward_workspace_bytes(T, H, E);
        if (workspace == nullptr || workspace_bytes < need)
            return fail(MOE_ERR_WORKSPACE, "%s: workspace of %zu bytes needed, %zu given", fn, need,
                        workspace ? workspace_bytes : (size_t)0);
        REQUIRE_PTR(fn, workspace);
    }
    if (dbias && (reinterpret_cast<uintptr_t>(dbias) & 3u)) return fail(MOE_ERR_INVALID_ARG, "%s: dbias is not 4-byte aligned", fn);
    launch_router_backward(x, w_router, logits, topk_idx, dgate, T, H, E, K, renormalize != 0, dt, dlogits, dx,
                           dw_router, dbias, workspace, static_cast<hipStream_t>(stream));
    return check_launch(fn);
}

struct BackwardLayout {
    size_t g, u, dh, dgdu, dy_t, h_t, dgdu_t, x_t, poff, zero, total;
    int rp_max;
};

static BackwardLayout backward_layout(int R_max, int H, int F, int E) {
    BackwardLayout L;
    // bound on the padded column axis of the transposed activations: every non-empty expert's
    // segment is at most 127 columns longer than its row count
    const long long nonempty = E < R_max ? E : R_max;
    L.rp_max = (int)(((long long)R_max + 127 * nonempty + 63) / 64 * 64);
    size_t o = 0;
    auto take = [&](size_t bytes) { const size_t at = o; o += up256(bytes); return at; };
    const size_t rf = (size_t)R_max * F * 2;
    L.g = take(rf);
    L.u = take(rf);
    L.dh = take(rf);
    L.dgdu = take(2 * rf);
    L.dy_t = take((size_t)H * L.rp_max * 2);
    L.h_t = take((size_t)F * L.rp_max * 2);
    L.dgdu_t = take((size_t)2 * F * L.rp_max * 2);
    L.x_t = take((size_t)H * L.rp_max * 2);
    L.poff = take((size_t)(E + 1) * 4);
    L.zero = take(1024);
    L.total = o;
    return L;
}

static bool backward_supported(int H, int F) { return H % 128 == 0 && F % 128 == 0 && H >= 128 && F >= 128; }

size_t moe_expert_backward_workspace_bytes(int R_max, int H, int F, int E) {
    if (R_max < 0 || H <= 0 || F <= 0 || E <= 0) return 0;
    return backward_layout(R_max, H, F, E).total;
}

moe_status_t moe_expert_weights_transpose(const void* w_gate, const void* w_up, const void* w_down,
                                          int H, int F, int E, void* wgu_t, void* wd_t,
                                          moe_stream_t stream) {
    static const char* fn = "moe_expert_weights_transpose";
    if (H <= 0 || F <= 0 || E <= 0) return fail(MOE_ERR_INVALID_ARG, "%s: need H, F, E > 0", fn);
    if (!backward_supported(H, F)) return fail(MOE_ERR_UNSUPPORTED, "%s: H=%d and F=%d must be multiples of 128", fn, H, F);
    REQUIRE_PTR(fn, w_gate);
    REQUIRE_PTR(fn, w_up);
    REQUIRE_PTR(fn, w_down);
    REQUIRE_PTR(fn, wgu_t);
    REQUIRE_PTR(fn, wd_t);
    hipStream_t s = static_cast<hipStream_t>(stream);
    launch_transpose_batched(w_gate, E, F, H, wgu_t, (size_t)2 * F, 0, s);   // [E,F,H] -> [E,H,0:F]
    launch_transpose_batched(w_up, E, F, H, wgu_t, (size_t)2 * F, F, s);     //            [E,H,F:2F]
    launch_transpose_batched(w_down, E, H, F, wd_t, (size_t)H, 0, s);        // [E,H,F] -> [E,F,H]
    return check_launch(fn);
}

moe_status_t moe_expert_gate_up_saving(const void* x_perm, const int32_t* expert_offsets, int R_max,
                                       int H, int F, int E, const void* w_gate, const void* w_up,
                                       void* h, void* gu, moe_stream_t stream) {
    static const char* fn = "moe_expert_gate_up_saving";
    if (R_max < 0 || H <= 0 || F <= 0 || E <= 0) return fail(MOE_ERR_INVALID_ARG, "%s: need R_max >= 0 and H, F, E > 0", fn);
    if (E > kMaxExperts) return fail(MOE_ERR_UNSUPPORTED, "%s: E=%d exceeds the limit %d", fn, E, kMaxExperts);
    if (!backward_supported(H, F)) return fail(MOE_ERR_UNSUPPORTED, "%s: H=%d and F=%d must be multiples of 128", fn, H, F);
    if (R_max == 0) return MOE_OK;
    REQUIRE_PTR(fn, x_perm);
    REQUIRE_PTR(fn, expert_offsets);
    REQUIRE_PTR(fn, w_gate);
    REQUIRE_PTR(fn, w_up);
    REQUIRE_PTR(fn, h);
    REQUIRE_PTR(fn, gu);
    if (!launch_gate_up_saving(x_perm, expert_offsets, R_max, H, F, E, w_gate, w_up, h, gu,
                               static_cast<hipStream_t>(stream)))
        return fail(MOE_ERR_UNSUPPORTED, "%s: no kernel for H=%d F=%d", fn, H, F);
    return check_launch(fn);
}

moe_status_t moe_grouped_gemm_swiglu_backward(const void* x_perm, const void* h, const void* gu,
                                              const void* dy_perm,
                                              const int32_t* expert_offsets, int R_max, int H, int F,
                                              int E, const void* w_gate, const void* w_up,
                                              const void* wgu_t, const void* wd_t, void* dx_perm,
                                              void* dw_gate, void* dw_up, void* dw_down,
                                              void* workspace, size_t workspace_bytes,
                                              moe_stream_t stream) {
    static const char* fn = "moe_grouped_gemm_swiglu_backward";
    if (R_max < 0 || H <= 0 || F <= 0 || E <= 0) return fail(MOE_ERR_INVALID_ARG, "%s: need R_max >= 0 and H, F, E > 0", fn);
    if (E > kMaxExperts) return fail(MOE_ERR_UNSUPPORTED, "%s: E=%d exceeds the limit %d", fn, E, kMaxExperts);
    if (!backward_supported(H, F)) return fail(MOE_ERR_UNSUPPORTED, "%s: H=%d and F=%d must be multiples of 128", fn, H, F);
    REQUIRE_PTR(fn, expert_offsets);
    REQUIRE_PTR(fn, dw_gate);
    REQUIRE_PTR(fn, dw_up);
    REQUIRE_PTR(fn, dw_down);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const BackwardLayout L = backward_layout(R_max, H, F, E);
    if (R_max > 0) {
        REQUIRE_PTR(fn, x_perm);
        REQUIRE_PTR(fn, h);
        REQUIRE_PTR(fn, dy_perm);
        if (gu == nullptr) {
            REQUIRE_PTR(fn, w_gate);
            REQUIRE_PTR(fn, w_up);
        } else if (!aligned16(gu)) {
            return fail(MOE_ERR_INVALID_ARG, "%s: gu is not 16-byte aligned", fn);
        }
        REQUIRE_PTR(fn, wgu_t);
        REQUIRE_PTR(fn, wd_t);
        REQUIRE_PTR(fn, dx_perm);
        if (workspace == nullptr || workspace_bytes < L.total)
            return fail(MOE_ERR_WORKSPACE, "%s: workspace of %zu bytes needed, %zu given", fn, L.total,
                        workspace ? workspace_bytes : (size_t)0);
        REQUIRE_PTR(fn, workspace);
    }
    uint8_t* ws = static_cast<uint8_t*>(workspace);
    if (R_max > 0) {
        // g and u (the forward's, or recomputed); dh; the SwiGLU's derivative; the input gradient
        bool ok = true;
        if (gu == nullptr) {
            ok = launch_grouped_nt(x_perm, expert_offsets, R_max, E, F, H, w_gate, ws + L.g, s);
            ok = ok && launch_grouped_nt(x_perm, expert_offsets, R_max, E, F, H, w_up, ws + L.u, s);
        }
        if (gu) {
            // dh is formed in the GEMM's accumulators and turned into dg | du in its epilogue
            ok = launch_grouped_nt_swiglu_bwd(dy_perm, expert_offsets, R_max, E, F, H, wd_t, gu, ws + L.dgdu, s);
        } else {
            ok = ok && launch_grouped_nt(dy_perm, expert_offsets, R_max, E, F, H, wd_t, ws + L.dh, s);
            if (ok)
                launch_swiglu_backward(ws + L.dh, ws + L.g, ws + L.u, (size_t)F, expert_offsets + E, R_max, F,
                                       ws + L.dgdu, s);
        }
        if (!ok) return fail(MOE_ERR_UNSUPPORTED, "%s: no kernel for H=%d F=%d", fn, H, F);
        if (!launch_grouped_nt(ws + L.dgdu, expert_offsets, R_max, E, H, 2 * F, wgu_t, dx_perm, s))
            return fail(MOE_ERR_UNSUPPORTED, "%s: no kernel for H=%d F=%d", fn, H, F);
    }
    const bool pipe3 = g_gemm_variant == 30 || g_gemm_variant == 31;
    if (g_wgrad_rowmajor && !pipe3) {
        // weight gradients straight from the row-major activations; rows past an expert's end read a zero row
        if (R_max > 0) {
            launch_fill_i32(reinterpret_cast<int32_t*>(ws + L.zero), 256, 0, 0, s);
            launch_persist_wgrad_rowmajor(dy_perm, H, h, F, expert_offsets, E, H, F, ws + L.zero, dw_down, s);
            launch_persist_wgrad_rowmajor(ws + L.dgdu, 2 * F, x_perm, H, expert_offsets, E, F, H, ws + L.zero, dw_gate, s);
            launch_persist_wgrad_rowmajor(ws + L.dgdu + (size_t)F * 2, 2 * F, x_perm, H, expert_offsets, E, F, H,
                                          ws + L.zero, dw_up, s);
            return check_launch(fn);
        }
    } else if (R_max > 0) {
        // operands of the weight gradients, transposed with every expert's rows as a zero-padded column segment
        int32_t* poff = reinterpret_cast<int32_t*>(ws + L.poff);
        launch_ragged_offsets(expert_offsets, E, poff, s);
        launch_ragged_transpose(dy_perm, expert_offsets, poff, E, H, L.rp_max, ws + L.dy_t, s);
        launch_ragged_transpose(h, expert_offsets, poff, E, F, L.rp_max, ws + L.h_t, s);
        launch_ragged_transpose(ws + L.dgdu, expert_offsets, poff, E, 2 * F, L.rp_max, ws + L.dgdu_t, s);
        launch_ragged_transpose(x_perm, expert_offsets, poff, E, H, L.rp_max, ws + L.x_t, s);
    }
    // with R_max == 0 every segment is empty and the three launches below write zeros without reading
    const int ld = R_max > 0 ? L.rp_max : 64;
    // "gemm_variant" 30 / 31 select the one-workgroup-per-tile kernel, anything else the persistent one
    auto wgrad = pipe3 ? launch_pipe3_wgrad : launch_persist_wgrad;
    wgrad(ws + L.dy_t, ws + L.h_t, expert_offsets, E, H, F, ld, dw_down, s);
    wgrad(ws + L.dgdu_t, ws + L.x_t, expert_offsets, E, F, H, ld, dw_gate, s);
    wgrad(ws + L.dgdu_t + (size_t)F * ld * 2, ws + L.x_t, expert_offsets, E, F, H, ld, dw_up, s);
    return check_launch(fn);
}

size_t moe_layer_workspace_bytes(int T, int H, int E, int K, int F, int Fs, int capacity,
                                 moe_dtype_t dt) {
    if (T < 0 || H <= 0 || E <= 0 || K <= 0 || F <= 0 || Fs < 0) return 0;
    return layer_layout(T, H, E, K, F, Fs, capacity, dt).total;
}

size_t moe_workspace_bytes(int T, int H, int E, int K, int F, int capacity, moe_dtype_t dt) {
    return moe_layer_workspace_bytes(T, H, E, K, F, 0, capacity, dt);
}

moe_status_t moe_layer_workspace_layout(int T, int H, int E, int K, int F, int Fs, int capacity,
                                        moe_dtype_t dt, size_t* byte_offsets, int n) {
    if (byte_offsets == nullptr || n < 11) return fail(MOE_ERR_INVALID_ARG, "moe_layer_workspace_layout: need room for 11 offsets");
    const LayerLayout L = layer_layout(T, H, E, K, F, Fs, capacity, dt);
    const size_t v[11] = {L.logits, L.idx, L.gate, L.counts, L.offsets, L.roa, L.aor, L.x_perm, L.h, L.y_perm, L.s_y};
    memcpy(byte_offsets, v, sizeof v);
    return MOE_OK;
}

moe_status_t moe_layer_forward(const void* x, const void* w_router, const float* logit_bias,
                               const void* w_gate, const void* w_up, const void* w_down,
                               const void* ws_gate, const void* ws_up, const void* ws_down,
                               int T, int H, int E, int K, int F, int Fs, int renormalize,
                               int capacity, moe_dtype_t dt, void* y, void* workspace,
                               size_t workspace_bytes, moe_stream_t stream) {
    static const char* fn = "moe_layer_forward";
    if (moe_status_t st = check_dims(fn, T, H, E, K, dt)) return st;
    if (F <= 0 || Fs < 0) return fail(MOE_ERR_INVALID_ARG, "%s: need F > 0 and Fs >= 0", fn);
    const bool shared = Fs > 0;
    if (shared && !(ws_gate && ws_up && ws_down))
        return fail(MOE_ERR_INVALID_ARG, "%s: Fs > 0 needs ws_gate, ws_up and ws_down", fn);
    if (T == 0) return MOE_OK;
    REQUIRE_PTR(fn, y);
    const LayerLayout L = layer_layout(T, H, E, K, F, Fs, capacity, dt);
    if (workspace == nullptr || workspace_bytes < L.total)
        return fail(MOE_ERR_WORKSPACE, "%s: workspace of %zu bytes needed, %zu given", fn, L.total,
                    workspace ? workspace_bytes : (size_t)0);
    REQUIRE_PTR(fn, workspace);
    uint8_t* ws = static_cast<uint8_t*>(workspace);
    float* logits = reinterpret_cast<float*>(ws + L.logits);
    int32_t* idx = reinterpret_cast<int32_t*>(ws + L.idx);
    float* gate = reinterpret_cast<float*>(ws + L.gate);
    int32_t* counts = reinterpret_cast<int32_t*>(ws + L.counts);
    int32_t* offsets = reinterpret_cast<int32_t*>(ws + L.offsets);
    int32_t* roa = reinterpret_cast<int32_t*>(ws + L.roa);
    int32_t* aor = reinterpret_cast<int32_t*>(ws + L.aor);

    moe_status_t st = moe_router_topk(x, w_router, logit_bias, logits, T, H, E, K, renormalize, dt,
                                      idx, gate, stream);
    if (st) return st;
    st = moe_permute(x, idx, T, H, E, K, capacity, dt, ws + L.x_perm, counts, offsets, roa, aor,
                     ws + L.perm_ws, permute_workspace_bytes(T, K, E), stream);
    if (st) return st;
    st = moe_grouped_gemm_swiglu(ws + L.x_perm, offsets, L.r_max, H, F, E, w_gate, w_up, w_down, dt,
                                 ws + L.h, ws + L.y_perm, stream);
    if (st) return st;
    const void* addend = nullptr;
    if (shared) {
        // the shared expert sees every token: one "expert" owning rows [0, T)
        int32_t* so = reinterpret_cast<int32_t*>(ws + L.s_offsets);
        launch_fill_i32(so, 2, 0, T, static_cast<hipStream_t>(stream));
        st = moe_grouped_gemm_swiglu(x, so, T, H, Fs, 1, ws_gate, ws_up, ws_down, dt, ws + L.s_h,
                                     ws + L.s_y, stream);
        if (st) return st;
        addend = ws + L.s_y;
    }
    return moe_unpermute_combine(ws + L.y_perm, roa, gate, addend, T, H, K, L.r_max, dt, y, stream);
}

moe_status_t moe_layer_forward_train(const void* x, const void* w_router, const float* logit_bias,
                                     const void* w_gate, const void* w_up, const void* w_down, int T,
                                     int H, int E, int K, int F, int renormalize, int capacity, void* y,
                                     void* gu, void* workspace, size_t workspace_bytes,
                                     moe_stream_t stream) {
    static const char* fn = "moe_layer_forward_train";
    if (moe_status_t st = check_dims(fn, T, H, E, K, MOE_BF16)) return st;
    if (F <= 0) return fail(MOE_ERR_INVALID_ARG, "%s: need F > 0", fn);
    if (T == 0) return MOE_OK;
    REQUIRE_PTR(fn, y);
    REQUIRE_PTR(fn, gu);
    const LayerLayout L = layer_layout(T, H, E, K, F, 0, capacity, MOE_BF16);
    if (workspace == nullptr || workspace_bytes < L.total)
        return fail(MOE_ERR_WORKSPACE, "%s: workspace of %zu bytes needed, %zu given", fn, L.total,
                    workspace ? workspace_bytes : (size_t)0);
    REQUIRE_PTR(fn, workspace);
    uint8_t* ws = static_cast<uint8_t*>(workspace);
    float* logits = reinterpret_cast<float*>(ws + L.logits);
    int32_t* idx = reinterpret_cast<int32_t*>(ws + L.idx);
    float* gate = reinterpret_cast<float*>(ws + L.gate);
    int32_t* offsets = reinterpret_cast<int32_t*>(ws + L.offsets);
    int32_t* roa = reinterpret_cast<int32_t*>(ws + L.roa);
    moe_status_t st = moe_router_topk(x, w_router, logit_bias, logits, T, H, E, K, renormalize, MOE_BF16, idx,
                                      gate, stream);
    if (st) return st;
    st = moe_permute(x, idx, T, H, E, K, capacity, MOE_BF16, ws + L.x_perm, reinterpret_cast<int32_t*>(ws + L.counts),
                     offsets, roa, reinterpret_cast<int32_t*>(ws + L.aor), ws + L.perm_ws,
                     permute_workspace_bytes(T, K, E), stream);
    if (st) return st;
    st = moe_expert_gate_up_saving(ws + L.x_perm, offsets, L.r_max, H, F, E, w_gate, w_up, ws + L.h, gu, stream);
    if (st) return st;
    st = moe_expert_down(ws + L.h, offsets, L.r_max, H, F, E, w_down, MOE_BF16, ws + L.y_perm, stream);
    if (st) return st;
    return moe_unpermute_combine(ws + L.y_perm, roa, gate, nullptr, T, H, K, L.r_max, MOE_BF16, y, stream);
}

struct LayerBackwardLayout {
    size_t dy_perm, dx_perm, dgate, dlogits, dx_router, expert_ws, router_ws, total;
    size_t expert_bytes, router_bytes;
    int r_max;
};

static LayerBackwardLayout layer_backward_layout(int T, int H, int E, int K, int F, int capacity) {
    LayerBackwardLayout L;
    L.r_max = moe_max_rows(T, K, E, capacity);
    const size_t R = (size_t)L.r_max;
    size_t o = 0;
    auto take = [&](size_t bytes) { const size_t at = o; o = up256(o + bytes); return at; };
    L.dy_perm = take(R * H * 2);
    L.dx_perm = take(R * H * 2);
    L.dgate = take((size_t)T * K * 4);
    L.dlogits = take((size_t)T * E * 4);
    L.dx_router = take((size_t)T * H * 2);
    L.expert_bytes = moe_expert_backward_workspace_bytes(L.r_max, H, F, E);
    L.expert_ws = take(L.expert_bytes);
    L.router_bytes = router_backward_workspace_bytes(T, H, E);
    L.router_ws = take(L.router_bytes);
    L.total = o;
    return L;
}

size_t moe_layer_backward_workspace_bytes(int T, int H, int E, int K, int F, int capacity) {
    if (T < 0 || H <= 0 || E <= 0 || K <= 0 || F <= 0) return 0;
    return layer_backward_layout(T, H, E, K, F, capacity).total;
}

moe_status_t moe_layer_backward(const void* x, const void* w_router, const void* w_gate,
                                const void* w_up, const void* wgu_t, const void* wd_t, const void* dy,
                                int T, int H, int E, int K, int F, int renormalize, int capacity,
                                const void* forward_workspace, const void* gu, void* dx,
                                float* dw_router, float* dbias, void* dw_gate, void* dw_up,
                                void* dw_down, void* workspace, size_t workspace_bytes,
                                moe_stream_t stream) {
    static const char* fn = "moe_layer_backward";
    if (moe_status_t st = check_dims(fn, T, H, E, K, MOE_BF16)) return st;
    if (F <= 0) return fail(MOE_ERR_INVALID_ARG, "%s: need F > 0", fn);
    REQUIRE_PTR(fn, forward_workspace);
    REQUIRE_PTR(fn, dx);
    const LayerLayout Lf = layer_layout(T, H, E, K, F, 0, capacity, MOE_BF16);
    const LayerBackwardLayout L = layer_backward_layout(T, H, E, K, F, capacity);
    if (workspace == nullptr || workspace_bytes < L.total)
        return fail(MOE_ERR_WORKSPACE, "%s: workspace of %zu bytes needed, %zu given", fn, L.total,
                    workspace ? workspace_bytes : (size_t)0);
    REQUIRE_PTR(fn, workspace);
    const uint8_t* fw = static_cast<const uint8_t*>(forward_workspace);
    uint8_t* ws = static_cast<uint8_t*>(workspace);
    const float* logits = reinterpret_cast<const float*>(fw + Lf.logits);
    const int32_t* idx = reinterpret_cast<const int32_t*>(fw + Lf.idx);
    const float* gate = reinterpret_cast<const float*>(fw + Lf.gate);
    const int32_t* offsets = reinterpret_cast<const int32_t*>(fw + Lf.offsets);
    const int32_t* roa = reinterpret_cast<const int32_t*>(fw + Lf.roa);
    float* dgate = reinterpret_cast<float*>(ws + L.dgate);
    // the forward workflow in reverse: combine, experts, router, dispatch
    moe_status_t st = moe_unpermute_combine_backward(dy, fw + Lf.y_perm, roa, gate, T, H, K, L.r_max, MOE_BF16,
                                                     ws + L.dy_perm, dgate, stream);
    if (st) return st;
    st = moe_grouped_gemm_swiglu_backward(fw + Lf.x_perm, fw + Lf.h, gu, ws + L.dy_perm, offsets, L.r_max, H, F, E,
                                          w_gate, w_up, wgu_t, wd_t, ws + L.dx_perm, dw_gate, dw_up, dw_down,
                                          ws + L.expert_ws, L.expert_bytes, stream);
    if (st) return st;
    st = moe_router_backward(x, w_router, logits, idx, dgate, T, H, E, K, renormalize, MOE_BF16,
                             reinterpret_cast<float*>(ws + L.dlogits), ws + L.dx_router, dw_router, dbias,
                             ws + L.router_ws, L.router_bytes, stream);
    if (st) return st;
    return moe_permute_backward(ws + L.dx_perm, roa, ws + L.dx_router, T, H, K, L.r_max, MOE_BF16, dx, stream);
}

float moe_fp8_delayed_scale(const float* amax_history, int len, int margin) {
    float m = 0.f;
    for (int i = 0; amax_history && i < len; ++i)
        if (std::isfinite(amax_history[i]) && amax_history[i] > m) m = amax_history[i];
    if (!(m > 0.f)) return 1.f;
    return (float)(448.0 / ((double)m * std::ldexp(1.0, margin)));
}

moe_status_t moe_fp8_quantize(const void* src, moe_dtype_t dt, size_t n, float scale, void* dst,
                              float* amax, moe_stream_t stream) {
    static const char* fn = "moe_fp8_quantize";
    if (dt != MOE_F32 && dt != MOE_BF16) return fail(MOE_ERR_INVALID_ARG, "%s: unknown dtype %d", fn, (int)dt);
    if (!std::isfinite(scale) || !(scale > 0.f)) return fail(MOE_ERR_INVALID_ARG, "%s: scale must be positive and finite", fn);
    if (n == 0) return MOE_OK;
    REQUIRE_PTR(fn, src);
    REQUIRE_PTR(fn, dst);
    if (amax && (reinterpret_cast<uintptr_t>(amax) & 3u)) return fail(MOE_ERR_INVALID_ARG, "%s: amax is not 4-byte aligned", fn);
    launch_fp8_quantize(src, dt, n, scale, dst, amax, static_cast<hipStream_t>(stream));
    return check_launch(fn);
}

moe_status_t moe_permute_fp8(const void* x_bf16, const int32_t* topk_idx, int T, int H, int E, int K,
                             int capacity, float scale, void* x_perm_fp8, int32_t* expert_counts,
                             int32_t* expert_offsets, int32_t* row_of_assign, int32_t* assign_of_row,
                             float* amax, void* workspace, size_t workspace_bytes,
                             moe_stream_t stream) {
    static const char* fn = "moe_permute_fp8";
    if (moe_status_t st = check_dims(fn, T, H, E, K, MOE_BF16)) return st;
    if (!std::isfinite(scale) || !(scale > 0.f)) return fail(MOE_ERR_INVALID_ARG, "%s: scale must be positive and finite", fn);
    REQUIRE_PTR(fn, expert_counts);
    REQUIRE_PTR(fn, expert_offsets);
    if (T == 0) {
        launch_fill_i32(expert_counts, E, 0, 0, static_cast<hipStream_t>(stream));
        launch_fill_i32(expert_offsets, E + 1, 0, 0, static_cast<hipStream_t>(stream));
        return check_launch(fn);
    }
    REQUIRE_PTR(fn, x_bf16);
    REQUIRE_PTR(fn, x_perm_fp8);
    REQUIRE_PTR(fn, topk_idx);
    REQUIRE_PTR(fn, row_of_assign);
    REQUIRE_PTR(fn, assign_of_row);
    if (amax && (reinterpret_cast<uintptr_t>(amax) & 3u)) return fail(MOE_ERR_INVALID_ARG, "%s: amax is not 4-byte aligned", fn);
    const size_t need = permute_workspace_bytes(T, K, E);
    if (workspace == nullptr || workspace_bytes < need)
        return fail(MOE_ERR_WORKSPACE, "%s: workspace of %zu bytes needed, %zu given", fn, need,
                    workspace ? workspace_bytes : (size_t)0);
    REQUIRE_PTR(fn, workspace);
    const int r_max = moe_max_rows(T, K, E, capacity);
    launch_permute_fp8(x_bf16, topk_idx, T, H, E, K, capacity, r_max, scale, x_perm_fp8, expert_counts,
                       expert_offsets, row_of_assign, assign_of_row, amax, workspace,
                       static_cast<hipStream_t>(stream));
    return check_launch(fn);
}

static moe_status_t expert_ffn_fp8(const char* fn, int phase, const void* x_perm, const int32_t* expert_offsets,
                                   int R_max, int H, int F, int E, const void* w_gate, const void* w_up,
                                   const void* w_down, float dq_gate, float dq_up, float scale_h, float dq_down,
                                   void* h, float* amax_h, void* y_perm, moe_stream_t stream) {
    if (R_max < 0 || H <= 0 || F <= 0 || E <= 0)
        return fail(MOE_ERR_INVALID_ARG, "%s: need R_max >= 0 and H, F, E > 0", fn);
    if (E > kMaxExperts) return fail(MOE_ERR_UNSUPPORTED, "%s: E=%d exceeds the limit %d", fn, E, kMaxExperts);
    if (!fp8_ffn_supported(H, F))
        return fail(MOE_ERR_UNSUPPORTED, "%s: H=%d and F=%d must be multiples of 128 and at least 256", fn, H, F);
    if ((phase & 1) && !(std::isfinite(dq_gate) && std::isfinite(dq_up) && std::isfinite(scale_h) && scale_h > 0.f))
        return fail(MOE_ERR_INVALID_ARG, "%s: dq_gate, dq_up and scale_h must be finite, scale_h positive", fn);
    if ((phase & 2) && !std::isfinite(dq_down)) return fail(MOE_ERR_INVALID_ARG, "%s: dq_down must be finite", fn);
    if (R_max == 0) return MOE_OK;
    REQUIRE_PTR(fn, expert_offsets);
    REQUIRE_PTR(fn, h);
    if (phase & 1) {
        REQUIRE_PTR(fn, x_perm);
        REQUIRE_PTR(fn, w_gate);
        REQUIRE_PTR(fn, w_up);
        if (amax_h && (reinterpret_cast<uintptr_t>(amax_h) & 3u))
            return fail(MOE_ERR_INVALID_ARG, "%s: amax_h is not 4-byte aligned", fn);
    }
    if (phase & 2) {
        REQUIRE_PTR(fn, w_down);
        REQUIRE_PTR(fn, y_perm);
    }
    launch_expert_ffn_fp8(x_perm, expert_offsets, R_max, H, F, E, w_gate, w_up, w_down, dq_gate, dq_up, scale_h,
                          dq_down, h, amax_h, y_perm, phase, static_cast<hipStream_t>(stream));
    return check_launch(fn);
}

moe_status_t moe_grouped_gemm_swiglu_fp8(const void* x_perm_fp8, const int32_t* expert_offsets,
                                         int R_max, int H, int F, int E, const void* w_gate_fp8,
                                         const void* w_up_fp8, const void* w_down_fp8, float dq_gate,
                                         float dq_up, float scale_h, float dq_down, void* h_fp8,
                                         float* amax_h, void* y_perm_bf16, moe_stream_t stream) {
    return expert_ffn_fp8("moe_grouped_gemm_swiglu_fp8", 3, x_perm_fp8, expert_offsets, R_max, H, F, E, w_gate_fp8,
                          w_up_fp8, w_down_fp8, dq_gate, dq_up, scale_h, dq_down, h_fp8, amax_h, y_perm_bf16, stream);
}

moe_status_t moe_expert_gate_up_fp8(const void* x_perm_fp8, const int32_t* expert_offsets, int R_max,
                                    int H, int F, int E, const void* w_gate_fp8, const void* w_up_fp8,
                                    float dq_gate, float dq_up, float scale_h, void* h_fp8,
                                    float* amax_h, moe_stream_t stream) {
    return expert_ffn_fp8("moe_expert_gate_up_fp8", 1, x_perm_fp8, expert_offsets, R_max, H, F, E, w_gate_fp8,
                          w_up_fp8, nullptr, dq_gate, dq_up, scale_h, 0.f, h_fp8, amax_h, nullptr, stream);
}

moe_status_t moe_expert_down_fp8(const void* h_fp8, const int32_t* expert_offsets, int R_max, int H,
                                 int F, int E, const void* w_down_fp8, float dq_down,
                                 void* y_perm_bf16, moe_stream_t stream) {
    return expert_ffn_fp8("moe_expert_down_fp8", 2, nullptr, expert_offsets, R_max, H, F, E, nullptr, nullptr,
                          w_down_fp8, 0.f, 0.f, 1.f, dq_down, const_cast<void*>(h_fp8), nullptr, y_perm_bf16, stream);
}

moe_status_t moe_probe_mfma_bf16(const void* image, int iters, int workgroups, float* sink,
                                 uint64_t* ticks, moe_stream_t stream) {
    static const char* fn = "moe_probe_mfma_bf16";
    if (iters < 1 || workgroups < 1 || workgroups > 65536)
        return fail(MOE_ERR_INVALID_ARG, "%s: need iters >= 1 and 1 <= workgroups <= 65536", fn);
    REQUIRE_PTR(fn, image);
    REQUIRE_PTR(fn, sink);
    launch_probe_mfma_bf16(image, iters, workgroups, sink, reinterpret_cast<unsigned long long*>(ticks),
                           static_cast<hipStream_t>(stream));
    return check_launch(fn);
}

moe_status_t moe_probe_mfma_fp8(const void* image, int iters, int workgroups, float* sink,
                                uint64_t* ticks, moe_stream_t stream) {
    static const char* fn = "moe_probe_mfma_fp8";
    if (iters < 1 || workgroups < 1 || workgroups > 65536)
        return fail(MOE_ERR_INVALID_ARG, "%s: need iters >= 1 and 1 <= workgroups <= 65536", fn);
    REQUIRE_PTR(fn, image);
    REQUIRE_PTR(fn, sink);
    launch_probe_mfma_fp8(image, iters, workgroups, sink, reinterpret_cast<unsigned long long*>(ticks),
                          static_cast<hipStream_t>(stream));
    return check_launch(fn);
}

moe_status_t moe_gemm_clock_sample(uint64_t* ticks) {
    if (reinterpret_cast<uintptr_t>(ticks) & 7u)
        return fail(MOE_ERR_INVALID_ARG, "moe_gemm_clock_sample: ticks is not 8-byte aligned");
    moe::set_persist_clock_sample(reinterpret_cast<unsigned long long*>(ticks));
    return MOE_OK;
}

moe_status_t moe_set_option(const char* name, int value) {
    if (name && strcmp(name, "gemm_idle_skip") == 0) {
        moe::set_persist_idle_skip(value < 0 ? -1 : (value != 0));
        return MOE_OK;
    }
    if (name && strcmp(name, "fp8_deep_weights") == 0) {
        moe::set_fp8_deep_b(value);
        return MOE_OK;
    }
    if (name && strcmp(name, "permute_fused") == 0) {
        moe::set_permute_fused(value);
        return MOE_OK;
    }
    if (name && strcmp(name, "wgrad_rowmajor") == 0) {
        g_wgrad_rowmajor = value != 0;
        return MOE_OK;
    }
    if (name && strcmp(name, "router_tile") == 0) {
        if (value != 0 && value != 1 && value != 2 && value != 4)
            return fail(MOE_ERR_INVALID_ARG, "moe_set_option: router_tile must be 0, 1, 2 or 4");
        moe::set_router_tile(value);
        return MOE_OK;
    }
    if (name && strcmp(name, "gemm_workgroups") == 0) {
        if (value < 0) return fail(MOE_ERR_INVALID_ARG, "moe_set_option: gemm_workgroups must be >= 0");
        moe::set_persist_workgroups(value);
        return MOE_OK;
    }
    if (name && strcmp(name, "gemm_variant") == 0) {
        g_gemm_variant = value;
        return MOE_OK;
    }
    return fail(MOE_ERR_INVALID_ARG, "moe_set_option: unknown option '%s'", name ? name : "(null)");
}

}  // extern "C"
