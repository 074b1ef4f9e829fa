/*
 * moe_oracle.c -- slow, plain CPU oracle for the MoE-layer forward hot path.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may link, load or
 * call this file; it exists so that the HIP kernels can be checked against an
 * implementation that can be compared with the paper by eye.  It shares no
 * code, tables or helpers with the HIP path.
 *
 * What it follows (arXiv 2504.14960):
 *   Eq. 1  (Section 3.1.1)  y = sum_e g_e(x) * f_e(x)
 *   Eq. 2  (Section 3.1.1)  Top-K gating: g_e = s_e for the K largest s, else 0
 *   Eq. 3  (Section 3.1.1)  s = G(W_g x), G = softmax (Section 3.3, router paragraph)
 *   Eq. 4  (Section 3.1.1)  capacity per expert = CF * L / E, over-capacity tokens dropped
 *   Section 3.1.2 "Token Dispatching" / "Token Restore": rows of one expert
 *   contiguous in memory; inverse permutation back to token order.
 *   Section 3.3: sub-sequence dropping -- the drop decision uses only the
 *   tokens of this call.
 *
 * The fast path (permute + grouped GEMM + unpermute) reaches Eq. 1 exactly up
 * to rounding order, so every function below is the plain definition written
 * out: no blocking, no fusion, no reordering.  All floating-point work is done
 * in double; inputs are fp32 or bf16 bit patterns and are widened exactly.
 * The one place where floating point decides an integer -- which K experts a
 * token selects -- is taken on fp32 logits, the precision the kernels hold
 * logits in, so both sides decide on the same numbers.
 *
 * Readings of points the paper leaves open (each is also listed in the
 * design notes of this repository):
 *   - Top-K runs over experts, per token (Eq. 2's index is garbled in print).
 *   - Selection order: larger logit first, equal logits -> lower expert index.
 *     -0.0 and +0.0 are equal.  NaN ranks as minus infinity.
 *   - Gates are softmax probabilities over all E experts (Eq. 2 uses raw s);
 *     `renormalize` optionally divides the K selected gates by their sum.
 *   - Eq. 4's L is the number of token-expert assignments T*K (the "average
 *     expected load" of an expert is T*K/E rows); the result is rounded up.
 *   - Over capacity, an expert keeps its first C assignments in token order.
 *   - Dropping does not change the remaining gates.
 *   - Rows inside an expert's block are in ascending token order, no padding.
 *   - f_e is a bias-free SwiGLU FFN: W_down (silu(W_gate x) * (W_up x)).
 *   - An expert index outside [0, E) is treated as a dropped assignment.
 *
 * Pins (tests/test_oracle_*.py): closed forms (equal logits -> 1/E, K = E ->
 * gates sum to 1, capacity values), E = 1 reduces to a dense MLP computed with
 * a library matmul, stable argsort cross-check of the permutation, identity
 * experts give permute/unpermute round trip, brute-force dense Eq. 1 below,
 * batch-split invariance, dropped-tokens-are-zero; the two backward functions by
 * the adjoint identity <F(a), b> = <a, F'(b)> on random tensors, finite
 * differences in the gates, and a library scatter-add; the chunk gather by
 * numpy split/concatenate, its inverse, and by a simulated expert-parallel
 * group whose output must equal the one-GPU layer's.  No function here is
 * "parity unpinned"; the paper prints no worked numeric example of the layer.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };

/* exact widening load of element i */
static inline double ld(const void* p, size_t i, int dt) {
    if (dt == ORACLE_F32) return (double)((const float*)p)[i];
    uint32_t u = ((uint32_t)((const uint16_t*)p)[i]) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static inline size_t elem_size(int dt) { return dt == ORACLE_F32 ? 4u : 2u; }

int oracle_num_threads(void) {
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---- Eq. 3, the linear part: logits[t,e] = sum_h x[t,h] W_g[e,h] (+ bias[e]) ---- */
void oracle_router_logits(const void* x, const void* w_router, const float* bias,
                          int T, int H, int E, int dt, double* logits) {
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t)
        for (int e = 0; e < E; ++e) {
            double acc = 0.0;
            for (int h = 0; h < H; ++h)
                acc += ld(x, (size_t)t * H + h, dt) * ld(w_router, (size_t)e * H + h, dt);
            if (bias) acc += (double)bias[e];
            logits[(size_t)t * E + e] = acc;
        }
}

/* selection order of Eq. 2's TopK: value descending, then expert index ascending */
static inline float sel_key(float v) { return isnan(v) ? -INFINITY : v; }
static inline int ranks_before(float a, int ia, float b, int ib) {
    a = sel_key(a);
    b = sel_key(b);
    if (a > b) return 1;
    if (a < b) return 0;
    return ia < ib; /* equal (including -0 == +0): lower index first */
}

/* ---- Eq. 2 + Eq. 3's G: softmax over all E, then the K best experts ----
 * logits are fp32 (the decision precision).  idx[t,k] in selection order,
 * gate[t,k] = softmax(logits[t,:])[idx[t,k]], optionally renormalised over the
 * K selected (sum taken in slot order).  probs (may be NULL) receives the full
 * softmax. */
void oracle_topk_gates(const float* logits, int T, int E, int K, int renormalize,
                       int32_t* idx, double* gate, double* probs) {
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        const float* l = logits + (size_t)t * E;
        double* p = (double*)malloc(sizeof(double) * (size_t)E);
        char* taken = (char*)calloc((size_t)E, 1);
        double m = -INFINITY;
        for (int e = 0; e < E; ++e)
            if ((double)l[e] > m) m = (double)l[e];
        double z = 0.0;
        for (int e = 0; e < E; ++e) {
            p[e] = exp((double)l[e] - m);
            z += p[e];
        }
        for (int e = 0; e < E; ++e) {
            p[e] /= z;
            if (probs) probs[(size_t)t * E + e] = p[e];
        }
        for (int k = 0; k < K; ++k) {
            int best = -1;
            for (int e = 0; e < E; ++e) {
                if (taken[e]) continue;
                if (best < 0 || ranks_before(l[e], e, l[best], best)) best = e;
            }
            taken[best] = 1;
            idx[(size_t)t * K + k] = best;
            gate[(size_t)t * K + k] = p[best];
        }
        if (renormalize) {
            double s = 0.0;
            for (int k = 0; k < K; ++k) s += gate[(size_t)t * K + k];
            for (int k = 0; k < K; ++k) gate[(size_t)t * K + k] /= s;
        }
        free(p);
        free(taken);
    }
}

/* ---- Eq. 4 with L = T*K, rounded up ---- */
int oracle_capacity(double capacity_factor, int T, int K, int E) {
    return (int)ceil(capacity_factor * (double)T * (double)K / (double)E);
}

/* ---- Section 3.1.2 "Token Dispatching", the local part ----
 * Walk the assignments a = t*K + k in ascending order; the j-th assignment
 * that names expert e gets rank j inside e and is kept iff dropless
 * (capacity <= 0) or j < capacity.  Kept rows of expert e occupy
 * [offsets[e], offsets[e+1]) in rank order.  x_perm rows are byte copies of x
 * rows.  r_max = number of rows x_perm / assign_of_row have room for; rows
 * beyond the kept total get assign_of_row = -1 and are left untouched in
 * x_perm.  Returns the kept total R. */
int oracle_permute(const void* x, const int32_t* idx, int T, int H, int E, int K,
                   int capacity, int dt, int r_max, void* x_perm, int32_t* counts,
                   int32_t* offsets, int32_t* row_of_assign, int32_t* assign_of_row) {
    const size_t row_bytes = (size_t)H * elem_size(dt);
    int64_t* n = (int64_t*)calloc((size_t)E, sizeof(int64_t));
    const size_t A = (size_t)T * K;
    /* pass 1: how many assignments name each expert */
    for (size_t a = 0; a < A; ++a) {
        int e = idx[a];
        if (e >= 0 && e < E) n[e]++;
    }
    offsets[0] = 0;
    for (int e = 0; e < E; ++e) {
        int64_t c = (capacity > 0 && n[e] > capacity) ? capacity : n[e];
        counts[e] = (int32_t)c;
        offsets[e + 1] = offsets[e] + (int32_t)c;
    }
    const int R = offsets[E];
    for (int r = 0; r < r_max; ++r) assign_of_row[r] = -1;
    /* pass 2: ranks in assignment order */
    memset(n, 0, sizeof(int64_t) * (size_t)E);
    for (size_t a = 0; a < A; ++a) {
        int e = idx[a];
        if (e < 0 || e >= E) {
            row_of_assign[a] = -1;
            continue;
        }
        int64_t rank = n[e]++;
        if (capacity > 0 && rank >= capacity) {
            row_of_assign[a] = -1;
            continue;
        }
        int row = offsets[e] + (int)rank;
        row_of_assign[a] = row;
        assign_of_row[row] = (int32_t)a;
        if (x && x_perm)
            memcpy((char*)x_perm + (size_t)row * row_bytes,
                   (const char*)x + (a / (size_t)K) * row_bytes, row_bytes);
    }
    free(n);
    return R;
}

/* ---- variants of the local dispatch: which assignments an over-subscribed
 * expert drops, and whether every expert's block is padded to the capacity.
 * (Eq. 4 fixes the capacity; the paper's benchmark drops by position.  These two
 * variants are the other drop rule and the fixed-shape layout of capacity-based
 * MoE training.)
 *
 * by_score = 0: an expert keeps its first `capacity` assignments in assignment
 *   order (as oracle_permute).
 * by_score = 1: it keeps the `capacity` assignments with the largest score
 *   (scores [T,K] float, compared as floats; equal scores: the lower assignment
 *   index is better).
 * Either way the kept rows of an expert are laid out in ascending assignment
 * index.
 * pad = 0: experts packed back to back (offsets = running sum of the counts).
 * pad = 1: expert e owns rows [e*capacity, (e+1)*capacity): offsets[e] =
 *   e*capacity, counts[e] = rows really kept, the rest of the block is zero rows
 *   with assign_of_row = -1.  Needs capacity > 0 and r_max >= E*capacity.
 * Returns offsets[E]. */
typedef struct { float score; int32_t a; } scored_t;

static int better_first(const void* pa, const void* pb) {
    const scored_t* a = (const scored_t*)pa;
    const scored_t* b = (const scored_t*)pb;
    if (a->score > b->score) return -1;
    if (a->score < b->score) return 1;
    return (a->a > b->a) - (a->a < b->a);
}

int oracle_permute_variant(const void* x, const int32_t* idx, const float* scores, int T, int H,
                           int E, int K, int capacity, int by_score, int pad, int dt, int r_max,
                           void* x_perm, int32_t* counts, int32_t* offsets,
                           int32_t* row_of_assign, int32_t* assign_of_row) {
    const size_t row_bytes = (size_t)H * elem_size(dt);
    const size_t A = (size_t)T * K;
    if (pad && capacity <= 0) return -1;
    char* keep = (char*)calloc(A + 1, 1);
    scored_t* list = (scored_t*)malloc(sizeof(scored_t) * (A + 1));
    for (size_t a = 0; a < A; ++a) row_of_assign[a] = -1;
    for (int r = 0; r < r_max; ++r) assign_of_row[r] = -1;
    if (x_perm && pad) memset(x_perm, 0, (size_t)r_max * row_bytes);
    /* the kept set, expert by expert */
    for (int e = 0; e < E; ++e) {
        size_t n = 0;
        for (size_t a = 0; a < A; ++a)
            if (idx[a] == e) {
                list[n].score = (by_score && scores) ? scores[a] : 0.0f;
                list[n].a = (int32_t)a;
                ++n;
            }
        /* by position: all scores equal, so the order below is the assignment order */
        qsort(list, n, sizeof(scored_t), better_first);
        size_t kept = (capacity > 0 && n > (size_t)capacity) ? (size_t)capacity : n;
        for (size_t i = 0; i < kept; ++i) keep[list[i].a] = 1;
        counts[e] = (int32_t)kept;
    }
    offsets[0] = 0;
    for (int e = 0; e < E; ++e) offsets[e + 1] = pad ? (e + 1) * capacity : offsets[e] + counts[e];
    /* rows: kept assignments of an expert in ascending assignment index */
    int32_t* next = (int32_t*)calloc((size_t)E, sizeof(int32_t));
    for (size_t a = 0; a < A; ++a) {
        if (!keep[a]) continue;
        const int e = idx[a];
        const int row = (pad ? e * capacity : offsets[e]) + next[e]++;
        if (row >= r_max) continue; /* inconsistent r_max: never an address */
        row_of_assign[a] = row;
        assign_of_row[row] = (int32_t)a;
        if (x && x_perm)
            memcpy((char*)x_perm + (size_t)row * row_bytes,
                   (const char*)x + (a / (size_t)K) * row_bytes, row_bytes);
    }
    free(next);
    free(list);
    free(keep);
    return offsets[E];
}

/* ---- f_e for one expert over n_rows rows (Section 3.1.1's f_e; SwiGLU) ----
 * x_rows [n_rows,H]; w_gate, w_up [F,H]; w_down [H,F] (all of ONE expert).
 * h [n_rows,F] (may be NULL) and y [n_rows,H] are double. */
void oracle_expert_ffn_rows(const void* x_rows, int n_rows, int H, int F,
                            const void* w_gate, const void* w_up, const void* w_down,
                            int dt, double* h_out, double* y) {
    if (n_rows <= 0) return;
    double* h = h_out ? h_out : (double*)malloc(sizeof(double) * (size_t)n_rows * F);
#pragma omp parallel for collapse(2) schedule(static)
    for (int r = 0; r < n_rows; ++r)
        for (int f = 0; f < F; ++f) {
            double g = 0.0, u = 0.0;
            for (int k = 0; k < H; ++k) {
                double xv = ld(x_rows, (size_t)r * H + k, dt);
                g += xv * ld(w_gate, (size_t)f * H + k, dt);
                u += xv * ld(w_up, (size_t)f * H + k, dt);
            }
            double silu = g / (1.0 + exp(-g));
            h[(size_t)r * F + f] = silu * u;
        }
#pragma omp parallel for collapse(2) schedule(static)
    for (int r = 0; r < n_rows; ++r)
        for (int n = 0; n < H; ++n) {
            double acc = 0.0;
            for (int f = 0; f < F; ++f)
                acc += h[(size_t)r * F + f] * ld(w_down, (size_t)n * F + f, dt);
            y[(size_t)r * H + n] = acc;
        }
    if (!h_out) free(h);
}

/* ---- "Expert Computation": every expert over its contiguous rows ---- */
void oracle_experts(const void* x_perm, const int32_t* offsets, int E, int H, int F,
                    const void* w_gate, const void* w_up, const void* w_down, int dt,
                    double* h_out, double* y_perm) {
    const size_t es = elem_size(dt);
    for (int e = 0; e < E; ++e) {
        int lo = offsets[e], hi = offsets[e + 1];
        if (hi <= lo) continue;
        oracle_expert_ffn_rows((const char*)x_perm + (size_t)lo * H * es, hi - lo, H, F,
                               (const char*)w_gate + (size_t)e * F * H * es,
                               (const char*)w_up + (size_t)e * F * H * es,
                               (const char*)w_down + (size_t)e * H * F * es, dt,
                               h_out ? h_out + (size_t)lo * F : NULL,
                               y_perm + (size_t)lo * H);
    }
}

/* ---- backward of "Expert Computation" (Section 3.3: the backward workflow mirrors
 * the forward one; f_e of Eq. 1 differentiated by the chain rule) ----
 * For every expert e over its rows r, with g = x W_gate^T, u = x W_up^T,
 * s = 1 / (1 + exp(-g)), h = g s u, y = h W_down^T and dy given:
 *   dW_down[e][n][f] = sum_r dy[r,n] h[r,f]
 *   dh[r,f]          = sum_n dy[r,n] W_down[e][n][f]
 *   du[r,f]          = dh[r,f] g s                      (d h / d u = silu(g))
 *   dg[r,f]          = dh[r,f] u s (1 + g (1 - s))      (d silu / d g = s (1 + g (1 - s)))
 *   dW_gate[e][f][k] = sum_r dg[r,f] x[r,k],  dW_up[e][f][k] = sum_r du[r,f] x[r,k]
 *   dx[r,k]          = sum_f dg[r,f] W_gate[e][f][k] + du[r,f] W_up[e][f][k]
 * dy [R,H] double; x_perm and the weights in dt.  Outputs (double): dx [R,H],
 * dw_gate, dw_up [E,F,H], dw_down [E,H,F] (experts without rows get zeros). */
void oracle_experts_backward(const void* x_perm, const int32_t* offsets, int E, int H, int F,
                             const void* w_gate, const void* w_up, const void* w_down, int dt,
                             const double* dy, double* dx, double* dw_gate, double* dw_up,
                             double* dw_down) {
    memset(dw_gate, 0, sizeof(double) * (size_t)E * F * H);
    memset(dw_up, 0, sizeof(double) * (size_t)E * F * H);
    memset(dw_down, 0, sizeof(double) * (size_t)E * H * F);
    for (int e = 0; e < E; ++e) {
        const int lo = offsets[e], hi = offsets[e + 1], n_rows = hi - lo;
        if (n_rows <= 0) continue;
        const size_t wo = (size_t)e * F * H;
        double* g = (double*)malloc(sizeof(double) * (size_t)n_rows * F);
        double* u = (double*)malloc(sizeof(double) * (size_t)n_rows * F);
        double* dg = (double*)malloc(sizeof(double) * (size_t)n_rows * F);
        double* du = (double*)malloc(sizeof(double) * (size_t)n_rows * F);
#pragma omp parallel for collapse(2) schedule(static)
        for (int r = 0; r < n_rows; ++r)
            for (int f = 0; f < F; ++f) {
                double gs = 0.0, us = 0.0;
                for (int k = 0; k < H; ++k) {
                    double xv = ld(x_perm, (size_t)(lo + r) * H + k, dt);
                    gs += xv * ld(w_gate, wo + (size_t)f * H + k, dt);
                    us += xv * ld(w_up, wo + (size_t)f * H + k, dt);
                }
                g[(size_t)r * F + f] = gs;
                u[(size_t)r * F + f] = us;
            }
#pragma omp parallel for collapse(2) schedule(static)
        for (int r = 0; r < n_rows; ++r)
            for (int f = 0; f < F; ++f) {
                double dh = 0.0;
                for (int n = 0; n < H; ++n)
                    dh += dy[(size_t)(lo + r) * H + n] * ld(w_down, wo + (size_t)n * F + f, dt);
                double gv = g[(size_t)r * F + f], uv = u[(size_t)r * F + f];
                double sg = 1.0 / (1.0 + exp(-gv));
                du[(size_t)r * F + f] = dh * gv * sg;
                dg[(size_t)r * F + f] = dh * uv * sg * (1.0 + gv * (1.0 - sg));
            }
#pragma omp parallel for collapse(2) schedule(static)
        for (int n = 0; n < H; ++n)
            for (int f = 0; f < F; ++f) {
                double acc = 0.0;
                for (int r = 0; r < n_rows; ++r) {
                    double gv = g[(size_t)r * F + f], uv = u[(size_t)r * F + f];
                    acc += dy[(size_t)(lo + r) * H + n] * (gv / (1.0 + exp(-gv)) * uv);
                }
                dw_down[wo + (size_t)n * F + f] = acc;
            }
#pragma omp parallel for collapse(2) schedule(static)
        for (int f = 0; f < F; ++f)
            for (int k = 0; k < H; ++k) {
                double ag = 0.0, au = 0.0;
                for (int r = 0; r < n_rows; ++r) {
                    double xv = ld(x_perm, (size_t)(lo + r) * H + k, dt);
                    ag += dg[(size_t)r * F + f] * xv;
                    au += du[(size_t)r * F + f] * xv;
                }
                dw_gate[wo + (size_t)f * H + k] = ag;
                dw_up[wo + (size_t)f * H + k] = au;
            }
#pragma omp parallel for collapse(2) schedule(static)
        for (int r = 0; r < n_rows; ++r)
            for (int k = 0; k < H; ++k) {
                double acc = 0.0;
                for (int f = 0; f < F; ++f)
                    acc += dg[(size_t)r * F + f] * ld(w_gate, wo + (size_t)f * H + k, dt) +
                           du[(size_t)r * F + f] * ld(w_up, wo + (size_t)f * H + k, dt);
                dx[(size_t)(lo + r) * H + k] = acc;
            }
        free(g);
        free(u);
        free(dg);
        free(du);
    }
}

/* ---- "Token Restore" + Eq. 1's weighted sum ----
 * y[t,:] = sum over k ascending of gate[t,k] * y_perm[row_of_assign[t,k],:]
 * (dropped assignments contribute nothing) (+ addend[t,:]). */
void oracle_combine(const double* y_perm, const int32_t* row_of_assign, const double* gate,
                    const double* addend, int T, int H, int K, double* y) {
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t)
        for (int n = 0; n < H; ++n) {
            double acc = 0.0;
            for (int k = 0; k < K; ++k) {
                int row = row_of_assign[(size_t)t * K + k];
                if (row < 0) continue;
                acc += gate[(size_t)t * K + k] * y_perm[(size_t)row * H + n];
            }
            if (addend) acc += addend[(size_t)t * H + n];
            y[(size_t)t * H + n] = acc;
        }
}

/* ---- backward of the router (Eq. 2 + Eq. 3 by the chain rule; Section 3.3: the
 * backward workflow mirrors the forward one) ----
 * Forward: l = x W_g^T (+ bias), p = softmax(l), gate_k = p[idx_k], optionally
 * divided by S = sum_k p[idx_k].  The selection idx is piecewise constant, so
 * its derivative is zero; given dgate [T,K]:
 *   without renormalisation  q_k = dgate_k
 *   with renormalisation     q_k = (dgate_k - sum_j dgate_j gate_j) / S
 *   dl_e = [e = idx_k] q_k p_e  -  p_e sum_k q_k p[idx_k]          (softmax Jacobian)
 *   dx[t,:] = sum_e dl[t,e] W_g[e,:]    dW_g[e,:] = sum_t dl[t,e] x[t,:]    dbias[e] = sum_t dl[t,e]
 * logits are the fp32 logits the forward kept.  An index outside [0,E) has no gradient.
 * dx, dw, dbias may be NULL. */
void oracle_router_backward(const void* x, const void* w_router, const float* logits,
                            const int32_t* idx, const double* dgate, int T, int H, int E, int K,
                            int renormalize, int dt, double* dlogits, double* dx, double* dw,
                            double* dbias) {
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        const float* l = logits + (size_t)t * E;
        double* p = (double*)malloc(sizeof(double) * (size_t)E);
        double* q = (double*)malloc(sizeof(double) * (size_t)K);
        double m = -INFINITY, z = 0.0;
        for (int e = 0; e < E; ++e)
            if ((double)l[e] > m) m = (double)l[e];
        for (int e = 0; e < E; ++e) {
            p[e] = exp((double)l[e] - m);
            z += p[e];
        }
        for (int e = 0; e < E; ++e) p[e] /= z;
        double S = 0.0, a = 0.0;
        for (int k = 0; k < K; ++k) {
            int e = idx[(size_t)t * K + k];
            if (e >= 0 && e < E) S += p[e];
        }
        for (int k = 0; k < K; ++k) {
            int e = idx[(size_t)t * K + k];
            if (e >= 0 && e < E) a += dgate[(size_t)t * K + k] * (p[e] / S);
        }
        double sum_qp = 0.0;
        for (int k = 0; k < K; ++k) {
            int e = idx[(size_t)t * K + k];
            q[k] = 0.0;
            if (e < 0 || e >= E) continue;
            q[k] = renormalize ? (dgate[(size_t)t * K + k] - a) / S : dgate[(size_t)t * K + k];
            sum_qp += q[k] * p[e];
        }
        for (int e = 0; e < E; ++e) dlogits[(size_t)t * E + e] = -p[e] * sum_qp;
        for (int k = 0; k < K; ++k) {
            int e = idx[(size_t)t * K + k];
            if (e >= 0 && e < E) dlogits[(size_t)t * E + e] += q[k] * p[e];
        }
        free(p);
        free(q);
    }
    if (dx) {
#pragma omp parallel for collapse(2) schedule(static)
        for (int t = 0; t < T; ++t)
            for (int n = 0; n < H; ++n) {
                double acc = 0.0;
                for (int e = 0; e < E; ++e) acc += dlogits[(size_t)t * E + e] * ld(w_router, (size_t)e * H + n, dt);
                dx[(size_t)t * H + n] = acc;
            }
    }
    if (dw) {
#pragma omp parallel for collapse(2) schedule(static)
        for (int e = 0; e < E; ++e)
            for (int n = 0; n < H; ++n) {
                double acc = 0.0;
                for (int t = 0; t < T; ++t) acc += dlogits[(size_t)t * E + e] * ld(x, (size_t)t * H + n, dt);
                dw[(size_t)e * H + n] = acc;
            }
    }
    if (dbias)
        for (int e = 0; e < E; ++e) {
            double acc = 0.0;
            for (int t = 0; t < T; ++t) acc += dlogits[(size_t)t * E + e];
            dbias[e] = acc;
        }
}

/* ---- backward of the dispatcher's two data movements (Section 3.3: the
 * backward workflow mirrors the forward one) ----
 *
 * "Token Restore" + weighted sum, y[t,:] = sum_k gate[t,k] * y_perm[row(t,k),:]:
 *   dy_perm[row(t,k),:] = gate[t,k] * dy[t,:]        (every kept row has one source)
 *   dgate[t,k]          = sum_n dy[t,n] * y_perm[row(t,k),n]   (0 for a dropped assignment)
 * dy_perm [R,H] is written for kept rows only (rows are hit exactly once). */
void oracle_combine_backward(const double* dy, const double* y_perm, const int32_t* row_of_assign,
                             const double* gate, int T, int H, int K, double* dy_perm, double* dgate) {
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t)
        for (int k = 0; k < K; ++k) {
            size_t a = (size_t)t * K + k;
            int row = row_of_assign[a];
            double dot = 0.0;
            if (row >= 0)
                for (int n = 0; n < H; ++n) {
                    dy_perm[(size_t)row * H + n] = gate[a] * dy[(size_t)t * H + n];
                    dot += dy[(size_t)t * H + n] * y_perm[(size_t)row * H + n];
                }
            dgate[a] = dot;
        }
}

/* "Token Dispatching", x_perm[row(t,k),:] = x[t,:] for kept assignments:
 *   dx[t,:] = sum over kept k of dx_perm[row(t,k),:]  (+ addend[t,:], the gradient that
 *   reaches x along other paths) */
void oracle_permute_backward(const double* dx_perm, const int32_t* row_of_assign, const double* addend,
                             int T, int H, int K, double* dx) {
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t)
        for (int n = 0; n < H; ++n) {
            double acc = 0.0;
            for (int k = 0; k < K; ++k) {
                int row = row_of_assign[(size_t)t * K + k];
                if (row >= 0) acc += dx_perm[(size_t)row * H + n];
            }
            if (addend) acc += addend[(size_t)t * H + n];
            dx[(size_t)t * H + n] = acc;
        }
}

/* ---- expert-parallel share of one GPU: received rows by source, needed by expert ----
 * Section 3.3, forward workflow: after the All-to-All-V over the EP group a GPU
 * holds, for every source rank in turn, that rank's rows for each of the local
 * experts; the expert computation needs all rows of one expert together, and the
 * way back needs the source order again.  The paper names no operation for this;
 * the reading here is a gather of row chunks: src is a sequence of n_src chunks,
 * chunk c having chunk_rows[c] rows (negative counts as 0); dst is the sequence
 * of chunks order[0], order[1], ... (a chunk named twice is copied twice, an index
 * outside [0, n_src) stands for an empty chunk).  A row is copied when it lies
 * below r_src in src and below r_dst in dst.  chunk_rows_out[p] = rows of dst
 * chunk p; group_offsets[g] = first dst row of chunk g*group (group > 0), with
 * one more entry for the total.  Returns the total number of dst rows. */
long long oracle_sort_chunks(const void* src, long long r_src, const int32_t* chunk_rows, int n_src,
                             const int32_t* order, int n_dst, int group, size_t row_bytes,
                             void* dst, long long r_dst, int32_t* chunk_rows_out,
                             int32_t* group_offsets) {
    long long* src_start = (long long*)malloc(sizeof(long long) * (size_t)(n_src + 1));
    src_start[0] = 0;
    for (int c = 0; c < n_src; ++c) src_start[c + 1] = src_start[c] + (chunk_rows[c] > 0 ? chunk_rows[c] : 0);
    long long d = 0;
    for (int p = 0; p < n_dst; ++p) {
        if (group_offsets && group > 0 && p % group == 0) group_offsets[p / group] = (int32_t)d;
        const int c = order[p];
        const long long n = (c >= 0 && c < n_src) ? src_start[c + 1] - src_start[c] : 0;
        if (chunk_rows_out) chunk_rows_out[p] = (int32_t)n;
        for (long long i = 0; i < n; ++i) {
            const long long from = src_start[c] + i, to = d + i;
            if (src && dst && from < r_src && to < r_dst)
                memcpy((char*)dst + (size_t)to * row_bytes, (const char*)src + (size_t)from * row_bytes, row_bytes);
        }
        d += n;
    }
    if (group_offsets && group > 0) group_offsets[(n_dst + group - 1) / group] = (int32_t)d;
    free(src_start);
    return d;
}

/* ---- the whole layer through the dispatcher's data path ----
 * shared expert (ws_* non-NULL, Fs > 0): y += f_shared(x) for every token,
 * ungated.  Optional outputs may be NULL.  Returns R. */
int oracle_layer_forward(const void* x, const void* w_router, const float* bias,
                         const void* w_gate, const void* w_up, const void* w_down,
                         const void* ws_gate, const void* ws_up, const void* ws_down,
                         int T, int H, int E, int K, int F, int Fs, int renormalize,
                         int capacity, int dt, float* logits32_out, int32_t* idx_out,
                         double* gate_out, int32_t* row_of_assign_out, double* y) {
    const size_t A = (size_t)T * K;
    double* logits = (double*)malloc(sizeof(double) * (size_t)T * E);
    float* l32 = (float*)malloc(sizeof(float) * (size_t)T * E);
    int32_t* idx = (int32_t*)malloc(sizeof(int32_t) * A);
    double* gate = (double*)malloc(sizeof(double) * A);
    oracle_router_logits(x, w_router, bias, T, H, E, dt, logits);
    for (size_t i = 0; i < (size_t)T * E; ++i) l32[i] = (float)logits[i];
    oracle_topk_gates(l32, T, E, K, renormalize, idx, gate, NULL);

    int r_max = (int)A;
    void* x_perm = malloc((size_t)r_max * H * elem_size(dt) + 1);
    int32_t* counts = (int32_t*)malloc(sizeof(int32_t) * (size_t)E);
    int32_t* offsets = (int32_t*)malloc(sizeof(int32_t) * (size_t)(E + 1));
    int32_t* roa = (int32_t*)malloc(sizeof(int32_t) * A);
    int32_t* aor = (int32_t*)malloc(sizeof(int32_t) * (size_t)r_max + 4);
    int R = oracle_permute(x, idx, T, H, E, K, capacity, dt, r_max, x_perm, counts, offsets, roa, aor);

    double* y_perm = (double*)malloc(sizeof(double) * ((size_t)R * H + 1));
    oracle_experts(x_perm, offsets, E, H, F, w_gate, w_up, w_down, dt, NULL, y_perm);

    double* shared = NULL;
    if (Fs > 0 && ws_gate && ws_up && ws_down) {
        shared = (double*)malloc(sizeof(double) * (size_t)T * H);
        oracle_expert_ffn_rows(x, T, H, Fs, ws_gate, ws_up, ws_down, dt, NULL, shared);
    }
    oracle_combine(y_perm, roa, gate, shared, T, H, K, y);

    if (logits32_out) memcpy(logits32_out, l32, sizeof(float) * (size_t)T * E);
    if (idx_out) memcpy(idx_out, idx, sizeof(int32_t) * A);
    if (gate_out) memcpy(gate_out, gate, sizeof(double) * A);
    if (row_of_assign_out) memcpy(row_of_assign_out, roa, sizeof(int32_t) * A);
    free(logits); free(l32); free(idx); free(gate); free(x_perm); free(counts);
    free(offsets); free(roa); free(aor); free(y_perm); free(shared);
    return R;
}

/* ---- Eq. 1 literally, with no permutation anywhere (tiny inputs only) ----
 * Builds the dense gate matrix g[T,E] (zero for unselected and for dropped),
 * evaluates EVERY expert on EVERY token and sums g[t,e] * f_e(x_t).  The
 * selection here is a full sort of (logit, index) pairs and the capacity rule
 * is applied per expert by walking tokens, so it shares no logic with
 * oracle_topk_gates / oracle_permute above. */
typedef struct { float v; int e; } pair_t;
static int pair_cmp(const void* a, const void* b) {
    const pair_t* p = (const pair_t*)a;
    const pair_t* q = (const pair_t*)b;
    float pv = isnan(p->v) ? -INFINITY : p->v, qv = isnan(q->v) ? -INFINITY : q->v;
    if (pv > qv) return -1;
    if (pv < qv) return 1;
    return (p->e > q->e) - (p->e < q->e);
}

void oracle_dense_bruteforce(const void* x, const void* w_router, const float* bias,
                             const void* w_gate, const void* w_up, const void* w_down,
                             int T, int H, int E, int K, int F, int renormalize,
                             int capacity, int dt, double* g_dense_out, double* y) {
    const size_t es = elem_size(dt);
    double* g = (double*)calloc((size_t)T * E, sizeof(double));
    char* sel = (char*)calloc((size_t)T * E, 1);
    pair_t* pr = (pair_t*)malloc(sizeof(pair_t) * (size_t)E);
    for (int t = 0; t < T; ++t) {
        double m = -INFINITY, z = 0.0;
        for (int e = 0; e < E; ++e) {
            double acc = 0.0;
            for (int h = 0; h < H; ++h)
                acc += ld(x, (size_t)t * H + h, dt) * ld(w_router, (size_t)e * H + h, dt);
            if (bias) acc += (double)bias[e];
            pr[e].v = (float)acc;
            pr[e].e = e;
            if ((double)pr[e].v > m) m = (double)pr[e].v;
        }
        for (int e = 0; e < E; ++e) z += exp((double)pr[e].v - m);
        qsort(pr, (size_t)E, sizeof(pair_t), pair_cmp);
        double s = 0.0;
        for (int k = 0; k < K; ++k) {
            g[(size_t)t * E + pr[k].e] = exp((double)pr[k].v - m) / z;
            sel[(size_t)t * E + pr[k].e] = 1;
            s += g[(size_t)t * E + pr[k].e];
        }
        if (renormalize)
            for (int k = 0; k < K; ++k) g[(size_t)t * E + pr[k].e] /= s;
    }
    if (capacity > 0)
        for (int e = 0; e < E; ++e) {
            int seen = 0;
            for (int t = 0; t < T; ++t)
                if (sel[(size_t)t * E + e]) {
                    if (seen >= capacity) g[(size_t)t * E + e] = 0.0;
                    ++seen;
                }
        }
    double* fe = (double*)malloc(sizeof(double) * (size_t)H);
    for (int t = 0; t < T; ++t) {
        for (int n = 0; n < H; ++n) y[(size_t)t * H + n] = 0.0;
        for (int e = 0; e < E; ++e) {
            oracle_expert_ffn_rows((const char*)x + (size_t)t * H * es, 1, H, F,
                                   (const char*)w_gate + (size_t)e * F * H * es,
                                   (const char*)w_up + (size_t)e * F * H * es,
                                   (const char*)w_down + (size_t)e * H * F * es, dt, NULL, fe);
            for (int n = 0; n < H; ++n) y[(size_t)t * H + n] += g[(size_t)t * E + e] * fe[n];
        }
    }
    if (g_dense_out) memcpy(g_dense_out, g, sizeof(double) * (size_t)T * E);
    free(fe); free(pr); free(g); free(sel);
}
