/*
 * moe_oracle_fp8.c -- slow, plain CPU oracle for the FP8 variant of the expert
 * FFN (Section 4.5 "FP8 Training Performance": FP8 with delayed scaling).
 *
 * TEST INFRASTRUCTURE ONLY, like moe_oracle.c: nothing in the product path may
 * link, load or call this file, and it shares no code with the HIP path.
 *
 * The paper names the recipe (FP8, delayed scaling) and gives no formulas, so
 * everything below is a reading, listed in the design notes as well:
 *   - FP8 means the OCP 8-bit format E4M3 (1 sign, 4 exponent bits with bias 7,
 *     3 mantissa bits, no infinities, one NaN code per sign, largest finite
 *     value 448), the forward-pass format of the cited FP8 recipe.
 *   - Scaling is per tensor: q = round_to_e4m3(x * scale), x ~ q / scale.
 *     Rounding is to nearest, ties to even; magnitudes above 448 (infinities
 *     included) saturate to 448; NaN stays NaN.
 *   - "Delayed": the scale used in this step comes from the largest |x| seen in
 *     earlier steps (a history of amax values), scale = 448 / (amax * 2^margin);
 *     this step's amax is only recorded.  The scale of the intermediate h is
 *     therefore known before h is computed.
 *   - The product x * scale is rounded to fp32 before it is rounded to E4M3,
 *     because that is the precision the kernels hold it in (where floating
 *     point decides an integer code, both sides decide in the same precision).
 *   - The expert FFN itself is the one of moe_oracle.c: products of the
 *     dequantised operands accumulated in double, SwiGLU in double, h then
 *     quantised with its (delayed) scale and the second GEMM run on the
 *     quantised h.
 *
 * Pins (tests/test_oracle_fp8.py): decode against a library's E4M3 table for
 * all 256 codes; encode(decode(c)) = c; encode against a library cast on
 * in-range values; hand-worked ties, subnormals and saturation; integer-valued
 * inputs with unit scales reduce to an exact integer matmul; h before
 * quantisation equals moe_oracle.c's expert FFN on the dequantised operands;
 * closed-form scale values.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };

static inline float ldf(const void* p, size_t i, int dt) {
    if (dt == ORACLE_F32) return ((const float*)p)[i];
    uint32_t u = ((uint32_t)((const uint16_t*)p)[i]) << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* value of an E4M3 code; the two NaN codes (0x7f, 0xff) give NaN */
double oracle_fp8_decode(uint8_t c) {
    int s = c >> 7, e = (c >> 3) & 15, m = c & 7;
    double v;
    if (e == 15 && m == 7) return NAN;
    if (e == 0)
        v = ldexp((double)m / 8.0, -6);        /* subnormal: m/8 * 2^-6 */
    else
        v = ldexp(1.0 + (double)m / 8.0, e - 7);
    return s ? -v : v;
}

/* nearest E4M3 code of x, ties to even, saturating at +-448 */
uint8_t oracle_fp8_encode(float x) {
    uint8_t sign = signbit(x) ? 0x80 : 0x00;
    if (isnan(x)) return (uint8_t)(sign | 0x7f);
    double a = fabs((double)x);
    if (a > 448.0) return (uint8_t)(sign | 0x7e);                    /* 0x7e = 448 */
    if (a < ldexp(1.0, -6)) {
        /* subnormal range: multiples of 2^-9; 8 * 2^-9 is the smallest normal, code 0x08 */
        int q = (int)rint(ldexp(a, 9));
        return (uint8_t)(sign | q);
    }
    int ex;
    double fr = frexp(a, &ex);      /* a = fr * 2^ex, fr in [0.5, 1) */
    int e = ex - 1;                 /* a = (2 fr) * 2^e, 2 fr in [1, 2) */
    int q = (int)rint((2.0 * fr - 1.0) * 8.0);
    if (q == 8) {
        q = 0;
        e += 1;
    }
    if (e > 8 || (e == 8 && q == 7)) return (uint8_t)(sign | 0x7e);  /* rounded past 448 */
    return (uint8_t)(sign | ((e + 7) << 3) | q);
}

/* dst[i] = encode(fp32(src[i] * scale)); *amax = max(*amax, max |src[i]|) */
void oracle_fp8_quantize(const void* src, int dt, size_t n, float scale, uint8_t* dst, float* amax) {
    float m = amax ? *amax : 0.0f;
#pragma omp parallel for schedule(static) reduction(max : m)
    for (long long i = 0; i < (long long)n; ++i) {
        float v = ldf(src, (size_t)i, dt);
        volatile float p = v * scale;   /* one fp32 rounding, never contracted or widened */
        dst[i] = oracle_fp8_encode(p);
        float av = fabsf(v);
        if (av > m) m = av;             /* NaN never enters */
    }
    if (amax) *amax = m;
}

/* scale for this step from the amax values of earlier steps */
float oracle_fp8_delayed_scale(const float* amax_history, int len, int margin) {
    float m = 0.0f;
    for (int i = 0; i < len; ++i)
        if (amax_history[i] > m && isfinite(amax_history[i])) m = amax_history[i];
    if (!(m > 0.0f)) return 1.0f;
    return (float)(448.0 / ((double)m * ldexp(1.0, margin)));
}

/* the 256 code values, filled by the definition above (a loop, not a second definition) */
static double code_value[256];
static void fill_code_values(void) {
    for (int c = 0; c < 256; ++c) code_value[c] = oracle_fp8_decode((uint8_t)c);
}

/*
 * Expert FFN on quantised operands, every expert over its contiguous rows.
 *   xq [R,H], wg/wu [E,F,H], wd [E,H,F]: E4M3 codes.
 *   g = dq_gate * sum_k x w_gate, u = dq_up * sum_k x w_up   (dq = 1 / (scale_x * scale_w))
 *   h = silu(g) * u;  amax_h = max |h|;  hq = encode(fp32(h) * scale_h)
 *   y = dq_down * sum_f dec(hq) w_down                         (dq_down = 1 / (scale_h * scale_wd))
 * h_val (optional) receives h before quantisation.
 */
void oracle_experts_fp8(const uint8_t* xq, const int32_t* offsets, int E, int H, int F,
                        const uint8_t* wg, const uint8_t* wu, const uint8_t* wd,
                        double dq_gate, double dq_up, float scale_h, double dq_down,
                        uint8_t* hq, double* h_val, double* amax_h, double* y) {
    double am = 0.0;
    fill_code_values();
    for (int e = 0; e < E; ++e) {
        const int lo = offsets[e], hi = offsets[e + 1];
        if (hi <= lo) continue;
        const uint8_t* g_w = wg + (size_t)e * F * H;
        const uint8_t* u_w = wu + (size_t)e * F * H;
        const uint8_t* d_w = wd + (size_t)e * H * F;
#pragma omp parallel for collapse(2) schedule(static) reduction(max : am)
        for (int r = lo; r < hi; ++r)
            for (int f = 0; f < F; ++f) {
                double g = 0.0, u = 0.0;
                for (int k = 0; k < H; ++k) {
                    double xv = code_value[xq[(size_t)r * H + k]];
                    g += xv * code_value[g_w[(size_t)f * H + k]];
                    u += xv * code_value[u_w[(size_t)f * H + k]];
                }
                g *= dq_gate;
                u *= dq_up;
                double hv = (g / (1.0 + exp(-g))) * u;
                if (h_val) h_val[(size_t)r * F + f] = hv;
                if (fabs(hv) > am) am = fabs(hv);
                volatile float p = (float)hv * scale_h;
                hq[(size_t)r * F + f] = oracle_fp8_encode(p);
            }
#pragma omp parallel for collapse(2) schedule(static)
        for (int r = lo; r < hi; ++r)
            for (int n = 0; n < H; ++n) {
                double acc = 0.0;
                for (int f = 0; f < F; ++f)
                    acc += code_value[hq[(size_t)r * F + f]] * code_value[d_w[(size_t)n * F + f]];
                y[(size_t)r * H + n] = acc * dq_down;
            }
    }
    if (amax_h) *amax_h = am;
}
