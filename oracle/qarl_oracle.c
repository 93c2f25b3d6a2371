/*
 * qarl_oracle.c -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow CPU statement of what the QaRL low-bit MoE hot path computes:
 * weight quantization (integer and floating-point forms, paper section 2.2
 * "Quantization", the Quant/Dequant equations), the quantized GEMM of eq. (1)
 * and eq. (2), a softmax top-k router, the SiLU-gated expert FFN, the per-token
 * log-probability, the token / sequence mismatch weights (eq. (3) and the
 * sequence-level definitions of section 3.2 and the appendix figure "Sequence
 * ratio and weight definition"), and the sequence-level surrogate of section
 * 3.2 ("Sequence Level Objectives") built from them.
 *
 * It shares no code, header, table or constant with the HIP library.  Only the
 * tests, the smoke check and the benchmark's cpu_baseline leg may call it; the
 * product path never does.  Floating point is evaluated in double unless the
 * step is one whose precision the workload fixes (the quantizer's fp32 divide
 * and bf16 scale; the optional fp32 accumulator used only to size the
 * accumulation-order noise floor).
 *
 * No blocking, fusion or reordering: every function is the definition written
 * out as loops.  OpenMP only splits independent outer iterations.
 *
 * Pins: tests/test_oracle_*.py (exact rational nearest-code checks, all 256
 * e4m3 patterns, full-sort routing, one-hot / exact-integer GEMM regimes,
 * closed-form log-probs, geometric-mean / finite-difference checks of the
 * sequence objective).  Anything not covered there is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ bf16 -- */

static inline float bf16_to_f32(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* Nearest bf16 (8 significant bits), ties to even, from a double.  Done on the
 * value, not on bits of an intermediate float, so there is one rounding. */
static uint16_t bf16_from_double(double d)
{
    if (isnan(d)) return 0x7fc0;
    uint16_t sign = signbit(d) ? 0x8000 : 0;
    double a = fabs(d);
    if (a == 0.0) return sign;
    if (isinf(a)) return sign | 0x7f80;
    int e = ilogb(a);
    if (e < -126) e = -126;                 /* subnormal range: fixed quantum */
    double q = nearbyint(ldexp(a, 7 - e));  /* default mode: ties to even     */
    double r = ldexp(q, e - 7);
    if (r >= ldexp(1.0, 128)) return sign | 0x7f80;
    float f = (float)r;                     /* exact: r has <= 8 significant bits */
    uint32_t u;
    memcpy(&u, &f, 4);
    return sign | (uint16_t)(u >> 16);
}

uint16_t oracle_bf16_from_double(double d) { return bf16_from_double(d); }
double oracle_bf16_to_double(uint16_t h) { return (double)bf16_to_f32(h); }

/* ------------------------------------------------------------- e4m3 (OCP) -- */
/* alpha = 448 is the largest finite e4m3 value (paper section 2.2): that is the
 * OCP "fn" flavour: bias 7, no infinities, 0x7f/0xff = NaN, subnormals kept. */

double oracle_e4m3_decode(uint8_t c)
{
    int s = c >> 7, e = (c >> 3) & 15, m = c & 7;
    double v;
    if (e == 15 && m == 7) return NAN;
    if (e == 0) v = ldexp((double)m, -9);            /* m/8 * 2^-6 */
    else        v = ldexp(1.0 + m / 8.0, e - 7);
    return s ? -v : v;
}

/* Nearest representable value, ties to the even code, saturating at +-448. */
uint8_t oracle_e4m3_encode(double x)
{
    if (isnan(x)) return 0x7f;
    uint8_t sign = signbit(x) ? 0x80 : 0;
    double a = fabs(x);
    if (a >= 448.0) return sign | 0x7e;
    int lo = 0;                                      /* largest code with value <= a */
    for (int c = 0; c <= 0x7e; ++c)
        if (oracle_e4m3_decode((uint8_t)c) <= a) lo = c;
    if (lo == 0x7e) return sign | 0x7e;
    double dl = a - oracle_e4m3_decode((uint8_t)lo);
    double dh = oracle_e4m3_decode((uint8_t)(lo + 1)) - a;
    int pick = (dl < dh) ? lo : (dl > dh) ? lo + 1 : ((lo & 1) ? lo + 1 : lo);
    return sign | (uint8_t)pick;
}

/* Same rounding, but the bracket is found by bisection over a table of the 127
 * non-negative finite values so that whole weight matrices finish in reasonable
 * time.  test_oracle_fp8 checks it against the linear search above. */
static void e4m3_table(double *tab)
{
    for (int c = 0; c <= 0x7e; ++c) tab[c] = oracle_e4m3_decode((uint8_t)c);
}

static uint8_t e4m3_encode_tab(const double *tab, double x)
{
    if (isnan(x)) return 0x7f;
    uint8_t sign = signbit(x) ? 0x80 : 0;
    double a = fabs(x);
    if (a >= 448.0) return sign | 0x7e;
    int lo = 0, hi = 0x7e;                           /* tab[lo] <= a < tab[hi] */
    while (hi - lo > 1) {
        int mid = (lo + hi) / 2;
        if (tab[mid] <= a) lo = mid; else hi = mid;
    }
    double dl = a - tab[lo], dh = tab[lo + 1] - a;
    int pick = (dl < dh) ? lo : (dl > dh) ? lo + 1 : ((lo & 1) ? lo + 1 : lo);
    return sign | (uint8_t)pick;
}

uint8_t oracle_e4m3_encode_fast(double x)
{
    double tab[0x7f];
    e4m3_table(tab);
    return e4m3_encode_tab(tab, x);
}

/* ------------------------------------------------- integer quantizer (W4) -- */
/* Section 2.2, integer Quant with z = 0, q in [-8, 7], one scale per group of
 * `group` consecutive k of a row.  scale = bf16(absmax / 7) with an fp32 divide;
 * code = clamp(round_half_even(w / scale)) with an fp32 divide by the stored
 * (already rounded) scale.  A zero group has scale 0 and codes 0.
 * Packing: word[r][k/8] holds element 8*(k/8)+i in bits [4i, 4i+3] as q + 8. */
void oracle_quantize_int4(const uint16_t *w, int64_t rows, int K, int group,
                          uint32_t *codes, uint16_t *scales)
{
    int G = K / group;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        const uint16_t *wr = w + r * K;
        uint32_t *cr = codes + r * (K / 8);
        memset(cr, 0, sizeof(uint32_t) * (K / 8));
        for (int g = 0; g < G; ++g) {
            float am = 0.0f;
            for (int k = g * group; k < (g + 1) * group; ++k) {
                float a = fabsf(bf16_to_f32(wr[k]));
                if (a > am) am = a;
            }
            volatile float s32 = am / 7.0f;
            uint16_t sb = bf16_from_double((double)s32);
            scales[r * G + g] = sb;
            float s = bf16_to_f32(sb);
            for (int k = g * group; k < (g + 1) * group; ++k) {
                int q = 0;
                if (s != 0.0f) {
                    volatile float t = bf16_to_f32(wr[k]) / s;
                    float rr = nearbyintf(t);
                    if (rr < -8.0f) rr = -8.0f;
                    if (rr > 7.0f) rr = 7.0f;
                    q = (int)rr;
                }
                cr[k / 8] |= (uint32_t)(q + 8) << (4 * (k % 8));
            }
        }
    }
}

/* Dequant of section 2.2: What = s * (q - z), z = 0; exact in fp32 (8-bit x 4-bit). */
void oracle_dequant_int4(const uint32_t *codes, const uint16_t *scales, int64_t rows,
                         int K, int group, float *out)
{
    int G = K / group;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r)
        for (int k = 0; k < K; ++k) {
            int q = (int)((codes[r * (K / 8) + k / 8] >> (4 * (k % 8))) & 15) - 8;
            out[r * K + k] = bf16_to_f32(scales[r * G + k / group]) * (float)q;
        }
}

/* ------------------------------------------- floating-point quantizer (FP8) -- */
/* Section 2.2, FP Quant: s = max|row| / 448 (fp32 divide), code = e4m3(w / s)
 * with an fp32 divide.  One scale per row: per output channel for weights,
 * per token for activations.  A zero row has scale 0 and codes +0. */
void oracle_quantize_fp8_rows(const uint16_t *x, int64_t rows, int K, uint8_t *codes,
                              float *scales)
{
    double tab[0x7f];
    e4m3_table(tab);
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        float am = 0.0f;
        for (int k = 0; k < K; ++k) {
            float a = fabsf(bf16_to_f32(x[r * K + k]));
            if (a > am) am = a;
        }
        volatile float s = am / 448.0f;
        scales[r] = s;
        for (int k = 0; k < K; ++k) {
            if (s == 0.0f) { codes[r * K + k] = 0; continue; }
            volatile float t = bf16_to_f32(x[r * K + k]) / s;
            codes[r * K + k] = e4m3_encode_tab(tab, (double)t);
        }
    }
}

/* -------------------------------------------------------------- e2m1 (FP4) -- */
/* Section 2.2, FP Quant with alpha = 6 for FP4: the e2m1 format (1 sign, 2 exponent, 1 mantissa bit, bias 1,
 * no infinities or NaN).  Code c = s e1 e0 m; magnitudes 0, 0.5 (the one subnormal), 1, 1.5, 2, 3, 4, 6. */
double oracle_e2m1_decode(uint8_t c)
{
    int s = (c >> 3) & 1, e = (c >> 1) & 3, m = c & 1;
    double v = (e == 0) ? 0.5 * m : ldexp(1.0 + 0.5 * m, e - 1);
    return s ? -v : v;
}

/* Nearest representable value, ties to the even code, saturating at +-6. */
uint8_t oracle_e2m1_encode(double x)
{
    if (isnan(x)) return 0;
    uint8_t sign = signbit(x) ? 8 : 0;
    double a = fabs(x);
    if (a >= 6.0) return sign | 7;
    int lo = 0;                                      /* largest magnitude code with value <= a */
    for (int c = 0; c <= 7; ++c)
        if (oracle_e2m1_decode((uint8_t)c) <= a) lo = c;
    double dl = a - oracle_e2m1_decode((uint8_t)lo);
    double dh = oracle_e2m1_decode((uint8_t)(lo + 1)) - a;
    int pick = (dl < dh) ? lo : (dl > dh) ? lo + 1 : ((lo & 1) ? lo + 1 : lo);
    return sign | (uint8_t)pick;
}

/* FP Quant of section 2.2 with alpha = 6: s = max|row| / 6 (fp32 divide), code = e2m1(w / s) with an fp32
 * divide, one scale per row (output channel).  Codes are returned one per byte (values 0..15); how a
 * consumer packs them is not part of the definition.  A zero row has scale 0 and codes +0. */
void oracle_quantize_fp4_rows(const uint16_t *x, int64_t rows, int K, uint8_t *codes, float *scales)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        float am = 0.0f;
        for (int k = 0; k < K; ++k) {
            float a = fabsf(bf16_to_f32(x[r * K + k]));
            if (a > am) am = a;
        }
        volatile float s = am / 6.0f;
        scales[r] = s;
        for (int k = 0; k < K; ++k) {
            if (s == 0.0f) { codes[r * K + k] = 0; continue; }
            volatile float t = bf16_to_f32(x[r * K + k]) / s;
            codes[r * K + k] = oracle_e2m1_encode((double)t);
        }
    }
}

/* ------------------------------------------------------------------ router -- */
/* Softmax over all E logits, the top `topk` experts ordered by (logit
 * descending, expert id ascending), their probabilities renormalised to 1. */
void oracle_route(const uint16_t *logits, int T, int E, int topk, int renorm,
                  int32_t *ids, double *wts)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        const uint16_t *lr = logits + (int64_t)t * E;
        double m = -INFINITY, z = 0.0;
        for (int e = 0; e < E; ++e) if (bf16_to_f32(lr[e]) > m) m = bf16_to_f32(lr[e]);
        for (int e = 0; e < E; ++e) z += exp((double)bf16_to_f32(lr[e]) - m);
        char *taken = (char *)calloc(E, 1);
        double psum = 0.0;
        for (int j = 0; j < topk; ++j) {
            int best = -1;
            for (int e = 0; e < E; ++e) {
                if (taken[e]) continue;
                if (best < 0 || bf16_to_f32(lr[e]) > bf16_to_f32(lr[best])) best = e;
            }
            taken[best] = 1;
            ids[(int64_t)t * topk + j] = best;
            wts[(int64_t)t * topk + j] = exp((double)bf16_to_f32(lr[best]) - m) / z;
            psum += wts[(int64_t)t * topk + j];
        }
        if (renorm)
            for (int j = 0; j < topk; ++j) wts[(int64_t)t * topk + j] /= psum;
        free(taken);
    }
}

/* Tokens grouped by expert: counts, exclusive offsets, and the (token, slot)
 * pairs p = t*topk + slot listed by (expert, t, slot). */
void oracle_group(const int32_t *ids, int T, int E, int topk, int32_t *counts,
                  int32_t *offsets, int32_t *sorted_pairs)
{
    int64_t pos = 0;
    for (int e = 0; e < E; ++e) {
        offsets[e] = (int32_t)pos;
        int c = 0;
        for (int t = 0; t < T; ++t)
            for (int j = 0; j < topk; ++j)
                if (ids[(int64_t)t * topk + j] == e) {
                    sorted_pairs[pos++] = t * topk + j;
                    ++c;
                }
        counts[e] = c;
    }
    offsets[E] = (int32_t)pos;
}

/* ------------------------------------------------------------ grouped GEMM -- */
/* eq. (1) with 16-bit activations: Y[i][n] = sum_k What_e[n][k] * x[row(i)][k]
 * for the rows i in [offsets[e], offsets[e+1]) of expert e, where
 * What = s * q is the exact fp32 dequantized weight.  acc32 != 0 accumulates in
 * fp32 in ascending k (noise-floor reference); otherwise in double. */
void oracle_qgemm_w4a16(const uint16_t *x, int K, const int32_t *row_map, int64_t M,
                        const int32_t *offsets, int E, const uint32_t *codes,
                        const uint16_t *scales, int N, int group, int acc32, double *out)
{
    float *wd = (float *)malloc(sizeof(float) * (size_t)N * K);
    for (int e = 0; e < E; ++e) {
        int64_t lo = offsets[e], hi = offsets[e + 1];
        if (hi <= lo) continue;
        oracle_dequant_int4(codes + (int64_t)e * N * (K / 8),
                            scales + (int64_t)e * N * (K / group), N, K, group, wd);
#pragma omp parallel for collapse(2) schedule(static)
        for (int64_t i = lo; i < hi; ++i)
            for (int n = 0; n < N; ++n) {
                const uint16_t *xr = x + (row_map ? (int64_t)row_map[i] : i) * K;
                const float *wn = wd + (int64_t)n * K;
                if (acc32) {
                    float a = 0.0f;
                    for (int k = 0; k < K; ++k) a += wn[k] * bf16_to_f32(xr[k]);
                    out[i * N + n] = (double)a;
                } else {
                    double a = 0.0;
                    for (int k = 0; k < K; ++k) a += (double)wn[k] * (double)bf16_to_f32(xr[k]);
                    out[i * N + n] = a;
                }
            }
    }
    free(wd);
    (void)M;
}

/* Backward of eq. (1) under the straight-through estimator (section 3.1, item 2: the forward runs on the low-bit
 * weights, gradients are taken as if Quant were the identity and applied to the BF16 masters).  With
 * Y[i] = What_e x[row(i)] the two gradients are
 *     dX[i][k]    = sum_n dY[i][n] * What_e[n][k]                  (the input gradient sees the dequantized weight),
 *     dW[e][n][k] = sum_{i in expert e} dY[i][n] * x[row(i)][k]    (the weight gradient passes straight to the master),
 * dY bf16 [M][N] in the row order of the forward's output, everything accumulated in double. */
void oracle_qgemm_w4a16_dx(const uint16_t *dy, int K, int64_t M, const int32_t *offsets, int E,
                           const uint32_t *codes, const uint16_t *scales, int N, int group, double *dx)
{
    float *wd = (float *)malloc(sizeof(float) * (size_t)N * K);
    for (int e = 0; e < E; ++e) {
        int64_t lo = offsets[e], hi = offsets[e + 1];
        if (hi <= lo) continue;
        oracle_dequant_int4(codes + (int64_t)e * N * (K / 8),
                            scales + (int64_t)e * N * (K / group), N, K, group, wd);
#pragma omp parallel for collapse(2) schedule(static)
        for (int64_t i = lo; i < hi; ++i)
            for (int k = 0; k < K; ++k) {
                double a = 0.0;
                for (int n = 0; n < N; ++n) a += (double)bf16_to_f32(dy[i * N + n]) * (double)wd[(int64_t)n * K + k];
                dx[i * K + k] = a;
            }
    }
    free(wd);
    (void)M;
}

void oracle_grouped_dw(const uint16_t *dy, const uint16_t *x, int K, const int32_t *row_map, int64_t M,
                       const int32_t *offsets, int E, int N, double *dw)
{
    for (int e = 0; e < E; ++e) {
        int64_t lo = offsets[e], hi = offsets[e + 1];
#pragma omp parallel for collapse(2) schedule(static)
        for (int n = 0; n < N; ++n)
            for (int k = 0; k < K; ++k) {
                double a = 0.0;
                for (int64_t i = lo; i < hi; ++i) {
                    int64_t r = row_map ? (int64_t)row_map[i] : i;
                    a += (double)bf16_to_f32(dy[i * N + n]) * (double)bf16_to_f32(x[r * K + k]);
                }
                dw[((int64_t)e * N + n) * K + k] = a;
            }
    }
    (void)M;
}

/* eq. (2): Y[i][n] = s_x[row] * s_w[e][n] * sum_k x_q[row][k] * w_q[e][n][k]. */
void oracle_qgemm_fp8(const uint8_t *xq, const float *sx, int K, const int32_t *row_map,
                      int64_t M, const int32_t *offsets, int E, const uint8_t *wq,
                      const float *sw, int N, double *out)
{
    double dec[256];
    for (int c = 0; c < 256; ++c) dec[c] = oracle_e4m3_decode((uint8_t)c);
    for (int e = 0; e < E; ++e) {
        int64_t lo = offsets[e], hi = offsets[e + 1];
#pragma omp parallel for collapse(2) schedule(static)
        for (int64_t i = lo; i < hi; ++i)
            for (int n = 0; n < N; ++n) {
                int64_t r = row_map ? (int64_t)row_map[i] : i;
                const uint8_t *xr = xq + r * K;
                const uint8_t *wn = wq + ((int64_t)e * N + n) * K;
                double a = 0.0;
                for (int k = 0; k < K; ++k) a += dec[xr[k]] * dec[wn[k]];
                out[i * N + n] = (double)sx[r] * (double)sw[(int64_t)e * N + n] * a;
            }
    }
    (void)M;
}

/* eq. (2) with FP4 weights: Y[i][n] = s_x[row] * s_w[e][n] * sum_k x_q[row][k] * w_q[e][n][k], x_q e4m3 codes,
 * w_q e2m1 codes (one per byte). */
void oracle_qgemm_fp4w(const uint8_t *xq, const float *sx, int K, const int32_t *row_map,
                       int64_t M, const int32_t *offsets, int E, const uint8_t *wq,
                       const float *sw, int N, double *out)
{
    double dec8[256], dec4[16];
    for (int c = 0; c < 256; ++c) dec8[c] = oracle_e4m3_decode((uint8_t)c);
    for (int c = 0; c < 16; ++c) dec4[c] = oracle_e2m1_decode((uint8_t)c);
    for (int e = 0; e < E; ++e) {
        int64_t lo = offsets[e], hi = offsets[e + 1];
#pragma omp parallel for collapse(2) schedule(static)
        for (int64_t i = lo; i < hi; ++i)
            for (int n = 0; n < N; ++n) {
                int64_t r = row_map ? (int64_t)row_map[i] : i;
                const uint8_t *xr = xq + r * K;
                const uint8_t *wn = wq + ((int64_t)e * N + n) * K;
                double a = 0.0;
                for (int k = 0; k < K; ++k) a += dec8[xr[k]] * dec4[wn[k] & 15];
                out[i * N + n] = (double)sx[r] * (double)sw[(int64_t)e * N + n] * a;
            }
    }
    (void)M;
}

/* W4A8: the integer weight quantizer of eq. (1) (int4, one bf16 scale per group of k) with the activations of
 * eq. (2) (e4m3 codes, one fp32 scale per token row):
 * Y[i][n] = s_x[row] * sum_k (s_w[e][n][k / group] * q[e][n][k]) * x_q[row][k]. */
void oracle_qgemm_w4a8(const uint8_t *xq, const float *sx, int K, const int32_t *row_map, int64_t M,
                       const int32_t *offsets, int E, const uint32_t *codes, const uint16_t *scales,
                       int N, int group, double *out)
{
    double dec8[256];
    for (int c = 0; c < 256; ++c) dec8[c] = oracle_e4m3_decode((uint8_t)c);
    float *wd = (float *)malloc(sizeof(float) * (size_t)N * K);
    for (int e = 0; e < E; ++e) {
        int64_t lo = offsets[e], hi = offsets[e + 1];
        if (hi <= lo) continue;
        oracle_dequant_int4(codes + (int64_t)e * N * (K / 8),
                            scales + (int64_t)e * N * (K / group), N, K, group, wd);
#pragma omp parallel for collapse(2) schedule(static)
        for (int64_t i = lo; i < hi; ++i)
            for (int n = 0; n < N; ++n) {
                int64_t r = row_map ? (int64_t)row_map[i] : i;
                const uint8_t *xr = xq + r * K;
                const float *wn = wd + (int64_t)n * K;
                double a = 0.0;
                for (int k = 0; k < K; ++k) a += (double)wn[k] * dec8[xr[k]];
                out[i * N + n] = (double)sx[r] * a;
            }
    }
    free(wd);
    (void)M;
}

/* SiLU-gated product of an expert FFN: a[j] = bf16( g/(1+e^-g) * u ), with
 * g = gu[j], u = gu[I + j] taken unrounded from the gate_up GEMM. */
void oracle_silu_mul(const double *gu, int64_t M, int I, uint16_t *a_bf16, double *a_exact)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i)
        for (int j = 0; j < I; ++j) {
            double g = gu[i * 2 * I + j], u = gu[i * 2 * I + I + j];
            double v = g / (1.0 + exp(-g)) * u;
            if (a_exact) a_exact[i * I + j] = v;
            a_bf16[i * I + j] = bf16_from_double(v);
        }
}

/* out[t][n] = sum over slots 0..topk-1 (in slot order) of w[t][slot] * Y[row of
 * pair (t,slot)][n]; Y rows are in sorted order, sorted_pairs[i] = t*topk+slot. */
void oracle_combine(const double *y, const int32_t *sorted_pairs, const double *wts, int T,
                    int topk, int N, double *out, uint16_t *out_bf16)
{
    int64_t M = (int64_t)T * topk;
    int64_t *row_of_pair = (int64_t *)malloc(sizeof(int64_t) * M);
    for (int64_t i = 0; i < M; ++i) row_of_pair[sorted_pairs[i]] = i;
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t)
        for (int n = 0; n < N; ++n) {
            double a = 0.0;
            for (int j = 0; j < topk; ++j)
                a += wts[(int64_t)t * topk + j] * y[row_of_pair[(int64_t)t * topk + j] * N + n];
            out[(int64_t)t * N + n] = a;
            if (out_bf16) out_bf16[(int64_t)t * N + n] = bf16_from_double(a);
        }
    free(row_of_pair);
}

/* ----------------------------------------------------------------- log-prob -- */
/* lp[t] = z[y_t] - log sum_v exp(z[v]),  z[v] = inv_temp * <h[t], W[v]>. */
void oracle_token_logprob(const uint16_t *h, const uint16_t *wlm, const int32_t *target,
                          int T, int H, int V, double inv_temp, double *lp)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int t = 0; t < T; ++t) {
        double *z = (double *)malloc(sizeof(double) * V);
        double m = -INFINITY;
        for (int v = 0; v < V; ++v) {
            double a = 0.0;
            for (int k = 0; k < H; ++k)
                a += (double)bf16_to_f32(h[(int64_t)t * H + k]) *
                     (double)bf16_to_f32(wlm[(int64_t)v * H + k]);
            z[v] = inv_temp * a;
            if (z[v] > m) m = z[v];
        }
        double s = 0.0;
        for (int v = 0; v < V; ++v) s += exp(z[v] - m);
        lp[t] = z[target[t]] - (m + log(s));
        free(z);
    }
}

/* eq. (3) in log space, and the sequence-level weight (geometric mean of the
 * token ratios); cap reading: clip log w to [-log c, log c]. */
void oracle_mismatch(const double *lp_learner, const double *lp_sampler,
                     const int32_t *seq_offsets, int S, double c, double *delta, double *w,
                     double *w_seq, double *w_seq_clipped)
{
    for (int s = 0; s < S; ++s) {
        double acc = 0.0;
        int lo = seq_offsets[s], hi = seq_offsets[s + 1];
        for (int t = lo; t < hi; ++t) {
            delta[t] = lp_learner[t] - lp_sampler[t];
            w[t] = exp(delta[t]);
            acc += delta[t];
        }
        double mean = (hi > lo) ? acc / (double)(hi - lo) : 0.0;
        w_seq[s] = exp(mean);
        double lc = log(c);
        double cm = mean < -lc ? -lc : (mean > lc ? lc : mean);
        w_seq_clipped[s] = exp(cm);
    }
}

/* Sequence-level surrogate of section 3.2 ("Sequence Level Objectives"; ratio and weight as in
 * the appendix figure "Sequence ratio and weight definition").  A response o of L tokens is one
 * action whose probability is the geometric mean of its token probabilities, so in log space
 *     r  = exp(mean_t (lp_current - lp_old)),      w = exp(mean_t (lp_old - lp_sampler)),
 *     w~ = exp(clip(log w, -log c, log c))                    (the two-sided cap, c > 1),
 *     r~ = clip(r, 1 - eps_low,   1 + eps_high)   if A >= 0   (the paper's bound [0, 1 + eps_h] is eps_low = 1),
 *          clip(r, 1 - delta_low, 1 + delta_high) if A <  0,
 *     objective of the response = w~ * r~ * A,
 * and J is the mean over the responses that have tokens.  A response whose ratio leaves its band is
 * masked out of the update: in_band = (lower <= r <= upper), decided on the ratio itself in fp64
 * (section 3.2 compares the ratio with the band; a test that sets this against an fp32 implementation
 * leaves out responses whose ratio lies within rounding distance of a bound).  grad[t] = dJ/d lp_current[t] with w~ held constant
 * (it does not depend on the current policy) = in_band * w~ * A * r / (L * S'), S' = responses with
 * tokens.  An empty response has r = w = w~ = r~ = 1, objective 0, and does not count in S'. */
void oracle_tbpo(const double *lp_cur, const double *lp_old, const double *lp_smp,
                 const int32_t *seq_offsets, int S, const double *adv, double eps_low, double eps_high,
                 double delta_low, double delta_high, double c, double *r_seq, double *w_clip,
                 double *r_clip, int32_t *in_band, double *obj_seq, double *objective, double *grad)
{
    int nonempty = 0;
    for (int s = 0; s < S; ++s)
        if (seq_offsets[s + 1] > seq_offsets[s]) ++nonempty;
    double total = 0.0;
    for (int s = 0; s < S; ++s) {
        const int lo = seq_offsets[s], hi = seq_offsets[s + 1];
        const int L = hi - lo;
        if (L <= 0) {
            r_seq[s] = w_clip[s] = r_clip[s] = 1.0;
            in_band[s] = 1;
            obj_seq[s] = 0.0;
            continue;
        }
        double sum_r = 0.0, sum_w = 0.0;
        for (int t = lo; t < hi; ++t) {
            sum_r += lp_cur[t] - lp_old[t];
            sum_w += lp_old[t] - lp_smp[t];
        }
        const double r = exp(sum_r / L);
        const double lc = log(c);
        double lw = sum_w / L;
        if (lw < -lc) lw = -lc;
        if (lw > lc) lw = lc;
        const double wt = exp(lw);
        const double lower = adv[s] >= 0.0 ? 1.0 - eps_low : 1.0 - delta_low;
        const double upper = adv[s] >= 0.0 ? 1.0 + eps_high : 1.0 + delta_high;
        const int inside = (r >= lower) && (r <= upper);
        const double rt = inside ? r : (r < lower ? lower : upper);
        r_seq[s] = r;
        w_clip[s] = wt;
        r_clip[s] = rt;
        in_band[s] = inside;
        obj_seq[s] = wt * rt * adv[s];
        total += obj_seq[s];
        if (grad)
            for (int t = lo; t < hi; ++t) grad[t] = inside ? wt * adv[s] * r / ((double)L * (double)nonempty) : 0.0;
    }
    *objective = nonempty ? total / (double)nonempty : 0.0;
}
