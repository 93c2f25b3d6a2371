/*
 * qarl.h -- C ABI of the MI355X (gfx950) hot path of QaRL: the low-bit quantized MoE
 * expert GEMM at decode and at prefill / training-forward shapes, the weight quantizer
 * that feeds both, the softmax top-k router, and the per-token log-prob comparison.
 *
 * Conventions (all entry points)
 *   - plain C, no exceptions cross the boundary; the return value is a qarl_status;
 *     qarl_last_error() gives the text of the last failure on the calling thread;
 *   - every data pointer is a DEVICE pointer owned by the caller unless the comment says
 *     "host"; the library never frees or keeps them; descriptor structs live on the host;
 *   - the library enqueues kernels on `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream) and returns without synchronising the host; it allocates nothing;
 *   - threads: calls may be made from several host threads at once (no mutable state besides the
 *     per-thread error text and one-time, per-device kernel set-up that is safe to race), as long as
 *     calls that run concurrently do not share output or workspace buffers;
 *   - shapes and alignments are checked before any launch; device-side index arrays
 *     (row_map, expert_offsets, sorted_pairs, target) are trusted to be in range;
 *   - bf16 tensors are raw 16-bit patterns; e4m3 is the OCP "fn" flavour whose largest
 *     finite value is 448 (the alpha of the paper's FP quantizer).
 */
#ifndef QARL_H
#define QARL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    QARL_OK = 0,
    QARL_ERR_INVALID_ARG = -1,
    QARL_ERR_UNSUPPORTED = -2,
    QARL_ERR_ALIGNMENT = -3,
    QARL_ERR_WORKSPACE = -4,
    QARL_ERR_HIP = -5
} qarl_status;

/* Weight formats (the WxAy schemes of section 2.2). */
typedef enum {
    QARL_W4A16_G128 = 1,  /* int4 symmetric, one bf16 scale per 128 consecutive k; bf16 activations */
    QARL_FP8_E4M3_CH = 2, /* e4m3 weights, one fp32 scale per output channel; e4m3 activations, one
                             fp32 scale per token row */
    QARL_FP4_E2M1_CH = 3, /* FP4 weights: e2m1 (the FP quantizer's alpha = 6), one fp32 scale per output
                             channel; activations as for FP8_E4M3_CH (a floating-point W4A8) */
    QARL_W4A8_G128 = 4    /* the weights of W4A16_G128 (same codes, scales and quantizer) with the
                             activations of FP8_E4M3_CH: the W4A8 scheme of the scheme ablation */
} qarl_format;

/* Which kernel family runs the contraction.  Both read the same codes and scales and
 * form the same dequantized weight s*q; they differ in tiling and accumulation order
 * (section 3.1: the learner's low-bit forward mirrors the rollout engine's arithmetic
 * without being bitwise identical). */
typedef enum { QARL_PATH_AUTO = 0, QARL_PATH_DECODE = 1, QARL_PATH_PREFILL = 2 } qarl_path;

typedef enum {
    QARL_EPI_NONE = 0,     /* out[i][n] = Y[i][n]                                  (N columns)  */
    QARL_EPI_SILU_MUL = 1, /* out[i][j] = silu(Y[i][j]) * Y[i][N/2 + j], j < N/2  (N/2 columns) */
    QARL_EPI_COMBINE = 2   /* out[t][n] = sum_slot combine_w[t][slot] * Y[row of (t,slot)][n]   */
} qarl_epilogue;

typedef enum { QARL_OUT_BF16 = 0, QARL_OUT_F32 = 1 } qarl_out_dtype;

/* Quantized weights of E matrices [N][K] (K contiguous).  Host struct, device buffers.
 *   W4A16_G128: codes  uint32, E*N*K/8 words in 1 KiB blocks of 16 rows x 128 k (one scale group
 *                      of 16 consecutive rows), the unit a wavefront of the GEMM kernels loads:
 *                      [E*N/16 row tiles][K/128 groups][4 (k%128)/32][16 n%16][4 (k%32)/8] words;
 *                      a word holds 8 consecutive k as 4-bit codes u = q+8, q in [-8,7]: elements 2i and 2i+1
 *                      (i = 0, 1, 2) occupy bits [3+4i, 6+4i] and [19+4i, 22+4i]; element 6 bits [15, 18];
 *                      element 7 wraps around the word: its low bit is bit 31, its upper three bits are
 *                      bits [0, 2].  (The pair (2i, 2i+1) lands in the top mantissa bits of the two bf16
 *                      halves of a dword after a right shift by 4i, the last pair after a rotation by 12.)
 *               scales bf16   [E][N][K/128]; dequantized weight = float(scale) * q, exact in
 *                      fp32 and never rounded to 16 bits.
 *   FP8_E4M3_CH: codes uint8  [E][N][K] (e4m3 bit patterns); scales float [E][N].
 *   FP4_E2M1_CH: codes uint32 [E][N][K/8]: a word holds 8 consecutive k as e2m1 codes (sign, 2 exponent bits,
 *                      1 mantissa bit; magnitudes 0, 0.5, 1, 1.5, 2, 3, 4, 6): byte b of the word carries
 *                      element b in its low nibble and element 4 + b in its high nibble; scales float [E][N].
 *   W4A8_G128:   as W4A16_G128.
 * Requirements: K % 128 == 0, N % 32 == 0, buffers 16-byte aligned. */
typedef struct {
    int32_t fmt; /* qarl_format */
    int32_t E, N, K;
    int32_t group; /* 128 for W4A16_G128, 0 for FP8_E4M3_CH */
    void *codes;
    void *scales;
} qarl_qweight;

const char *qarl_last_error(void);

/* Bytes of `ws` that qarl_qgemm_grouped may need for a call with these weights, x_rows activation
 * rows, M problem rows and this epilogue, whichever path runs: fp32 staging of Y [M][N] for COMBINE,
 * plus, for W4A16, one fp32 sum per activation row and 128-k scale group (the prefill path computes
 * them once per call).  qarl_token_logprob has its own query. */
size_t qarl_qgemm_workspace_bytes(const qarl_qweight *W, int64_t x_rows, int64_t M, int epilogue);
size_t qarl_logprob_workspace_bytes(int T, int H, int V);

/* Quant of section 2.2 applied to bf16 master weights w [E][N][K], the on-the-fly
 * W_lowbit = Quant(theta_BF16) of section 3.1; writes out->codes and out->scales.
 *   W4A16_G128 (integer Quant, z = 0): per row and group of 128 k, scale =
 *     bf16_rne(absmax / 7) with an IEEE fp32 divide, q = clamp(rne(w / scale), -8, 7)
 *     dividing by the stored scale; a zero group gets scale 0 and codes 0.
 *   FP8_E4M3_CH (FP Quant, alpha = 448): per row, scale = absmax / 448 (fp32),
 *     code = e4m3_rne_saturating(w / scale); a zero row gets scale 0 and codes +0.
 *   FP4_E2M1_CH (FP Quant, alpha = 6): per row, scale = absmax / 6 (fp32),
 *     code = e2m1_rne_saturating(w / scale); a zero row gets scale 0 and codes +0.
 *   W4A8_G128: as W4A16_G128.
 * Errors: INVALID_ARG (null pointers, E/N/K <= 0, wrong group), ALIGNMENT, UNSUPPORTED. */
int qarl_quantize_weights(const void *w_bf16, const qarl_qweight *out, void *stream);

/* Sizes of the two buffers of a qarl_qweight, in bytes (0 for an unknown format or non-positive sizes). */
size_t qarl_codes_bytes(int fmt, int E, int N, int K);
size_t qarl_scales_bytes(int fmt, int E, int N, int K);

/* The codes of W in a layout-free form, for a consumer outside this library (section 3.1, item 3: the low-bit
 * tensors the learner materialises are what is published to the rollout engine).  The GEMM kernels read the 4-bit
 * formats in a blocked, bit-permuted packing; this call writes the plain one:
 *   W4A16_G128 / W4A8_G128: uint32 [E][N][K/8], element i of a word (k = 8 * word + i) in bits [4i, 4i+3] as q + 8;
 *   FP4_E2M1_CH:            uint32 [E][N][K/8], element i in bits [4i, 4i+3] as the e2m1 code;
 *   FP8_E4M3_CH:            uint8  [E][N][K], a copy (the format is stored this way).
 * codes_out: qarl_codes_bytes(...) bytes, 16-byte aligned.  Scales need no conversion. */
int qarl_codes_to_canonical(const qarl_qweight *W, void *codes_out, void *stream);

/* FP Quant of section 2.2 with one scale per row, for activations (the s_x of eq. (2)):
 * x bf16 [rows][K] -> codes uint8 [rows][K], scales float [rows].  K % 8 == 0. */
int qarl_quantize_rows_fp8(const void *x_bf16, int64_t rows, int K, void *codes, float *scales,
                           void *stream);

/* MoE router.  Per token: softmax over the E bf16 logits in fp32, the topk experts ordered
 * by (logit descending, expert id ascending) as slots 0..topk-1, weights = their
 * probabilities (renormalised to sum 1 if renorm != 0).  Then tokens are grouped by
 * expert: expert_counts[E], expert_offsets[E+1] (exclusive prefix sum), and the
 * (token, slot) pairs p = t*topk + slot listed by (expert, t, slot) in sorted_pairs[T*topk];
 * sorted_tokens[i] = sorted_pairs[i] / topk.  Section 4.1 names the router as where
 * quantized MoE rollouts drift, so ids and grouping are exact integer work.
 * Supported: E % 64 == 0, E <= 256, 1 <= topk <= min(E, 32).  T == 0 is a no-op that
 * still writes zero counts and offsets.  With all four grouping outputs NULL only topk_ids and
 * topk_w are written (what qarl_qgemm_routed consumes). */
int qarl_moe_route(const void *logits_bf16, int T, int E, int topk, int renorm, int32_t *topk_ids,
                   float *topk_w, int32_t *expert_counts, int32_t *expert_offsets,
                   int32_t *sorted_pairs, int32_t *sorted_tokens, void *stream);

/* Grouped quantized GEMM, eq. (1) (W4A16: Y = X * (s_w q)^T with 16-bit X) and eq. (2)
 * (FP8: Y = s_x s_w (X_q W_q^T)), fp32 accumulation.  Row i of the problem, for i in
 * [expert_offsets[e], expert_offsets[e+1]), multiplies expert e's matrix and reads
 * activation row row_map[i] (row i if row_map is NULL).  M = expert_offsets[E] must be
 * passed by the caller (host value).
 *   x          W4A16: bf16 [x_rows][K];  FP8, FP4 and W4A8: uint8 e4m3 [x_rows][K] with x_scales float [x_rows]
 *              (W4A8: Y = s_x * X_q * (s_w q)^T, the integer weights of eq. (1) under the activations of eq. (2))
 *   epilogue   NONE:     out [M][N]
 *              SILU_MUL: rows [0,N/2) of each expert matrix are the gate, [N/2,N) the up
 *                        projection; out bf16 [M][N/2], rounded once from fp32
 *              COMBINE:  Y is staged in ws as fp32 [M][N]; out [T][N] sums the topk rows of each
 *                        token in slot order with weights combine_w [T][topk]; sorted_pairs as
 *                        written by qarl_moe_route
 *   out_dtype  QARL_OUT_BF16 or QARL_OUT_F32 (SILU_MUL: bf16 only)
 *   path       AUTO picks DECODE when the mean rows per expert is small and the shape fits it
 *              (DECODE keeps whole rows of x in LDS: W4A16 needs K % 256 == 0 and K <= 4096, with 16-row
 *              instead of 32-row blocks beyond 2048)
 * Errors: INVALID_ARG, ALIGNMENT, UNSUPPORTED (shape outside the kernels' domain),
 * WORKSPACE (ws missing or smaller than the call needs).  M == 0 is a no-op. */
int qarl_qgemm_grouped(const qarl_qweight *W, const void *x, const float *x_scales, int64_t x_rows,
                       const int32_t *row_map, const int32_t *expert_offsets, int64_t M,
                       int epilogue, const float *combine_w, const int32_t *sorted_pairs, int T,
                       int topk, void *out, int out_dtype, int path, void *ws, size_t ws_bytes,
                       void *stream);

/* Backward of qarl_qgemm_grouped (W4A16, epilogue NONE) under the straight-through estimator of section 3.1, item 2:
 * the forward ran on What = s*q; the gradients are those of Y[i] = What_e x[row_map[i]] with Quant treated as the
 * identity, computed in the trainer's 16-bit precision with fp32 accumulation and meant for the BF16 masters.
 *   qarl_qgemm_grouped_dx:  dx[o(i)][k] = sum_n dy[i][n] * What_e[n][k],  e the expert of row i, o(i) = out_row_map[i]
 *       (i if NULL).  dy bf16 [M][N] in the forward's output row order, dx [M][K] bf16 or fp32.  The scaled gradient
 *       dy[i][n] * s[n][k/128] is rounded to bf16 once before it meets the exact integer codes (so a one-hot dy
 *       returns a row of s*q exactly).  Supported: E <= 256, N % 128 == 0, N <= 8192.
 *   qarl_grouped_dw:        dw[e][n][k] = sum over the rows i of expert e of dy[i][n] * x[row_map[i]][k]
 *       (bf16 x bf16 products, fp32 sums; experts without rows get zeros).  dw [E][N][K] bf16 or fp32.
 *       Supported: N % 128 == 0, K % 128 == 0.
 * Errors: INVALID_ARG, ALIGNMENT, UNSUPPORTED.  M == 0: dx is a no-op, dw is all zeros. */
int qarl_qgemm_grouped_dx(const qarl_qweight *W, const void *dy_bf16, const int32_t *expert_offsets, int64_t M,
                          const int32_t *out_row_map, void *dx, int out_dtype, void *stream);
int qarl_grouped_dw(const void *dy_bf16, const void *x_bf16, const int32_t *row_map, const int32_t *expert_offsets,
                    int64_t M, int E, int N, int K, void *dw, int out_dtype, void *stream);

/* The same contraction driven by the router's ids directly, for decode-sized batches (section 4.1's
 * rollout regime: a few hundred tokens over all experts), so that no grouping pass sits between the
 * router and the expert GEMMs: problem row pr = t*topk + slot, pr in [0, T*topk), multiplies expert
 * topk_ids[pr].  It reads activation row t (x_per_token != 0: x is bf16 [T][K]) or row pr (x is bf16
 * [T*topk][K]) and writes output row pr; every workgroup lists its expert's rows itself, in increasing
 * pr, which is the (expert, token, slot) order of qarl_moe_route's grouping.
 *   epilogue   NONE: out [T*topk][N];  SILU_MUL: out bf16 [T*topk][N/2];
 *              COMBINE: Y staged in ws as fp32 [T*topk][N] (qarl_qgemm_workspace_bytes with M = T*topk),
 *              out [T][N] = sum over slots of combine_w[t][slot] * Y[t*topk + slot], in slot order
 * x is 16-bit for every format.  For the e4m3-activation formats FP8, FP4 and W4A8 the kernel applies the activation
 * quantizer of eq. (2) to the rows it gathers (s_x = absmax / 448 per row, e4m3 codes of x / s_x: the arithmetic
 * of qarl_quantize_rows_fp8), so a decode step has no separate quantizer launch for x or for the intermediate.
 * Results equal those of qarl_qgemm_grouped on the DECODE path with the grouping of the same ids (after
 * qarl_quantize_rows_fp8 for the e4m3-activation formats), bit for bit (same kernels, same order of operations per row).
 * Supported: W4A16_G128 and W4A8_G128 (N % 32 == 0, K % 256 == 0, K <= 2048), FP8_E4M3_CH and FP4_E2M1_CH (N % 32 == 0,
 * K % 128 == 0, K <= 4096); T <= 512, T*topk <= 4096, a token listing an expert at most once (as the router's
 * output does; rows past 512 of one expert would be dropped); ids outside [0, E) select no expert and leave their
 * output rows unwritten.  topk_ids 16-byte aligned.  Errors as for qarl_qgemm_grouped.  T == 0 is a no-op. */
int qarl_qgemm_routed(const qarl_qweight *W, const void *x, int x_per_token, const int32_t *topk_ids,
                      int T, int topk, int epilogue, const float *combine_w, void *out, int out_dtype,
                      void *ws, size_t ws_bytes, void *stream);

/* LM head fused with the per-token log-prob: z = inv_temperature * h W_lm^T (bf16 inputs,
 * fp32 accumulation, logits never stored), logprob[t] = z[t][target[t]] - logsumexp_v z[t][v].
 * If ref_logprob is given, also the mismatch comparison of eq. (3) in log space:
 * delta[t] = logprob[t] - ref_logprob[t], and per sequence s (tokens
 * [seq_offsets[s], seq_offsets[s+1])) the sequence-level weight of section 3.2,
 * seq_w[s] = exp(mean_t delta[t]), with the two-sided cap seq_w_clipped[s] =
 * exp(clip(mean delta, -log c, log c)), c = tis_cap_c > 1.
 *   h bf16 [T][H], w_lm bf16 [V][H], target int32 [T]; H % 64 == 0; inv_temperature > 0
 *   and finite.  A target outside [0, V) gives logprob NaN for that token.
 *   delta, seq_w, seq_w_clipped may each be NULL; seq outputs need seq_offsets and S > 0. */
int qarl_token_logprob(const void *h_bf16, const void *w_lm_bf16, const int32_t *target, int T,
                       int H, int V, float inv_temperature, float *logprob,
                       const float *ref_logprob, const int32_t *seq_offsets, int S,
                       float tis_cap_c, float *delta, float *seq_w, float *seq_w_clipped, void *ws,
                       size_t ws_bytes, void *stream);

/* qarl_token_logprob for callers that cannot allocate device memory or hand over a workspace: code under HIP
 * graph capture, tight serving loops that score the tokens of a decode step, harnesses that forbid hipMalloc.
 * Same arguments, results and errors as qarl_token_logprob without `ws`: the partial maxima and sums of the
 * vocabulary blocks go to an array built into the library's device code, qarl_token_logprob_static_limit()
 * bytes (4 MiB) on every GPU the library runs on, held until the process ends.  The call allocates and frees
 * nothing.  A call whose partials exceed the limit (qarl_logprob_workspace_bytes(T, H, V) > limit; at V = 151936
 * that is T > 881) returns QARL_ERR_WORKSPACE.  The array keeps the last call's contents; every element a
 * call reads it has written before, so nothing needs clearing.  All calls on one GPU share the array: calls
 * that overlap on one GPU (different streams or threads) race and must be serialised by the caller.  The
 * array's address on a device is looked up on the first call made with that device current (make that call
 * outside a graph capture). */
int qarl_token_logprob_static(const void *h_bf16, const void *w_lm_bf16, const int32_t *target, int T, int H,
                              int V, float inv_temperature, float *logprob, const float *ref_logprob,
                              const int32_t *seq_offsets, int S, float tis_cap_c, float *delta, float *seq_w,
                              float *seq_w_clipped, void *stream);
size_t qarl_token_logprob_static_limit(void);

/* The comparison half of qarl_token_logprob on two existing log-prob streams (learner
 * and sampler): delta, token weight w = exp(delta) (eq. (3)), seq_w and seq_w_clipped as
 * above.  Any output may be NULL. */
int qarl_logprob_mismatch(const float *lp_learner, const float *lp_sampler, int T,
                          const int32_t *seq_offsets, int S, float tis_cap_c, float *delta,
                          float *token_w, float *seq_w, float *seq_w_clipped, void *stream);

/* Sequence-level surrogate of section 3.2 ("Sequence Level Objectives"; ratio and weight as in the
 * appendix figure "Sequence ratio and weight definition") on the log-probs the two calls above
 * produce.  Response s = tokens [seq_offsets[s], seq_offsets[s+1]), L of them, is one action whose
 * probability is the geometric mean of its token probabilities:
 *   r_seq[s]         = exp(mean_t (lp_current[t] - lp_old[t]))
 *   w_seq_clipped[s] = exp(clip(mean_t (lp_old[t] - lp_sampler[t]), -log c, log c)),  c = tis_cap_c > 1
 *   r_clipped[s]     = clip(r_seq, 1 - eps_low,   1 + eps_high)    if advantage[s] >= 0
 *                      clip(r_seq, 1 - delta_low, 1 + delta_high)  if advantage[s] <  0
 *                      (the section's band [0, 1 + eps_h] for non-negative advantages is eps_low = 1)
 *   in_band[s]       = 1 if the ratio lies inside its band (bounds included), else 0: a response
 *                      outside is masked out of the update
 *   objective_seq[s] = w_seq_clipped * r_clipped * advantage[s]
 *   objective[0]     = mean of objective_seq over the responses that have tokens (0 if none)
 *   grad_lp_current[t] = d objective / d lp_current[t], the mismatch weight held constant:
 *                      in_band * w_seq_clipped * advantage * r_seq / (L * responses with tokens)
 * A response without tokens has ratio and weights 1, objective 0 and does not count in the mean.
 * All streams fp32 [T], advantage fp32 [S], seq_offsets int32 [S+1] ascending within [0, T].
 * objective and objective_seq are required; r_seq, w_seq_clipped, r_clipped, in_band and
 * grad_lp_current may each be NULL.  Tokens outside every response keep their old grad value.
 * Sums run in a fixed order in fp64, exp in fp32.  Errors: INVALID_ARG. */
int qarl_tbpo_objective(const float *lp_current, const float *lp_old, const float *lp_sampler, int T,
                        const int32_t *seq_offsets, int S, const float *advantage, float eps_low,
                        float eps_high, float delta_low, float delta_high, float tis_cap_c,
                        float *r_seq, float *w_seq_clipped, float *r_clipped, int32_t *in_band,
                        float *objective_seq, float *objective, float *grad_lp_current, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* QARL_H */
