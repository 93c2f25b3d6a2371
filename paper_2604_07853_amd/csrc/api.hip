// C ABI of the library: argument validation and dispatch only.  See include/qarl.h.
#include <stdarg.h>
#include <stdio.h>

#include "common.hpp"

namespace qarl {

static thread_local char g_err[512] = "";

void set_error(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

int check_hip(hipError_t e, const char *what)
{
    if (e == hipSuccess) return QARL_OK;
    set_error("%s: %s", what, hipGetErrorString(e));
    return QARL_ERR_HIP;
}

int raise_lds_limit(const void *kernel, LdsLimitOnce &done, const char *what)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) dev = -1;
    const bool tracked = dev >= 0 && dev < 64;
    if (tracked && (done.devices_done[dev >> 5].load(std::memory_order_acquire) >> (dev & 31) & 1u)) return QARL_OK;
    // the dynamic part may fill what the kernel's static LDS leaves of the CU's 160 KiB
    hipFuncAttributes fa;
    int rc = check_hip(hipFuncGetAttributes(&fa, kernel), what);
    if (rc) return rc;
    const int room = kMaxLdsBytes - (int)fa.sharedSizeBytes;
    rc = check_hip(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, room), what);
    if (rc) return rc;
    if (tracked) done.devices_done[dev >> 5].fetch_or(1u << (dev & 31), std::memory_order_release);
    return QARL_OK;
}

static bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }

static int check_qweight(const qarl_qweight *w, const char *who)
{
    if (!w) {
        set_error("%s: null weight descriptor", who);
        return QARL_ERR_INVALID_ARG;
    }
    if (w->fmt != QARL_W4A16_G128 && w->fmt != QARL_FP8_E4M3_CH && w->fmt != QARL_FP4_E2M1_CH && w->fmt != QARL_W4A8_G128) {
        set_error("%s: unknown weight format %d", who, w->fmt);
        return QARL_ERR_UNSUPPORTED;
    }
    if (w->E <= 0 || w->N <= 0 || w->K <= 0) {
        set_error("%s: E, N, K must be positive (got %d, %d, %d)", who, w->E, w->N, w->K);
        return QARL_ERR_INVALID_ARG;
    }
    if (w->K % 128 != 0 || w->N % 32 != 0) {
        set_error("%s: need K %% 128 == 0 and N %% 32 == 0 (got N=%d, K=%d)", who, w->N, w->K);
        return QARL_ERR_UNSUPPORTED;
    }
    if ((w->fmt == QARL_W4A16_G128 || w->fmt == QARL_W4A8_G128) && w->group != 128) {
        set_error("%s: int4 weights support group 128 only (got %d)", who, w->group);
        return QARL_ERR_UNSUPPORTED;
    }
    if (!w->codes || !w->scales) {
        set_error("%s: null codes or scales buffer", who);
        return QARL_ERR_INVALID_ARG;
    }
    if (!aligned16(w->codes) || !aligned16(w->scales)) {
        set_error("%s: codes and scales must be 16-byte aligned", who);
        return QARL_ERR_ALIGNMENT;
    }
    return QARL_OK;
}

}  // namespace qarl

using namespace qarl;

extern "C" {

const char *qarl_last_error(void) { return g_err; }

static size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

static size_t ws_stage_bytes(const qarl_qweight *W, int64_t M, int epilogue)
{
    return epilogue == QARL_EPI_COMBINE ? align256((size_t)M * (size_t)W->N * sizeof(float)) : 0;
}

static bool int4_weights(int fmt) { return fmt == QARL_W4A16_G128 || fmt == QARL_W4A8_G128; }
static bool fp8_activations(int fmt) { return fmt == QARL_FP8_E4M3_CH || fmt == QARL_FP4_E2M1_CH || fmt == QARL_W4A8_G128; }

static size_t ws_sums_bytes(const qarl_qweight *W, int64_t x_rows)
{
    return int4_weights(W->fmt) ? align256((size_t)x_rows * (size_t)(W->K / 128) * sizeof(float)) : 0;
}

// Format bridge: W4A8 widens the e4m3 activations to bf16 (exact) for the W4A16 kernels.
static size_t ws_xwide_bytes(const qarl_qweight *W, int64_t x_rows)
{
    return W->fmt == QARL_W4A8_G128 ? align256((size_t)x_rows * (size_t)W->K * 2) : 0;
}

size_t qarl_qgemm_workspace_bytes(const qarl_qweight *W, int64_t x_rows, int64_t M, int epilogue)
{
    if (!W || M <= 0 || x_rows <= 0 || W->N <= 0 || W->K <= 0) return 0;
    return ws_stage_bytes(W, M, epilogue) + ws_sums_bytes(W, x_rows) + ws_xwide_bytes(W, x_rows);
}

size_t qarl_logprob_workspace_bytes(int T, int H, int V)
{
    if (T <= 0 || H <= 0 || V <= 0) return 0;
    return logprob_ws_bytes(T, H, V);
}

int qarl_quantize_weights(const void *w_bf16, const qarl_qweight *out, void *stream)
{
    int rc = check_qweight(out, "qarl_quantize_weights");
    if (rc) return rc;
    if (!w_bf16) {
        set_error("qarl_quantize_weights: null input");
        return QARL_ERR_INVALID_ARG;
    }
    if (!aligned16(w_bf16)) {
        set_error("qarl_quantize_weights: input must be 16-byte aligned");
        return QARL_ERR_ALIGNMENT;
    }
    const int64_t rows = (int64_t)out->E * out->N;
    if (int4_weights(out->fmt))
        return launch_quantize_int4(w_bf16, rows, out->K, out->codes, out->scales, (hipStream_t)stream);
    if (out->fmt == QARL_FP4_E2M1_CH)
        return launch_quantize_fp4_rows(w_bf16, rows, out->K, out->codes, (float *)out->scales, (hipStream_t)stream);
    return launch_quantize_fp8_rows(w_bf16, rows, out->K, out->codes, (float *)out->scales, (hipStream_t)stream);
}

size_t qarl_codes_bytes(int fmt, int E, int N, int K)
{
    if (E <= 0 || N <= 0 || K <= 0) return 0;
    const size_t n = (size_t)E * (size_t)N * (size_t)K;
    if (fmt == QARL_FP8_E4M3_CH) return n;
    if (fmt == QARL_W4A16_G128 || fmt == QARL_W4A8_G128 || fmt == QARL_FP4_E2M1_CH) return n / 2;
    return 0;
}

size_t qarl_scales_bytes(int fmt, int E, int N, int K)
{
    if (E <= 0 || N <= 0 || K <= 0) return 0;
    if (fmt == QARL_W4A16_G128 || fmt == QARL_W4A8_G128) return (size_t)E * N * (size_t)(K / 128) * 2;
    if (fmt == QARL_FP8_E4M3_CH || fmt == QARL_FP4_E2M1_CH) return (size_t)E * N * sizeof(float);
    return 0;
}

int qarl_codes_to_canonical(const qarl_qweight *W, void *codes_out, void *stream)
{
    int rc = check_qweight(W, "qarl_codes_to_canonical");
    if (rc) return rc;
    if (!codes_out) {
        set_error("qarl_codes_to_canonical: null output");
        return QARL_ERR_INVALID_ARG;
    }
    if (!aligned16(codes_out)) {
        set_error("qarl_codes_to_canonical: output must be 16-byte aligned");
        return QARL_ERR_ALIGNMENT;
    }
    const int64_t rows = (int64_t)W->E * W->N;
    if (W->fmt == QARL_FP8_E4M3_CH)   // stored canonically already: a plain copy
        return check_hip(hipMemcpyAsync(codes_out, W->codes, (size_t)rows * W->K, hipMemcpyDeviceToDevice, (hipStream_t)stream),
                         "hipMemcpyAsync(codes)");
    if (int4_weights(W->fmt) && W->N % 16 != 0) {
        set_error("qarl_codes_to_canonical: N %% 16 == 0 required");
        return QARL_ERR_UNSUPPORTED;
    }
    return launch_canonical_codes(W->fmt, W->codes, rows, W->K, codes_out, (hipStream_t)stream);
}

int qarl_quantize_rows_fp8(const void *x_bf16, int64_t rows, int K, void *codes, float *scales, void *stream)
{
    if (rows < 0 || K <= 0) {
        set_error("qarl_quantize_rows_fp8: rows >= 0 and K > 0 required (got %lld, %d)", (long long)rows, K);
        return QARL_ERR_INVALID_ARG;
    }
    if (rows == 0) return QARL_OK;
    if (!x_bf16 || !codes || !scales) {
        set_error("qarl_quantize_rows_fp8: null pointer");
        return QARL_ERR_INVALID_ARG;
    }
    if (K % 8 != 0) {
        set_error("qarl_quantize_rows_fp8: K %% 8 == 0 required (got %d)", K);
        return QARL_ERR_UNSUPPORTED;
    }
    if (!aligned16(x_bf16) || ((uintptr_t)codes & 7u)) {
        set_error("qarl_quantize_rows_fp8: x must be 16-byte and codes 8-byte aligned");
        return QARL_ERR_ALIGNMENT;
    }
    return launch_quantize_fp8_rows(x_bf16, rows, K, codes, scales, (hipStream_t)stream);
}

int qarl_moe_route(const void *logits_bf16, int T, int E, int topk, int renorm, int32_t *topk_ids, float *topk_w,
                   int32_t *expert_counts, int32_t *expert_offsets, int32_t *sorted_pairs, int32_t *sorted_tokens,
                   void *stream)
{
    if (T < 0 || E <= 0 || topk <= 0) {
        set_error("qarl_moe_route: T >= 0, E > 0, topk > 0 required (got %d, %d, %d)", T, E, topk);
        return QARL_ERR_INVALID_ARG;
    }
    if (E % 64 != 0 || E > 256 || topk > 32 || topk > E) {
        set_error("qarl_moe_route: supports E %% 64 == 0, E <= 256, topk <= min(E, 32) (got E=%d, topk=%d)", E, topk);
        return QARL_ERR_UNSUPPORTED;
    }
    if ((int64_t)T * topk > 0x7fffffffLL) {
        set_error("qarl_moe_route: T*topk overflows int32");
        return QARL_ERR_UNSUPPORTED;
    }
    const bool no_grouping = !expert_counts && !expert_offsets && !sorted_pairs && !sorted_tokens;
    if (no_grouping) {   // ids and weights only (for qarl_qgemm_routed)
        if (T == 0) return QARL_OK;
        if (!logits_bf16 || !topk_ids || !topk_w) {
            set_error("qarl_moe_route: null pointer");
            return QARL_ERR_INVALID_ARG;
        }
        return launch_route_only(logits_bf16, T, E, topk, renorm, topk_ids, topk_w, (hipStream_t)stream);
    }
    if (!expert_counts || !expert_offsets || (T > 0 && (!logits_bf16 || !topk_ids || !topk_w || !sorted_pairs || !sorted_tokens))) {
        set_error("qarl_moe_route: null pointer");
        return QARL_ERR_INVALID_ARG;
    }
    return launch_route(logits_bf16, T, E, topk, renorm, topk_ids, topk_w, expert_counts, expert_offsets,
                        sorted_pairs, sorted_tokens, (hipStream_t)stream);
}

int qarl_qgemm_grouped(const qarl_qweight *W, const void *x, const float *x_scales, int64_t x_rows,
                       const int32_t *row_map, const int32_t *expert_offsets, int64_t M, int epilogue,
                       const float *combine_w, const int32_t *sorted_pairs, int T, int topk, void *out,
                       int out_dtype, int path, void *ws, size_t ws_bytes, void *stream)
{
    int rc = check_qweight(W, "qarl_qgemm_grouped");
    if (rc) return rc;
    if (M < 0 || x_rows < 0) {
        set_error("qarl_qgemm_grouped: negative M or x_rows");
        return QARL_ERR_INVALID_ARG;
    }
    if (epilogue != QARL_EPI_NONE && epilogue != QARL_EPI_SILU_MUL && epilogue != QARL_EPI_COMBINE) {
        set_error("qarl_qgemm_grouped: unknown epilogue %d", epilogue);
        return QARL_ERR_INVALID_ARG;
    }
    if (out_dtype != QARL_OUT_BF16 && out_dtype != QARL_OUT_F32) {
        set_error("qarl_qgemm_grouped: unknown out_dtype %d", out_dtype);
        return QARL_ERR_INVALID_ARG;
    }
    if (path != QARL_PATH_AUTO && path != QARL_PATH_DECODE && path != QARL_PATH_PREFILL) {
        set_error("qarl_qgemm_grouped: unknown path %d", path);
        return QARL_ERR_INVALID_ARG;
    }
    if (epilogue == QARL_EPI_SILU_MUL && (out_dtype != QARL_OUT_BF16 || W->N % 32 != 0)) {
        set_error("qarl_qgemm_grouped: SILU_MUL needs bf16 output and N %% 32 == 0");
        return QARL_ERR_UNSUPPORTED;
    }
    if (M > 0x7fffffffLL / 2 || x_rows > 0x7fffffffLL) {
        set_error("qarl_qgemm_grouped: M or x_rows too large");
        return QARL_ERR_UNSUPPORTED;
    }
    hipStream_t st = (hipStream_t)stream;
    if (epilogue == QARL_EPI_COMBINE) {
        if (T < 0 || topk <= 0 || (int64_t)T * topk != M) {
            set_error("qarl_qgemm_grouped: COMBINE needs T*topk == M (got T=%d, topk=%d, M=%lld)", T, topk, (long long)M);
            return QARL_ERR_INVALID_ARG;
        }
        if (W->N % 4 != 0) {
            set_error("qarl_qgemm_grouped: COMBINE needs N %% 4 == 0");
            return QARL_ERR_UNSUPPORTED;
        }
    }
    if (M == 0) return QARL_OK;
    if (!x || !expert_offsets || !out) {
        set_error("qarl_qgemm_grouped: null pointer");
        return QARL_ERR_INVALID_ARG;
    }
    if (fp8_activations(W->fmt) && !x_scales) {
        set_error("qarl_qgemm_grouped: e4m3 activations need x_scales");
        return QARL_ERR_INVALID_ARG;
    }
    if (!aligned16(x) || !aligned16(out)) {
        set_error("qarl_qgemm_grouped: x and out must be 16-byte aligned");
        return QARL_ERR_ALIGNMENT;
    }
    GemmArgs a;
    a.fmt = W->fmt;
    a.E = W->E;
    a.N = W->N;
    a.K = W->K;
    a.codes = W->codes;
    a.scales = W->scales;
    a.x = x;
    a.x_scales = x_scales;
    a.row_map = row_map;
    a.out_row_map = nullptr;
    a.offsets = expert_offsets;
    a.M = M;
    a.x_rows = x_rows;
    a.epilogue = epilogue;
    a.out = out;
    a.out_f32 = (out_dtype == QARL_OUT_F32);
    a.x_group_sums = nullptr;
    int use = path;
    if (use == QARL_PATH_AUTO)
        use = (M <= (int64_t)W->E * 64 && qgemm_stream_supported(W->fmt, W->N, W->K)) ? QARL_PATH_DECODE : QARL_PATH_PREFILL;
    const size_t stage = ws_stage_bytes(W, M, epilogue);
    const size_t sums = (use == QARL_PATH_PREFILL) ? ws_sums_bytes(W, x_rows) : 0;
    const size_t xwide = ws_xwide_bytes(W, x_rows);
    const size_t need = stage + sums + xwide;
    if (need > 0 && (!ws || ws_bytes < need || !aligned16(ws))) {
        set_error("qarl_qgemm_grouped: this call needs %zu bytes of 16-byte aligned workspace (got %zu)", need, ws_bytes);
        return QARL_ERR_WORKSPACE;
    }
    if (xwide) {   // W4A8: e4m3 rows -> the same values as bf16 rows; the kernels scale by s_x in their epilogue
        void *x16 = (char *)ws + stage + sums;
        rc = launch_e4m3_to_bf16(x, x_rows * (int64_t)W->K, x16, st);
        if (rc) return rc;
        a.x = x16;
    }
    if (epilogue == QARL_EPI_COMBINE) {
        if (!combine_w || !sorted_pairs) {
            set_error("qarl_qgemm_grouped: COMBINE needs combine_w and sorted_pairs");
            return QARL_ERR_INVALID_ARG;
        }
        a.epilogue = QARL_EPI_NONE;
        a.out = ws;
        a.out_f32 = 1;
        a.out_row_map = sorted_pairs;  // Y lands in pair order: row t*topk + slot
    }
    if (sums) {
        float *gs = (float *)((char *)ws + stage);
        rc = launch_group_sums(a.x, x_rows, W->K, gs, st);
        if (rc) return rc;
        a.x_group_sums = gs;
    }
    rc = (use == QARL_PATH_DECODE) ? launch_qgemm_stream(a, st) : launch_qgemm_tile(a, st);
    if (rc) return rc;
    if (epilogue == QARL_EPI_COMBINE)
        return launch_combine((const float *)ws, combine_w, T, topk, W->N, out, out_dtype == QARL_OUT_F32, st);
    return QARL_OK;
}

int qarl_qgemm_routed(const qarl_qweight *W, const void *x, int x_per_token, const int32_t *topk_ids, int T,
                      int topk, int epilogue, const float *combine_w, void *out, int out_dtype, void *ws,
                      size_t ws_bytes, void *stream)
{
    int rc = check_qweight(W, "qarl_qgemm_routed");
    if (rc) return rc;
    if (T < 0 || topk <= 0) {
        set_error("qarl_qgemm_routed: T >= 0 and topk > 0 required");
        return QARL_ERR_INVALID_ARG;
    }
    if (epilogue != QARL_EPI_NONE && epilogue != QARL_EPI_SILU_MUL && epilogue != QARL_EPI_COMBINE) {
        set_error("qarl_qgemm_routed: unknown epilogue %d", epilogue);
        return QARL_ERR_INVALID_ARG;
    }
    if (out_dtype != QARL_OUT_BF16 && out_dtype != QARL_OUT_F32) {
        set_error("qarl_qgemm_routed: unknown out_dtype %d", out_dtype);
        return QARL_ERR_INVALID_ARG;
    }
    if (epilogue == QARL_EPI_SILU_MUL && out_dtype != QARL_OUT_BF16) {
        set_error("qarl_qgemm_routed: SILU_MUL needs bf16 output");
        return QARL_ERR_UNSUPPORTED;
    }
    if (epilogue == QARL_EPI_COMBINE && W->N % 4 != 0) {
        set_error("qarl_qgemm_routed: COMBINE needs N %% 4 == 0");
        return QARL_ERR_UNSUPPORTED;
    }
    if (T == 0) return QARL_OK;
    if (!qgemm_stream_routed_supported(W->fmt, W->N, W->K, T, topk)) {
        set_error("qarl_qgemm_routed: supports W4A16 and W4A8 (N %% 32 == 0, K %% 256 == 0, K <= 2048), FP8 and FP4 (N %% 32 == 0, "
                  "K %% 128 == 0, K <= 4096) with T <= 512 and T * topk <= 4096 (got fmt=%d N=%d K=%d T=%d topk=%d)",
                  W->fmt, W->N, W->K, T, topk);
        return QARL_ERR_UNSUPPORTED;
    }
    if (!x || !topk_ids || !out) {
        set_error("qarl_qgemm_routed: null pointer");
        return QARL_ERR_INVALID_ARG;
    }
    if (!aligned16(x) || !aligned16(out) || !aligned16(topk_ids)) {
        set_error("qarl_qgemm_routed: x, topk_ids and out must be 16-byte aligned");
        return QARL_ERR_ALIGNMENT;
    }
    const int64_t M = (int64_t)T * topk;
    GemmArgs a;
    a.fmt = W->fmt;
    a.E = W->E;
    a.N = W->N;
    a.K = W->K;
    a.codes = W->codes;
    a.scales = W->scales;
    a.x = x;
    a.x_scales = nullptr;
    a.row_map = nullptr;
    a.out_row_map = nullptr;
    a.offsets = nullptr;
    a.M = M;
    a.x_rows = x_per_token ? T : M;
    a.epilogue = epilogue;
    a.out = out;
    a.out_f32 = (out_dtype == QARL_OUT_F32);
    a.x_group_sums = nullptr;
    a.ids = topk_ids;
    a.topk = topk;
    a.x_per_token = x_per_token ? 1 : 0;
    const size_t stage = ws_stage_bytes(W, M, epilogue);
    if (stage > 0 && (!ws || ws_bytes < stage || !aligned16(ws))) {
        set_error("qarl_qgemm_routed: this call needs %zu bytes of 16-byte aligned workspace (got %zu)", stage, ws_bytes);
        return QARL_ERR_WORKSPACE;
    }
    hipStream_t st = (hipStream_t)stream;
    if (epilogue == QARL_EPI_COMBINE) {
        if (!combine_w) {
            set_error("qarl_qgemm_routed: COMBINE needs combine_w");
            return QARL_ERR_INVALID_ARG;
        }
        a.epilogue = QARL_EPI_NONE;
        a.out = ws;
        a.out_f32 = 1;
    }
    rc = launch_qgemm_stream(a, st);
    if (rc) return rc;
    if (epilogue == QARL_EPI_COMBINE)
        return launch_combine((const float *)ws, combine_w, T, topk, W->N, out, out_dtype == QARL_OUT_F32, st);
    return QARL_OK;
}

int qarl_qgemm_grouped_dx(const qarl_qweight *W, const void *dy_bf16, const int32_t *expert_offsets, int64_t M,
                          const int32_t *out_row_map, void *dx, int out_dtype, void *stream)
{
    int rc = check_qweight(W, "qarl_qgemm_grouped_dx");
    if (rc) return rc;
    if (W->fmt != QARL_W4A16_G128) {
        set_error("qarl_qgemm_grouped_dx: W4A16_G128 weights only (got format %d)", W->fmt);
        return QARL_ERR_UNSUPPORTED;
    }
    if (M < 0 || M > 0x7fffffffLL / 2) {
        set_error("qarl_qgemm_grouped_dx: bad M");
        return QARL_ERR_INVALID_ARG;
    }
    if (out_dtype != QARL_OUT_BF16 && out_dtype != QARL_OUT_F32) {
        set_error("qarl_qgemm_grouped_dx: unknown out_dtype %d", out_dtype);
        return QARL_ERR_INVALID_ARG;
    }
    if (M == 0) return QARL_OK;
    if (!dy_bf16 || !expert_offsets || !dx) {
        set_error("qarl_qgemm_grouped_dx: null pointer");
        return QARL_ERR_INVALID_ARG;
    }
    if (!aligned16(dy_bf16) || !aligned16(dx)) {
        set_error("qarl_qgemm_grouped_dx: dy and dx must be 16-byte aligned");
        return QARL_ERR_ALIGNMENT;
    }
    GemmArgs a;
    a.fmt = W->fmt;
    a.E = W->E;
    a.N = W->N;
    a.K = W->K;
    a.codes = W->codes;
    a.scales = W->scales;
    a.x = dy_bf16;
    a.x_scales = nullptr;
    a.x_group_sums = nullptr;
    a.row_map = nullptr;
    a.out_row_map = out_row_map;
    a.offsets = expert_offsets;
    a.M = M;
    a.x_rows = M;
    a.epilogue = QARL_EPI_NONE;
    a.out = dx;
    a.out_f32 = (out_dtype == QARL_OUT_F32);
    return launch_qgemm_dx(a, (hipStream_t)stream);
}

int qarl_grouped_dw(const void *dy_bf16, const void *x_bf16, const int32_t *row_map, const int32_t *expert_offsets,
                    int64_t M, int E, int N, int K, void *dw, int out_dtype, void *stream)
{
    if (E <= 0 || N <= 0 || K <= 0 || M < 0) {
        set_error("qarl_grouped_dw: E, N, K > 0 and M >= 0 required");
        return QARL_ERR_INVALID_ARG;
    }
    if (out_dtype != QARL_OUT_BF16 && out_dtype != QARL_OUT_F32) {
        set_error("qarl_grouped_dw: unknown out_dtype %d", out_dtype);
        return QARL_ERR_INVALID_ARG;
    }
    if (!expert_offsets || !dw || (M > 0 && (!dy_bf16 || !x_bf16))) {
        set_error("qarl_grouped_dw: null pointer");
        return QARL_ERR_INVALID_ARG;
    }
    if (!aligned16(dy_bf16) || !aligned16(x_bf16) || !aligned16(dw)) {
        set_error("qarl_grouped_dw: dy, x and dw must be 16-byte aligned");
        return QARL_ERR_ALIGNMENT;
    }
    return launch_grouped_dw(dy_bf16, x_bf16, row_map, expert_offsets, E, N, K, dw, out_dtype == QARL_OUT_F32,
                             (hipStream_t)stream);
}

int qarl_tbpo_objective(const float *lp_current, const float *lp_old, const float *lp_sampler, int T,
                        const int32_t *seq_offsets, int S, const float *advantage, float eps_low, float eps_high,
                        float delta_low, float delta_high, float tis_cap_c, float *r_seq, float *w_seq_clipped,
                        float *r_clipped, int32_t *in_band, float *objective_seq, float *objective,
                        float *grad_lp_current, void *stream)
{
    if (T < 0 || S < 0) {
        set_error("qarl_tbpo_objective: negative T or S");
        return QARL_ERR_INVALID_ARG;
    }
    if (!(tis_cap_c > 1.0f) || !std::isfinite(tis_cap_c)) {
        set_error("qarl_tbpo_objective: cap c must exceed 1 (got %g)", (double)tis_cap_c);
        return QARL_ERR_INVALID_ARG;
    }
    if (!(eps_low >= 0.f) || !(eps_high >= 0.f) || !(delta_low >= 0.f) || !(delta_high >= 0.f)) {
        set_error("qarl_tbpo_objective: band widths must be non-negative");
        return QARL_ERR_INVALID_ARG;
    }
    if (!objective || (S > 0 && !objective_seq)) {
        set_error("qarl_tbpo_objective: objective and objective_seq are required");
        return QARL_ERR_INVALID_ARG;
    }
    if (S > 0 && (!seq_offsets || !advantage || (T > 0 && (!lp_current || !lp_old || !lp_sampler)))) {
        set_error("qarl_tbpo_objective: null pointer");
        return QARL_ERR_INVALID_ARG;
    }
    if (S == 0) {   // no response: J = 0, written by a one-element fill
        return launch_fill_f32(objective, 1, 0.f, (hipStream_t)stream);
    }
    return launch_tbpo(lp_current, lp_old, lp_sampler, seq_offsets, S, advantage, eps_low, eps_high, delta_low,
                       delta_high, tis_cap_c, r_seq, w_seq_clipped, r_clipped, in_band, objective_seq, objective,
                       grad_lp_current, (hipStream_t)stream);
}

int qarl_logprob_mismatch(const float *lp_learner, const float *lp_sampler, int T, const int32_t *seq_offsets, int S,
                          float tis_cap_c, float *delta, float *token_w, float *seq_w, float *seq_w_clipped,
                          void *stream)
{
    if (T < 0 || S < 0) {
        set_error("qarl_logprob_mismatch: negative T or S");
        return QARL_ERR_INVALID_ARG;
    }
    if (T == 0 && S == 0) return QARL_OK;
    if (!lp_learner || !lp_sampler) {
        set_error("qarl_logprob_mismatch: null log-prob stream");
        return QARL_ERR_INVALID_ARG;
    }
    if ((seq_w || seq_w_clipped) && (!seq_offsets || S <= 0)) {
        set_error("qarl_logprob_mismatch: sequence outputs need seq_offsets and S > 0");
        return QARL_ERR_INVALID_ARG;
    }
    if (seq_w_clipped && !(tis_cap_c > 1.f)) {
        set_error("qarl_logprob_mismatch: cap c must exceed 1 (got %g)", (double)tis_cap_c);
        return QARL_ERR_INVALID_ARG;
    }
    const bool seq = (seq_w || seq_w_clipped);
    return launch_mismatch(lp_learner, lp_sampler, T, seq ? seq_offsets : nullptr, seq ? S : 0, tis_cap_c, delta,
                           token_w, seq_w, seq_w_clipped, (hipStream_t)stream);
}

int qarl_token_logprob(const void *h_bf16, const void *w_lm_bf16, const int32_t *target, int T, int H, int V,
                       float inv_temperature, float *logprob, const float *ref_logprob, const int32_t *seq_offsets,
                       int S, float tis_cap_c, float *delta, float *seq_w, float *seq_w_clipped, void *ws,
                       size_t ws_bytes, void *stream)
{
    if (T < 0 || H <= 0 || V <= 0) {
        set_error("qarl_token_logprob: T >= 0, H > 0, V > 0 required");
        return QARL_ERR_INVALID_ARG;
    }
    if (T == 0) return QARL_OK;
    if (!(inv_temperature > 0.f) || inv_temperature > 3.0e38f) {
        set_error("qarl_token_logprob: inv_temperature must be positive and finite (got %g)", (double)inv_temperature);
        return QARL_ERR_INVALID_ARG;
    }
    if (!h_bf16 || !w_lm_bf16 || !target || !logprob) {
        set_error("qarl_token_logprob: null pointer");
        return QARL_ERR_INVALID_ARG;
    }
    if (H % 64 != 0) {
        set_error("qarl_token_logprob: H %% 64 == 0 required (got %d)", H);
        return QARL_ERR_UNSUPPORTED;
    }
    if (!aligned16(h_bf16) || !aligned16(w_lm_bf16)) {
        set_error("qarl_token_logprob: h and w_lm must be 16-byte aligned");
        return QARL_ERR_ALIGNMENT;
    }
    const size_t need = qarl_logprob_workspace_bytes(T, H, V);
    if (need && (!ws || ws_bytes < need || !aligned16(ws))) {
        set_error("qarl_token_logprob: needs %zu bytes of 16-byte aligned workspace (got %zu)", need, ws_bytes);
        return QARL_ERR_WORKSPACE;
    }
    if ((delta || seq_w || seq_w_clipped) && !ref_logprob) {
        set_error("qarl_token_logprob: comparison outputs need ref_logprob");
        return QARL_ERR_INVALID_ARG;
    }
    int rc = launch_logprob(h_bf16, w_lm_bf16, target, T, H, V, inv_temperature, logprob, ws, (hipStream_t)stream);
    if (rc) return rc;
    if (ref_logprob && (delta || seq_w || seq_w_clipped))
        return qarl_logprob_mismatch(logprob, ref_logprob, T, seq_offsets, S, tis_cap_c, delta, nullptr, seq_w,
                                     seq_w_clipped, stream);
    return QARL_OK;
}

int qarl_token_logprob_static(const void *h_bf16, const void *w_lm_bf16, const int32_t *target, int T, int H, int V,
                              float inv_temperature, float *logprob, const float *ref_logprob,
                              const int32_t *seq_offsets, int S, float tis_cap_c, float *delta, float *seq_w,
                              float *seq_w_clipped, void *stream)
{
    if (T < 0 || H <= 0 || V <= 0) {
        set_error("qarl_token_logprob_static: T >= 0, H > 0, V > 0 required");
        return QARL_ERR_INVALID_ARG;
    }
    if (T == 0) return QARL_OK;
    const size_t need = qarl_logprob_workspace_bytes(T, H, V);
    if (need > kLogprobScratchBytes) {
        set_error("qarl_token_logprob_static: T=%d tokens over V=%d need %zu bytes of partial results, more than the "
                  "library's %zu bytes of built-in scratch; use qarl_token_logprob with a caller workspace",
                  T, V, need, (size_t)kLogprobScratchBytes);
        return QARL_ERR_WORKSPACE;
    }
    void *ws = nullptr;
    int rc = logprob_static_scratch(&ws);
    if (rc) return rc;
    return qarl_token_logprob(h_bf16, w_lm_bf16, target, T, H, V, inv_temperature, logprob, ref_logprob, seq_offsets,
                              S, tis_cap_c, delta, seq_w, seq_w_clipped, ws, kLogprobScratchBytes, stream);
}

size_t qarl_token_logprob_static_limit(void) { return kLogprobScratchBytes; }

}  // extern "C"
