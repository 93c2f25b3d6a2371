// Weighted combine of the expert outputs and the log-prob mismatch comparison:
// small bandwidth-bound kernels with fixed summation order.
#include "common.hpp"

namespace qarl {

// out[t][n] = sum_{slot} w[t][slot] * Y[t*topk + slot][n], slots in ascending order, fp32,
// rounded once.  Y is in pair order (the grouped GEMM scatters its rows there).
__global__ __launch_bounds__(256) void combine_kernel(const float *__restrict__ y, const float *__restrict__ w,
                                                      int T, int topk, int N, void *__restrict__ out, int out_f32)
{
    const int n4 = N / 4;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)T * n4) return;
    const int t = (int)(idx / n4), c4 = (int)(idx % n4);
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    // eight slots' loads go out together (the rows are read once: nontemporal), the sum stays in slot order
    const float *yt = y + (int64_t)t * topk * N + c4 * 4;
    const float *wt = w + (int64_t)t * topk;
    for (int j0 = 0; j0 < topk; j0 += 8) {
        f32x4 v[8];
        float wj[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int jj = min(j0 + j, topk - 1);
            v[j] = __builtin_nontemporal_load((const f32x4 *)(yt + (int64_t)jj * N));
            wj[j] = wt[jj];
        }
#pragma unroll
        for (int j = 0; j < 8; ++j)
            if (j0 + j < topk) {
#pragma unroll
                for (int i = 0; i < 4; ++i) acc[i] = fmaf(wj[j], v[j][i], acc[i]);
            }
    }
    if (out_f32) {
        *(f32x4 *)((float *)out + (int64_t)t * N + c4 * 4) = acc;
    } else {
        u32x2 o;
        o[0] = f32_to_bf16_bits(acc[0]) | (f32_to_bf16_bits(acc[1]) << 16);
        o[1] = f32_to_bf16_bits(acc[2]) | (f32_to_bf16_bits(acc[3]) << 16);
        *(u32x2 *)((uint16_t *)out + (int64_t)t * N + c4 * 4) = o;
    }
}

int launch_combine(const float *y, const float *w, int T, int topk, int N, void *out, int out_f32, hipStream_t s)
{
    if (T == 0) return QARL_OK;
    const int64_t n = (int64_t)T * (N / 4);
    combine_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s>>>(y, w, T, topk, N, out, out_f32);
    return check_hip(hipGetLastError(), "combine_kernel");
}

// delta = lp_a - lp_b, w = exp(delta) per token (eq. (3) in log space); per sequence the
// geometric-mean weight exp(mean delta) and its two-sided cap (section 3.2).  One workgroup
// per sequence; the mean is a fixed-order tree so results do not depend on timing.
__global__ __launch_bounds__(256) void mismatch_kernel(const float *__restrict__ a, const float *__restrict__ b,
                                                       const int32_t *__restrict__ seq_offsets, float c,
                                                       float *__restrict__ delta, float *__restrict__ token_w,
                                                       float *__restrict__ seq_w, float *__restrict__ seq_wc)
{
    __shared__ double part[256];
    const int s = blockIdx.x;
    const int lo = seq_offsets[s], hi = seq_offsets[s + 1];
    double acc = 0.0;
    for (int t = lo + threadIdx.x; t < hi; t += 256) {
        const float d = a[t] - b[t];
        if (delta) delta[t] = d;
        if (token_w) token_w[t] = expf(d);
        acc += (double)d;
    }
    part[threadIdx.x] = acc;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if (threadIdx.x < o) part[threadIdx.x] += part[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        const float mean = (hi > lo) ? (float)(part[0] / (double)(hi - lo)) : 0.f;
        if (seq_w) seq_w[s] = expf(mean);
        if (seq_wc) {
            const float lc = logf(c);
            seq_wc[s] = expf(fminf(fmaxf(mean, -lc), lc));
        }
    }
}

__global__ __launch_bounds__(256) void mismatch_tokens_kernel(const float *__restrict__ a, const float *__restrict__ b,
                                                              int T, float *__restrict__ delta,
                                                              float *__restrict__ token_w)
{
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t >= T) return;
    const float d = a[t] - b[t];
    if (delta) delta[t] = d;
    if (token_w) token_w[t] = expf(d);
}

int launch_mismatch(const float *lp_a, const float *lp_b, int T, const int32_t *seq_offsets, int S, float c,
                    float *delta, float *token_w, float *seq_w, float *seq_wc, hipStream_t s)
{
    if (seq_offsets && S > 0) {
        // tokens outside every sequence are not touched by the per-sequence kernel, so cover all first
        if ((delta || token_w) && T > 0) {
            mismatch_tokens_kernel<<<dim3((T + 255) / 256), dim3(256), 0, s>>>(lp_a, lp_b, T, delta, token_w);
            int rc = check_hip(hipGetLastError(), "mismatch_tokens_kernel");
            if (rc) return rc;
        }
        mismatch_kernel<<<dim3(S), dim3(256), 0, s>>>(lp_a, lp_b, seq_offsets, c, nullptr, nullptr, seq_w, seq_wc);
        return check_hip(hipGetLastError(), "mismatch_kernel");
    }
    if ((delta || token_w) && T > 0) {
        mismatch_tokens_kernel<<<dim3((T + 255) / 256), dim3(256), 0, s>>>(lp_a, lp_b, T, delta, token_w);
        return check_hip(hipGetLastError(), "mismatch_tokens_kernel");
    }
    return QARL_OK;
}

}  // namespace qarl
