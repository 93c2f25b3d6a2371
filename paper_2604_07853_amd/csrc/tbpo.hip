// Sequence-level surrogate of section 3.2 ("Sequence Level Objectives"; ratio and weight as in the appendix
// figure "Sequence ratio and weight definition") on three log-prob streams: a response is one action whose
// probability is the geometric mean of its token probabilities, so
//     r  = exp(mean_t (lp_current - lp_old)),   w~ = exp(clip(mean_t (lp_old - lp_sampler), -log c, log c)),
//     r~ = clip(r, band of the advantage's sign),   objective of the response = w~ r~ A,
// J = mean over the responses that have tokens, and grad[t] = dJ / d lp_current[t] with w~ held constant:
// in_band * w~ * A * r / (L * S').  Two small kernels, fixed summation order (results do not depend on timing).
#include "common.hpp"

namespace qarl {

constexpr int kTbpoThreads = 256;

struct TbpoParams {
    const float *lp_cur, *lp_old, *lp_smp;
    const int32_t *seq_offsets;
    const float *adv;
    int S;
    float eps_low, eps_high, delta_low, delta_high, log_c;
    float *r_seq, *w_clip, *r_clip;
    int32_t *in_band;
    float *obj_seq;      // [S], always written (the second kernel reads it)
    float *objective;    // [1]
    float *grad;         // [T] or null
};

// Sum over the workgroup in a fixed tree order; every thread gets the result.
__device__ __forceinline__ double block_sum(double v, double *part)
{
    part[threadIdx.x] = v;
    __syncthreads();
    for (int o = kTbpoThreads / 2; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) part[threadIdx.x] += part[threadIdx.x + o];
        __syncthreads();
    }
    const double r = part[0];
    __syncthreads();
    return r;
}

// One workgroup per response: the two means, ratio, capped weight, band, objective of the response.
__global__ __launch_bounds__(kTbpoThreads) void tbpo_seq_kernel(TbpoParams p)
{
    __shared__ double part[kTbpoThreads];
    const int s = blockIdx.x;
    const int lo = p.seq_offsets[s], hi = p.seq_offsets[s + 1];
    double ar = 0.0, aw = 0.0;
    for (int t = lo + (int)threadIdx.x; t < hi; t += kTbpoThreads) {
        const float o = p.lp_old[t];
        ar += (double)(p.lp_cur[t] - o);
        aw += (double)(o - p.lp_smp[t]);
    }
    const double sr = block_sum(ar, part), sw = block_sum(aw, part);
    if (threadIdx.x != 0) return;
    float r = 1.f, wt = 1.f, rt = 1.f, obj = 0.f;
    int inside = 1;
    if (hi > lo) {
        const double L = (double)(hi - lo);
        r = expf((float)(sr / L));
        wt = expf(fminf(fmaxf((float)(sw / L), -p.log_c), p.log_c));
        const float a = p.adv[s];
        const float lower = a >= 0.f ? 1.f - p.eps_low : 1.f - p.delta_low;
        const float upper = a >= 0.f ? 1.f + p.eps_high : 1.f + p.delta_high;
        inside = (r >= lower) && (r <= upper);
        rt = inside ? r : (r < lower ? lower : upper);
        obj = wt * rt * a;
    }
    if (p.r_seq) p.r_seq[s] = r;
    if (p.w_clip) p.w_clip[s] = wt;
    if (p.r_clip) p.r_clip[s] = rt;
    if (p.in_band) p.in_band[s] = inside;
    p.obj_seq[s] = obj;
}

// One workgroup per response again: every workgroup counts the responses that have tokens (S / 256 steps),
// the first one also sums the objectives; then the gradient of the workgroup's own tokens.
__global__ __launch_bounds__(kTbpoThreads) void tbpo_grad_kernel(TbpoParams p)
{
    __shared__ double part[kTbpoThreads];
    const int s = blockIdx.x;
    double cnt = 0.0, tot = 0.0;
    for (int i = (int)threadIdx.x; i < p.S; i += kTbpoThreads) {
        const bool has = p.seq_offsets[i + 1] > p.seq_offsets[i];
        cnt += has ? 1.0 : 0.0;
        if (s == 0 && has) tot += (double)p.obj_seq[i];
    }
    const double n = block_sum(cnt, part);
    if (s == 0) {
        const double j = block_sum(tot, part);
        if (threadIdx.x == 0) p.objective[0] = n > 0.0 ? (float)(j / n) : 0.f;
    }
    if (!p.grad) return;
    const int lo = p.seq_offsets[s], hi = p.seq_offsets[s + 1];
    if (hi <= lo) return;
    // the response's statistics again, from what the first kernel stored or recomputed the same way
    const float a = p.adv[s];
    const float lower = a >= 0.f ? 1.f - p.eps_low : 1.f - p.delta_low;
    const float upper = a >= 0.f ? 1.f + p.eps_high : 1.f + p.delta_high;
    double ar = 0.0, aw = 0.0;
    for (int t = lo + (int)threadIdx.x; t < hi; t += kTbpoThreads) {
        const float o = p.lp_old[t];
        ar += (double)(p.lp_cur[t] - o);
        aw += (double)(o - p.lp_smp[t]);
    }
    const double sr = block_sum(ar, part), sw = block_sum(aw, part);
    const double L = (double)(hi - lo);
    const float r = expf((float)(sr / L));
    const float wt = expf(fminf(fmaxf((float)(sw / L), -p.log_c), p.log_c));
    const bool inside = (r >= lower) && (r <= upper);
    const float g = inside ? (float)((double)(wt * a * r) / (L * n)) : 0.f;
    for (int t = lo + (int)threadIdx.x; t < hi; t += kTbpoThreads) p.grad[t] = g;
}

__global__ void fill_f32_kernel(float *p, int n, float v)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = v;
}

int launch_fill_f32(float *p, int n, float v, hipStream_t s)
{
    if (n <= 0) return QARL_OK;
    fill_f32_kernel<<<dim3((n + 255) / 256), dim3(256), 0, s>>>(p, n, v);
    return check_hip(hipGetLastError(), "fill_f32_kernel");
}

int launch_tbpo(const float *lp_cur, const float *lp_old, const float *lp_smp, const int32_t *seq_offsets, int S,
                const float *adv, float eps_low, float eps_high, float delta_low, float delta_high, float c,
                float *r_seq, float *w_clip, float *r_clip, int32_t *in_band, float *obj_seq, float *objective,
                float *grad, hipStream_t s)
{
    TbpoParams p;
    p.lp_cur = lp_cur;
    p.lp_old = lp_old;
    p.lp_smp = lp_smp;
    p.seq_offsets = seq_offsets;
    p.adv = adv;
    p.S = S;
    p.eps_low = eps_low;
    p.eps_high = eps_high;
    p.delta_low = delta_low;
    p.delta_high = delta_high;
    p.log_c = logf(c);
    p.r_seq = r_seq;
    p.w_clip = w_clip;
    p.r_clip = r_clip;
    p.in_band = in_band;
    p.obj_seq = obj_seq;
    p.objective = objective;
    p.grad = grad;
    tbpo_seq_kernel<<<dim3((unsigned)S), dim3(kTbpoThreads), 0, s>>>(p);
    int rc = check_hip(hipGetLastError(), "tbpo_seq_kernel");
    if (rc) return rc;
    tbpo_grad_kernel<<<dim3((unsigned)S), dim3(kTbpoThreads), 0, s>>>(p);
    return check_hip(hipGetLastError(), "tbpo_grad_kernel");
}

}  // namespace qarl
