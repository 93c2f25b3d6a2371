// MoE router: fp32 softmax over bf16 logits, exact top-k by (logit desc, expert id asc),
// renormalised weights, then a stable grouping of the (token, slot) pairs by expert.
// One wavefront owns one token: E <= 256 logits sit 1..4 per lane, the arg-max of every
// round is a 6-step shuffle reduction on an integer key, so equal bf16 logits resolve to
// the lower expert id exactly as a full stable sort would.
#include "common.hpp"

namespace qarl {

constexpr int kRouteThreads = 256;
constexpr int kMaxPerLane = 4;  // E <= 256

// Order-preserving integer image of a bf16 pattern (-0 counted as +0), high half of the key;
// low half = 0xffff - expert id so that the lower id wins among equal logits.
__device__ __forceinline__ uint32_t sort_key(uint32_t h, int id)
{
    if (h == 0x8000u) h = 0;
    uint32_t k = (h & 0x8000u) ? (~h & 0xffffu) : (h | 0x8000u);
    return (k << 16) | (0xffffu - (uint32_t)id);
}

// Wavefront reductions on the data-parallel-primitive path (row shifts inside 16-lane rows, then two
// row broadcasts); the result is read from lane 63 into a scalar, so it is uniform.  `ident` fills the
// lanes a shift has no source for.
#define QARL_DPP_STEP(T, OP, CTRL, ROWMASK)                                                                   \
    v = OP(v, (T)__builtin_bit_cast(T, __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, ident),             \
                                                                   __builtin_bit_cast(int, v), CTRL, ROWMASK, 0xf, false)))
__device__ __forceinline__ uint32_t umax2(uint32_t a, uint32_t b) { return a > b ? a : b; }
__device__ __forceinline__ float fadd2(float a, float b) { return a + b; }
__device__ __forceinline__ uint32_t wave_max_u32_dpp(uint32_t v)
{
    const uint32_t ident = 0;
    QARL_DPP_STEP(uint32_t, umax2, 0x111, 0xf);  // row_shr:1
    QARL_DPP_STEP(uint32_t, umax2, 0x112, 0xf);  // row_shr:2
    QARL_DPP_STEP(uint32_t, umax2, 0x114, 0xf);  // row_shr:4
    QARL_DPP_STEP(uint32_t, umax2, 0x118, 0xf);  // row_shr:8
    QARL_DPP_STEP(uint32_t, umax2, 0x142, 0xa);  // row_bcast:15 into rows 1 and 3
    QARL_DPP_STEP(uint32_t, umax2, 0x143, 0xc);  // row_bcast:31 into rows 2 and 3
    return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}
__device__ __forceinline__ float wave_max_f32_dpp(float v)
{
    const float ident = -INFINITY;
    QARL_DPP_STEP(float, fmaxf, 0x111, 0xf);
    QARL_DPP_STEP(float, fmaxf, 0x112, 0xf);
    QARL_DPP_STEP(float, fmaxf, 0x114, 0xf);
    QARL_DPP_STEP(float, fmaxf, 0x118, 0xf);
    QARL_DPP_STEP(float, fmaxf, 0x142, 0xa);
    QARL_DPP_STEP(float, fmaxf, 0x143, 0xc);
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}
// Sum in the fixed order the shifts imply; every lane gets the same value.
__device__ __forceinline__ float wave_sum_f32_dpp(float v)
{
    const float ident = 0.f;
    QARL_DPP_STEP(float, fadd2, 0x111, 0xf);
    QARL_DPP_STEP(float, fadd2, 0x112, 0xf);
    QARL_DPP_STEP(float, fadd2, 0x114, 0xf);
    QARL_DPP_STEP(float, fadd2, 0x118, 0xf);
    QARL_DPP_STEP(float, fadd2, 0x142, 0xa);
    QARL_DPP_STEP(float, fadd2, 0x143, 0xc);
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}
#undef QARL_DPP_STEP

__global__ __launch_bounds__(kRouteThreads) void route_topk_kernel(const uint16_t *__restrict__ logits, int T,
                                                                  int E, int topk, int renorm,
                                                                  int32_t *__restrict__ ids,
                                                                  float *__restrict__ wts,
                                                                  int32_t *__restrict__ counts,
                                                                  int32_t *__restrict__ zero_me, int n_zero)
{
    // large batches: the per-expert counters the counting kernel behind this one adds to start at zero (saves a launch)
    if (blockIdx.x == 0 && (int)threadIdx.x < n_zero) zero_me[threadIdx.x] = 0;
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * (kRouteThreads / 64) + (threadIdx.x >> 6);
    if (t >= T) return;
    const int per = E / 64;
    uint32_t key[kMaxPerLane];
    float val[kMaxPerLane];
#pragma unroll
    for (int j = 0; j < kMaxPerLane; ++j) {
        key[j] = 0;
        val[j] = -INFINITY;
        if (j < per) {
            const int e = lane + 64 * j;
            const uint32_t h = logits[(int64_t)t * E + e];
            key[j] = sort_key(h, e);
            val[j] = bf16_bits_to_f32(h);
        }
    }
    float m = -INFINITY;
#pragma unroll
    for (int j = 0; j < kMaxPerLane; ++j) m = fmaxf(m, val[j]);
    m = wave_max_f32_dpp(m);
    float z = 0.f;
#pragma unroll
    for (int j = 0; j < kMaxPerLane; ++j)
        if (j < per) z += expf(val[j] - m);
    z = wave_sum_f32_dpp(z);

    int my_id = 0;      // lane r keeps the r-th winner
    float my_p = 0.f;
    float psum = 0.f;
    for (int r = 0; r < topk; ++r) {
        uint32_t best = 0;
#pragma unroll
        for (int j = 0; j < kMaxPerLane; ++j) best = max(best, key[j]);
        best = wave_max_u32_dpp(best);
        const int e = 0xffff - (int)(best & 0xffffu);
        // the owner retires the winner and publishes its logit
        float lv = 0.f;
#pragma unroll
        for (int j = 0; j < kMaxPerLane; ++j)
            if (key[j] == best) {
                lv = val[j];
                key[j] = 0;
            }
        lv = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, lv), e & 63));
        const float p = expf(lv - m) / z;
        psum += p;
        if (lane == r) {
            my_id = e;
            my_p = p;
        }
    }
    if (lane < topk) {
        ids[(int64_t)t * topk + lane] = my_id;
        wts[(int64_t)t * topk + lane] = renorm ? my_p / psum : my_p;
        if (counts) atomicAdd(&counts[my_id], 1);
    }
}

__global__ void zero_i32_kernel(int32_t *p, int n)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

// Per-expert pair counts for large batches: every workgroup histograms its share of the ids in LDS and adds
// its E partial counts to the global ones, so a popular expert's counter sees one add per workgroup instead
// of one per routed token.
constexpr int kCountThreads = 1024;
constexpr int kCountBlocks = 64;

__global__ __launch_bounds__(kCountThreads) void count_experts_kernel(const int32_t *__restrict__ ids, int n_pairs,
                                                                     int E, int32_t *__restrict__ counts)
{
    __shared__ int s_hist[256];
    if (threadIdx.x < 256) s_hist[threadIdx.x] = 0;
    __syncthreads();
    for (int i = blockIdx.x * kCountThreads + threadIdx.x; i < n_pairs; i += kCountBlocks * kCountThreads)
        atomicAdd(&s_hist[ids[i]], 1);
    __syncthreads();
    if (threadIdx.x < E && s_hist[threadIdx.x] != 0) atomicAdd(&counts[threadIdx.x], s_hist[threadIdx.x]);
}

// One workgroup per expert: its offset is the sum of the counts before it; it then compacts the pairs routed
// to it in ascending pair order, which keeps (t, slot) order.  Every wavefront owns one contiguous range of the
// pairs and walks it 256 pairs at a time (4 consecutive pairs per lane, coalesced), once to count its hits and,
// after the only barrier (an exclusive scan of the 16 wavefront totals), once more to place them: inside the
// loop a wavefront-level prefix sum is all that is needed.  The ids are read twice; the second read hits cache.
constexpr int kGroupThreads = 1024;
constexpr int kGroupWaves = kGroupThreads / 64;
constexpr int kGroupStep = 256;   // pairs per wavefront and step

__global__ __launch_bounds__(kGroupThreads) void group_by_expert_kernel(const int32_t *__restrict__ ids,
                                                                       int n_pairs, int E, int topk,
                                                                       const int32_t *__restrict__ counts,
                                                                       int32_t *__restrict__ offsets,
                                                                       int32_t *__restrict__ pairs,
                                                                       int32_t *__restrict__ tokens, int ids_aligned)
{
    __shared__ int s_wave[kGroupWaves];
    __shared__ int s_base;
    const int e = blockIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    // exclusive offset of this expert
    int part = 0;
    for (int i = threadIdx.x; i < e; i += kGroupThreads) part += counts[i];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) part += __shfl_xor(part, o, 64);
    if (lane == 0) s_wave[wave] = part;
    __syncthreads();
    if (threadIdx.x == 0) {
        int b = 0;
        for (int i = 0; i < kGroupWaves; ++i) b += s_wave[i];
        s_base = b;
        offsets[e] = b;
        if (e == E - 1) offsets[E] = b + counts[e];
    }
    // this wavefront's range of pairs: a multiple of the step, so every 16-byte load is aligned
    const int steps = (n_pairs + kGroupWaves * kGroupStep - 1) / (kGroupWaves * kGroupStep);
    const int lo = wave * steps * kGroupStep;
    const int hi = min(n_pairs, lo + steps * kGroupStep);
    auto hits_of = [&](int p) -> uint32_t {   // bit j set: pair p + j goes to this expert
        uint32_t h = 0;
        if (ids_aligned && p + 3 < n_pairs) {
            const i32x4 v = *(const i32x4 *)(ids + p);
#pragma unroll
            for (int j = 0; j < 4; ++j) h |= (v[j] == e) ? (1u << j) : 0u;
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) h |= (p + j < n_pairs && ids[p + j] == e) ? (1u << j) : 0u;
        }
        return h;
    };
    int cnt = 0;
    for (int p0 = lo; p0 < hi; p0 += kGroupStep) cnt += __popc(hits_of(p0 + lane * 4));
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) cnt += __shfl_xor(cnt, o, 64);
    __syncthreads();   // s_base is written, the offset pass is done with s_wave
    if (lane == 0) s_wave[wave] = cnt;
    __syncthreads();
    int running = s_base;
    for (int i = 0; i < wave; ++i) running += s_wave[i];
    for (int p0 = lo; p0 < hi; p0 += kGroupStep) {
        const int p = p0 + lane * 4;
        uint32_t h = hits_of(p);
        const int c = __popc(h);
        int incl = c;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int v = __shfl_up(incl, o, 64);
            if (lane >= o) incl += v;
        }
        int pos = running + incl - c;
        for (; h; h &= h - 1) {
            const int pj = p + __builtin_ctz(h);
            pairs[pos] = pj;
            tokens[pos] = pj / topk;
            ++pos;
        }
        running += __shfl(incl, 63, 64);
    }
}

// Grouping for small batches (decode) by ONE workgroup, with no zeroing pass and no global atomics.
// A token selects an expert at most once, so the pairs of an expert are ordered by token alone: the
// workgroup builds a bit matrix B[expert][token] in LDS (atomic OR, order-free), prefix pop-counts per
// 32-token word give every word's start inside its expert, a scan over the experts gives the offsets, and
// a pair (t, slot) of expert e lands at offsets[e] + start[e][t / 32] + popcount(B[e][t / 32] below bit t):
// the same stable order (expert, token, slot) the large-batch kernels produce.
constexpr int kSmallThreads = 1024;
constexpr int kSmallMaxT = 512;
constexpr int kSmallWords = kSmallMaxT / 32;
constexpr int kSmallMaxPairs = 4096;

__global__ __launch_bounds__(kSmallThreads) void group_small_kernel(const int32_t *__restrict__ ids, int T, int E,
                                                                   int topk, int32_t *__restrict__ counts,
                                                                   int32_t *__restrict__ offsets,
                                                                   int32_t *__restrict__ pairs,
                                                                   int32_t *__restrict__ tokens)
{
    __shared__ uint32_t s_bits[256 * kSmallWords];
    __shared__ uint16_t s_start[256 * kSmallWords];
    __shared__ int s_off[257];
    const int tid = threadIdx.x, lane = tid & 63;
    const int n_pairs = T * topk, words = (T + 31) / 32;
    for (int i = tid; i < E * words; i += kSmallThreads) s_bits[i] = 0;
    __syncthreads();
    constexpr int kMine = kSmallMaxPairs / kSmallThreads;
    int my_e[kMine];
#pragma unroll
    for (int u = 0; u < kMine; ++u) {
        const int pidx = tid + u * kSmallThreads;
        my_e[u] = -1;
        if (pidx < n_pairs) {
            const int e = ids[pidx], t = pidx / topk;
            my_e[u] = e;
            atomicOr(&s_bits[e * words + (t >> 5)], 1u << (t & 31));
        }
    }
    __syncthreads();
    if (tid < E) {
        int run = 0;
        for (int w = 0; w < words; ++w) {
            s_start[tid * words + w] = (uint16_t)run;
            run += __popc(s_bits[tid * words + w]);
        }
        counts[tid] = run;
        s_off[tid + 1] = run;
    }
    if (tid == 0) s_off[0] = 0;
    __syncthreads();
    if (tid < 64) {   // inclusive scan of the counts over the experts, four per lane
        int v[4], sum = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            v[j] = (lane * 4 + j < E) ? s_off[lane * 4 + j + 1] : 0;
            sum += v[j];
        }
        int incl = sum;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int up = __shfl_up(incl, o, 64);
            if (lane >= o) incl += up;
        }
        int run = incl - sum;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            run += v[j];
            if (lane * 4 + j < E) s_off[lane * 4 + j + 1] = run;
        }
    }
    __syncthreads();
    if (tid <= E) offsets[tid] = s_off[tid];
#pragma unroll
    for (int u = 0; u < kMine; ++u) {
        const int pidx = tid + u * kSmallThreads;
        const int e = my_e[u];
        if (e >= 0) {
            const int t = pidx / topk;
            const uint32_t below = s_bits[e * words + (t >> 5)] & ((1u << (t & 31)) - 1u);
            const int pos = s_off[e] + s_start[e * words + (t >> 5)] + __popc(below);
            pairs[pos] = pidx;
            tokens[pos] = t;
        }
    }
}

int launch_route_only(const void *logits, int T, int E, int topk, int renorm, int32_t *ids, float *w, hipStream_t s)
{
    const int per_block = kRouteThreads / 64;
    route_topk_kernel<<<dim3((T + per_block - 1) / per_block), dim3(kRouteThreads), 0, s>>>(
        (const uint16_t *)logits, T, E, topk, renorm, ids, w, nullptr, nullptr, 0);
    return check_hip(hipGetLastError(), "route_topk_kernel");
}

int launch_route(const void *logits, int T, int E, int topk, int renorm, int32_t *ids, float *w,
                 int32_t *counts, int32_t *offsets, int32_t *pairs, int32_t *tokens, hipStream_t s)
{
    const int per_block = kRouteThreads / 64;
    const int64_t n_pairs = (int64_t)T * topk;
    if (T > 0 && T <= kSmallMaxT && n_pairs <= kSmallMaxPairs) {
        route_topk_kernel<<<dim3((T + per_block - 1) / per_block), dim3(kRouteThreads), 0, s>>>(
            (const uint16_t *)logits, T, E, topk, renorm, ids, w, nullptr, nullptr, 0);
        int rc = check_hip(hipGetLastError(), "route_topk_kernel");
        if (rc) return rc;
        group_small_kernel<<<dim3(1), dim3(kSmallThreads), 0, s>>>(ids, T, E, topk, counts, offsets, pairs, tokens);
        return check_hip(hipGetLastError(), "group_small_kernel");
    }
    int rc;
    if (T == 0) {   // no router launch to zero the counters: the grouping below then writes counts = 0, offsets = 0
        zero_i32_kernel<<<dim3((E + 255) / 256), dim3(256), 0, s>>>(counts, E);
        rc = check_hip(hipGetLastError(), "zero_i32_kernel");
        if (rc) return rc;
    }
    if (T > 0) {
        static_assert(kRouteThreads >= 256, "the router's first workgroup zeroes up to 256 expert counters");
        route_topk_kernel<<<dim3((T + per_block - 1) / per_block), dim3(kRouteThreads), 0, s>>>(
            (const uint16_t *)logits, T, E, topk, renorm, ids, w, nullptr, counts, E);
        rc = check_hip(hipGetLastError(), "route_topk_kernel");
        if (rc) return rc;
        count_experts_kernel<<<dim3(kCountBlocks), dim3(kCountThreads), 0, s>>>(ids, (int)n_pairs, E, counts);
        rc = check_hip(hipGetLastError(), "count_experts_kernel");
        if (rc) return rc;
    }
    group_by_expert_kernel<<<dim3(E), dim3(kGroupThreads), 0, s>>>(ids, T * topk, E, topk, counts, offsets,
                                                                   pairs, tokens, ((uintptr_t)ids & 15) == 0);
    return check_hip(hipGetLastError(), "group_by_expert_kernel");
}

}  // namespace qarl
