// LM head fused with the per-token log-prob: logits z = inv_T * h W^T are formed tile by
// tile in fp32 MFMA accumulators and reduced on the spot to (row max, row sum of
// exp(z - max)) per 256-column block plus the target logit; a second small kernel merges the
// blocks: logprob = z_target - (m + log sum).  The [T][V] logits never reach memory.
// This is the learner-forward half of the comparison in eq. (3).
#include "common.hpp"

namespace qarl {

constexpr int kLThreads = 512;
constexpr int kLBM = 128;
constexpr int kLBN = 256;
constexpr int kLKS = 64;                  // k per step
constexpr int kLStride = kLKS * 2 + 16;   // LDS bytes per activation row

struct LogprobParams {
    const uint16_t *h;
    const uint16_t *w;
    const int32_t *target;
    float *pmax, *psum, *tgt;  // [n_blocks][T], [n_blocks][T], [T]
    int T, H, V, n_blocks, m_tiles, total;
    float inv_temp;
};

__global__ __launch_bounds__(kLThreads, 1) void lmhead_lse_kernel(LogprobParams p)
{
    __shared__ __attribute__((aligned(16))) unsigned char xs_all[2 * kLBM * kLStride];
    __shared__ float s_m[4][kLBM], s_s[4][kLBM];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 2, wn = wave & 3;
    const int c = lane & 31, h = lane >> 5;

    // consecutive workgroup ids go round-robin over the 8 XCDs: hand each XCD a contiguous range of
    // tiles, token tiles fastest, so the token tiles that share a block of W_lm share an L2.
    const int per_xcd = p.total / 8;
    const int v = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
    const int mt = v % p.m_tiles, nb = v / p.m_tiles;
    if (nb >= p.n_blocks) return;

    const int T = p.T, H = p.H, V = p.V;
    const int row0 = mt * kLBM;
    int col[2];
    col[0] = nb * kLBN + wn * 64 + c;
    col[1] = col[0] + 32;
    const bool col_ok[2] = {col[0] < V, col[1] < V};
    const u32x4 *wrow[2];
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) wrow[nt] = (const u32x4 *)(p.w + (int64_t)(col_ok[nt] ? col[nt] : 0) * H);

    u32x4 ar[2];
    auto load_a = [&](int ks) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int idx = u * kLThreads + tid;
            const int r = idx >> 3, b = idx & 7;
            ar[u] = u32x4{0, 0, 0, 0};
            if (row0 + r < T) ar[u] = *(const u32x4 *)(p.h + (int64_t)(row0 + r) * H + ks * kLKS + b * 8);
        }
    };
    auto store_a = [&](int buf) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int idx = u * kLThreads + tid;
            const int r = idx >> 3, b = idx & 7;
            *(u32x4 *)(xs_all + buf * kLBM * kLStride + r * kLStride + b * 16) = ar[u];
        }
    };
    struct BRegs {
        u32x4 w[2][4];
    };
    auto load_b = [&](BRegs &dst, int ks) {
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                dst.w[nt][j] = u32x4{0, 0, 0, 0};
                if (col_ok[nt]) dst.w[nt][j] = wrow[nt][ks * (kLKS / 8) + h * 4 + j];
            }
    };

    f32x16 acc[2][2];
#pragma unroll
    for (int ms = 0; ms < 2; ++ms)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[ms][nt][i] = 0.f;

    const int steps = H / kLKS;
    BRegs bcur, bnxt;
    load_a(0);
    load_b(bcur, 0);
    store_a(0);
    lds_barrier();
    for (int ks = 0; ks < steps; ++ks) {
        if (ks + 1 < steps) {
            load_a(ks + 1);
            load_b(bnxt, ks + 1);
        }
        const unsigned char *xs = xs_all + (ks & 1) * kLBM * kLStride;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const bf16x8 b0 = __builtin_bit_cast(bf16x8, bcur.w[0][j]);
            const bf16x8 b1 = __builtin_bit_cast(bf16x8, bcur.w[1][j]);
#pragma unroll
            for (int ms = 0; ms < 2; ++ms) {
                const bf16x8 a = *(const bf16x8 *)(xs + (wm * 64 + ms * 32 + c) * kLStride + (h * 32 + j * 8) * 2);
                acc[ms][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b0, acc[ms][0], 0, 0, 0);
                acc[ms][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b1, acc[ms][1], 0, 0, 0);
            }
        }
        if (ks + 1 < steps) {
            store_a((ks + 1) & 1);
            bcur = bnxt;
        }
        lds_barrier();
    }

    // ---- per-row (max, sum exp) over this workgroup's 256 columns, and the target logit
#pragma unroll
    for (int ms = 0; ms < 2; ++ms) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int r = wm * 64 + ms * 32 + 8 * (i >> 2) + 4 * h + (i & 3);
            const float z0 = col_ok[0] ? acc[ms][0][i] * p.inv_temp : -INFINITY;
            const float z1 = col_ok[1] ? acc[ms][1][i] * p.inv_temp : -INFINITY;
            if (row0 + r < T) {
                const int y = p.target[row0 + r];
                if (y == col[0]) p.tgt[row0 + r] = z0;
                if (y == col[1]) p.tgt[row0 + r] = z1;
            }
            float m = fmaxf(z0, z1);
#pragma unroll
            for (int o = 1; o < 32; o <<= 1) m = fmaxf(m, __shfl_xor(m, o, 64));
            float s = 0.f;
            if (m > -INFINITY) s = expf(z0 - m) + expf(z1 - m);
#pragma unroll
            for (int o = 1; o < 32; o <<= 1) s += __shfl_xor(s, o, 64);
            if (c == 0) {
                s_m[wn][r] = m;
                s_s[wn][r] = s;
            }
        }
    }
    lds_barrier();
    if (tid < kLBM && row0 + tid < T) {
        float m = fmaxf(fmaxf(s_m[0][tid], s_m[1][tid]), fmaxf(s_m[2][tid], s_m[3][tid]));
        float s = 0.f;
#pragma unroll
        for (int w4 = 0; w4 < 4; ++w4)
            if (s_m[w4][tid] > -INFINITY) s += s_s[w4][tid] * expf(s_m[w4][tid] - m);
        p.pmax[(int64_t)nb * T + row0 + tid] = m;
        p.psum[(int64_t)nb * T + row0 + tid] = s;
    }
}

// Merge the per-block partials of one token (fixed order) and emit the log-prob.
__global__ __launch_bounds__(256) void lse_finalize_kernel(const float *__restrict__ pmax,
                                                           const float *__restrict__ psum,
                                                           const float *__restrict__ tgt, int T, int n_blocks,
                                                           float *__restrict__ logprob)
{
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t >= T) return;
    float m = -INFINITY;
    for (int b = 0; b < n_blocks; ++b) m = fmaxf(m, pmax[(int64_t)b * T + t]);
    double s = 0.0;
    for (int b = 0; b < n_blocks; ++b) s += (double)psum[(int64_t)b * T + t] * (double)expf(pmax[(int64_t)b * T + t] - m);
    logprob[t] = tgt[t] - (m + (float)log(s));
}

size_t logprob_ws_bytes(int T, int H, int V)
{
    (void)H;
    const size_t nb = (size_t)(V + kLBN - 1) / kLBN;
    return (2 * nb + 1) * (size_t)T * sizeof(float);
}

int launch_logprob(const void *h, const void *wlm, const int32_t *target, int T, int H, int V, float inv_temp,
                   float *logprob, void *ws, hipStream_t s)
{
    LogprobParams p;
    p.h = (const uint16_t *)h;
    p.w = (const uint16_t *)wlm;
    p.target = target;
    p.T = T;
    p.H = H;
    p.V = V;
    p.n_blocks = (V + kLBN - 1) / kLBN;
    p.m_tiles = (T + kLBM - 1) / kLBM;
    p.pmax = (float *)ws;
    p.psum = p.pmax + (size_t)p.n_blocks * T;
    p.tgt = p.psum + (size_t)p.n_blocks * T;
    p.inv_temp = inv_temp;
    const int64_t total = (((int64_t)p.n_blocks * p.m_tiles + 7) / 8) * 8;
    if (total > 0x7fffffffLL) {
        set_error("logprob: grid too large");
        return QARL_ERR_UNSUPPORTED;
    }
    p.total = (int)total;
    lmhead_lse_kernel<<<dim3((unsigned)total), dim3(kLThreads), 0, s>>>(p);
    int rc = check_hip(hipGetLastError(), "lmhead_lse_kernel");
    if (rc) return rc;
    lse_finalize_kernel<<<dim3((T + 255) / 256), dim3(256), 0, s>>>(p.pmax, p.psum, p.tgt, T, p.n_blocks, logprob);
    return check_hip(hipGetLastError(), "lse_finalize_kernel");
}

}  // namespace qarl
