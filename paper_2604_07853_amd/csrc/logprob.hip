// LM head fused with the per-token log-prob: logits z = inv_T * h W^T are formed tile by tile
// in fp32 MFMA accumulators and reduced on the spot to (max, sum of exp(z - max)) per token and
// 256-row block of the vocabulary; a second small kernel merges the blocks and subtracts from the
// target logit, which a third one computes as a plain dot product:
//     logprob = z_target - (m + log sum).
// The [T][V] logits never reach memory.  This is the learner-forward half of the comparison in
// eq. (3).
//
// The big kernel is a dense bf16 contraction, D^T = W_tile (256 vocab rows) x h_tile^T (256 tokens):
// vocabulary rows are the MFMA row operand, so that a lane ends up with 64 logits of ONE token per
// token tile and the max / sum-exp reduction runs down its own registers; only the two 32-lane halves
// and the two wavefronts that share a token meet through a shuffle and LDS.  Both operands reach LDS
// by asynchronous global -> LDS copies (no staging registers), two 64-k stages deep; 16-byte chunks of
// a row are XOR-swizzled with the row index so that the copies (8 rows x 128 bytes per wavefront
// instruction, coalesced) and the operand reads (32 rows, one chunk) are both free of bank conflicts.
// Operand reads run one 16-k slice ahead of the MFMAs, across the stage barrier as well.
#include "common.hpp"
#include <type_traits>

namespace qarl {

constexpr int kLThreads = 512;
constexpr int kLTile = 256;                 // vocabulary rows and tokens per workgroup
constexpr int kLKS = 64;                    // k per stage
constexpr int kLRowB = kLKS * 2;            // bytes per tile row and stage
constexpr int kLTileB = kLTile * kLRowB;    // one operand tile of one stage
constexpr int kLStageB = 2 * kLTileB;       // W tile, then h tile
constexpr int kLLds = 2 * kLStageB;         // two stages
constexpr int kLGroupM = 8, kLGroupN = 4;   // workgroups of one XCD that run together: 8 token x 4 vocab tiles

struct LogprobParams {
    const uint16_t *h;
    const uint16_t *w;
    float *pmax, *psum;  // [n_blocks][T]
    int T, H, V, n_blocks, m_tiles, n_mgroups;
    float inv_temp;
};

__global__ __launch_bounds__(kLThreads, 2) void lmhead_lse_kernel(LogprobParams p)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 2, wt = wave & 3;   // 128 vocabulary rows x 64 tokens per wavefront
    const int c = lane & 31, h = lane >> 5;

    // Consecutive workgroup ids go round-robin over the 8 XCDs.  The workgroups that run together on one
    // XCD (32 CUs, one workgroup each) form an 8-token-tile x 4-vocabulary-tile block, so that its L2
    // fetches 12 operand tiles for 32 output tiles.
    const int xcd = blockIdx.x % 8, idx = blockIdx.x / 8;
    const int super = (idx / (kLGroupM * kLGroupN)) * 8 + xcd, within = idx % (kLGroupM * kLGroupN);
    const int mt = (super % p.n_mgroups) * kLGroupM + within % kLGroupM;
    const int nb = (super / p.n_mgroups) * kLGroupN + within / kLGroupM;
    if (mt >= p.m_tiles || nb >= p.n_blocks) return;

    const int T = p.T, H = p.H, V = p.V;
    const int v0 = nb * kLTile, t0 = mt * kLTile;

    // ---- copies: a wavefront instruction moves 8 rows x 128 bytes; this wavefront owns rows
    // [32 wave, 32 wave + 32) of both tiles.  Chunk q of row r sits at r * 128 + (q ^ ((r >> 1) & 7)) * 16.
    uint32_t woff[4], hoff[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = wave * 32 + i * 8 + (lane >> 3);
        const int q = (lane & 7) ^ ((r >> 1) & 7);
        woff[i] = (uint32_t)min(r, V - 1 - v0) * (uint32_t)(H * 2) + q * 16;   // rows past V or T read the last
        hoff[i] = (uint32_t)min(r, T - 1 - t0) * (uint32_t)(H * 2) + q * 16;   // valid row: never used
    }
    const unsigned char *wbase = (const unsigned char *)p.w + (int64_t)v0 * H * 2;
    const unsigned char *hbase = (const unsigned char *)p.h + (int64_t)t0 * H * 2;
    // copy i of the wavefront's eight per stage (four W row groups, then four h row groups)
    auto copy_one = [&](int ks, int buf, int i) {
        unsigned char *dst = smem + buf * kLStageB + wave * 32 * kLRowB;
        if (i < 4) copy16_to_lds(wbase + (int64_t)ks * kLRowB + woff[i], dst + i * 8 * kLRowB);
        else copy16_to_lds(hbase + (int64_t)ks * kLRowB + hoff[i - 4], dst + kLTileB + (i - 4) * 8 * kLRowB);
    };
    auto copy_stage = [&](int ks, int buf) {
#pragma unroll
        for (int i = 0; i < 8; ++i) copy_one(ks, buf, i);
    };

    // ---- operand reads: lane (c,h) takes row c of a 32-row tile, k in [16 j + 8 h, +8) = chunk 2j + h
    int aoff[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) aoff[j] = c * kLRowB + (((2 * j + h) ^ ((c >> 1) & 7)) * 16);
    const int a_wave = wm * 128 * kLRowB, b_wave = kLTileB + wt * 64 * kLRowB;
    struct Frags {
        bf16x8 a[4], b[2];
    };
    f32x16 acc[4][2];
#pragma unroll
    for (int ms = 0; ms < 4; ++ms)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[ms][nt][i] = 0.f;
    auto mfma8 = [&](const Frags &f) {
#pragma unroll
        for (int ms = 0; ms < 4; ++ms)
#pragma unroll
            for (int nt = 0; nt < 2; ++nt)
                acc[ms][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[ms], f.b[nt], acc[ms][nt], 0, 0, 0);
    };
    // Slice j of a stage, in a fixed issue order: the eight MFMAs on `cur`; behind each of the first six, one of the
    // six operand reads of `nxt` (an LDS read every 32 cycles instead of six at once: 3 % faster than all six
    // behind the first MFMA); in slices 0 and 1, behind every second MFMA, one of the next stage's eight copies.
    // Measured at 16384 x 151936 x 2048: all eight at the top of the stage 9.0 ms (a wavefront that waits for room
    // in the memory pipeline is kept from its matrix instructions), two per slice 8.45, three-three-two 8.07,
    // four-four 7.86 (the later a copy goes out, the less of its latency the rest of the stage covers), one behind
    // each MFMA of slice 0 7.99.
    auto slice = [&](const Frags &cur, Frags &nxt, int ks, int j, auto more_t) {
        const int buf = ks & 1;
        const unsigned char *base = smem + buf * kLStageB + aoff[j];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int ms = i >> 1, nt = i & 1;
            acc[ms][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur.a[ms], cur.b[nt], acc[ms][nt], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            if (i < 4) nxt.a[i] = *(const bf16x8 *)(base + a_wave + i * 32 * kLRowB);
            else if (i < 6) nxt.b[i - 4] = *(const bf16x8 *)(base + b_wave + (i - 4) * 32 * kLRowB);
            if (decltype(more_t)::value && j < 2 && (i & 1)) copy_one(ks + 1, buf ^ 1, 4 * j + (i >> 1));
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    auto stage_barrier = [&]() {
        // own copies landed, own operand reads done; then everybody's
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    };

    // Rotated loop: the MFMAs of a stage's last slice run in the next trip, behind the stage barrier and
    // under the first operand reads of the next stage, so no operand read is outstanding at the back edge
    // and every wait inside the trip counts exactly the reads it needs.
    const int stages = H / kLKS;
    Frags last, f0, f1, f2, f3;
#pragma unroll
    for (int i = 0; i < 4; ++i) last.a[i] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int i = 0; i < 2; ++i) last.b[i] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
    copy_stage(0, 0);
    stage_barrier();
    // One stage; the last has no copies to issue, so the loop's last trip is peeled.
    auto stage = [&](int ks, auto more_t) {
        slice(last, f0, ks, 0, more_t);
        slice(f0, f1, ks, 1, more_t);
        slice(f1, f2, ks, 2, more_t);
        slice(f2, f3, ks, 3, more_t);
        stage_barrier();
        last = f3;
    };
    for (int ks = 0; ks + 1 < stages; ++ks) stage(ks, std::true_type{});
    stage(stages - 1, std::false_type{});
    mfma8(last);

    // ---- per token: max and sum of exp over this wavefront's 128 vocabulary rows.
    // lane (c,h), register i of acc[ms][nt] -> vocabulary row v0 + 128 wm + 32 ms + 8 (i/4) + 4 h + i%4,
    // token t0 + 64 wt + 32 nt + c.  exp(inv_T (a - m)) = exp2(k a - k m), k = inv_T log2 e > 0.
    float *s_m = (float *)smem, *s_s = s_m + 2 * kLTile;   // [wm][token] (the tiles are dead by now)
    const float k2 = p.inv_temp * 1.44269504088896340736f;
    const int vrow_lane = v0 + wm * 128 + 4 * h;
    const bool ragged = v0 + kLTile > V;
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
        if (ragged) {
#pragma unroll
            for (int ms = 0; ms < 4; ++ms)
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    if (vrow_lane + ms * 32 + 8 * (i >> 2) + (i & 3) >= V) acc[ms][nt][i] = -INFINITY;
        }
        float m = -INFINITY;
#pragma unroll
        for (int ms = 0; ms < 4; ++ms)
#pragma unroll
            for (int i = 0; i < 16; ++i) m = fmaxf(m, acc[ms][nt][i]);
        m = fmaxf(m, __shfl_xor(m, 32, 64));   // the other 64 rows of this token
        float s = 0.f;
        if (m > -INFINITY) {
            const float mk = m * k2;
#pragma unroll
            for (int ms = 0; ms < 4; ++ms)
#pragma unroll
                for (int i = 0; i < 16; ++i) s += __builtin_amdgcn_exp2f(fmaf(acc[ms][nt][i], k2, -mk));
        }
        s += __shfl_xor(s, 32, 64);
        if (h == 0) {
            s_m[wm * kLTile + wt * 64 + nt * 32 + c] = m;
            s_s[wm * kLTile + wt * 64 + nt * 32 + c] = s;
        }
    }
    lds_barrier();
    if (tid < kLTile && t0 + tid < T) {
        const float m0 = s_m[tid], m1 = s_m[kLTile + tid];
        const float m = fmaxf(m0, m1);
        float s = 0.f;
        if (m0 > -INFINITY) s += s_s[tid] * __builtin_amdgcn_exp2f((m0 - m) * k2);
        if (m1 > -INFINITY) s += s_s[kLTile + tid] * __builtin_amdgcn_exp2f((m1 - m) * k2);
        p.pmax[(int64_t)nb * T + t0 + tid] = m * p.inv_temp;
        p.psum[(int64_t)nb * T + t0 + tid] = s;
    }
}

// Target logit of each token: inv_T * <h_t, w_{y_t}> in fp32, one wavefront per token.  A target outside
// [0, V) yields NaN.
__global__ __launch_bounds__(256) void target_logit_kernel(const uint16_t *__restrict__ hmat,
                                                           const uint16_t *__restrict__ w,
                                                           const int32_t *__restrict__ target, int T, int H, int V,
                                                           float inv_temp, float *__restrict__ tgt)
{
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (t >= T) return;
    const int y = target[t];
    if (y < 0 || y >= V) {
        if (lane == 0) tgt[t] = __uint_as_float(0x7fc00000u);
        return;
    }
    const u32x4 *hr = (const u32x4 *)(hmat + (int64_t)t * H), *wr = (const u32x4 *)(w + (int64_t)y * H);
    float s = 0.f;
    for (int q = lane; q < H / 8; q += 64) {
        const u32x4 a = hr[q], b = wr[q];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            s = fmaf(__uint_as_float(a[i] << 16), __uint_as_float(b[i] << 16), s);
            s = fmaf(__uint_as_float(a[i] & 0xffff0000u), __uint_as_float(b[i] & 0xffff0000u), s);
        }
    }
    s = wave_sum(s);
    if (lane == 0) tgt[t] = s * inv_temp;
}

// Merge the per-block partials of one token and emit the log-prob.  16 tokens per workgroup; sixteen
// threads per token each fold every sixteenth block into a running (max, sum) (a chain of n_blocks / 16
// dependent steps: with four threads per token the launch took 88 us at 594 blocks), and the sixteen meet in
// LDS in a fixed order, so the result does not depend on scheduling.
constexpr int kFinTokens = 16, kFinSlices = 16;
__global__ __launch_bounds__(256) void lse_finalize_kernel(const float *__restrict__ pmax,
                                                           const float *__restrict__ psum,
                                                           const float *__restrict__ tgt, int T, int n_blocks,
                                                           float *__restrict__ logprob)
{
    __shared__ float s_m[kFinSlices][kFinTokens], s_s[kFinSlices][kFinTokens];
    const int tl = threadIdx.x % kFinTokens, slice = threadIdx.x / kFinTokens;
    const int t = blockIdx.x * kFinTokens + tl;
    float m = -INFINITY, s = 0.f;
    if (t < T) {
        for (int b = slice; b < n_blocks; b += kFinSlices) {
            const float mb = pmax[(int64_t)b * T + t], sb = psum[(int64_t)b * T + t];
            if (mb > m) {
                s = s * expf(m - mb) + sb;   // exp(-inf) = 0 on the first block
                m = mb;
            } else if (mb > -INFINITY) {
                s += sb * expf(mb - m);
            }
        }
    }
    s_m[slice][tl] = m;
    s_s[slice][tl] = s;
    __syncthreads();
    if (slice == 0 && t < T) {
        float mm = -INFINITY;
#pragma unroll
        for (int q = 0; q < kFinSlices; ++q) mm = fmaxf(mm, s_m[q][tl]);
        double ss = 0.0;
#pragma unroll
        for (int q = 0; q < kFinSlices; ++q)
            if (s_m[q][tl] > -INFINITY) ss += (double)s_s[q][tl] * (double)expf(s_m[q][tl] - mm);
        logprob[t] = tgt[t] - (mm + (float)log(ss));
    }
}

size_t logprob_ws_bytes(int T, int H, int V)
{
    (void)H;
    const size_t nb = (size_t)(V + kLTile - 1) / kLTile;
    return (2 * nb + 1) * (size_t)T * sizeof(float);
}

int launch_logprob(const void *h, const void *wlm, const int32_t *target, int T, int H, int V, float inv_temp,
                   float *logprob, void *ws, hipStream_t s)
{
    LogprobParams p;
    p.h = (const uint16_t *)h;
    p.w = (const uint16_t *)wlm;
    p.T = T;
    p.H = H;
    p.V = V;
    p.n_blocks = (V + kLTile - 1) / kLTile;
    p.m_tiles = (T + kLTile - 1) / kLTile;
    p.n_mgroups = (p.m_tiles + kLGroupM - 1) / kLGroupM;
    p.pmax = (float *)ws;
    p.psum = p.pmax + (size_t)p.n_blocks * T;
    float *tgt = p.psum + (size_t)p.n_blocks * T;
    p.inv_temp = inv_temp;
    if ((int64_t)kLTile * H * 2 >= (1LL << 31)) {
        set_error("logprob: H too large");
        return QARL_ERR_UNSUPPORTED;
    }
    const int64_t n_ngroups = (p.n_blocks + kLGroupN - 1) / kLGroupN;
    const int64_t supers = (((int64_t)p.n_mgroups * n_ngroups + 7) / 8) * 8;
    const int64_t grid = supers * kLGroupM * kLGroupN;
    if (grid > 0x7fffffffLL) {
        set_error("logprob: grid too large");
        return QARL_ERR_UNSUPPORTED;
    }
    static LdsLimitOnce once;
    if (int rc0 = raise_lds_limit((const void *)lmhead_lse_kernel, once, "hipFuncSetAttribute(lmhead)")) return rc0;
    target_logit_kernel<<<dim3((T + 3) / 4), dim3(256), 0, s>>>(p.h, p.w, target, T, H, V, inv_temp, tgt);
    int rc = check_hip(hipGetLastError(), "target_logit_kernel");
    if (rc) return rc;
    lmhead_lse_kernel<<<dim3((unsigned)grid), dim3(kLThreads), kLLds, s>>>(p);
    rc = check_hip(hipGetLastError(), "lmhead_lse_kernel");
    if (rc) return rc;
    lse_finalize_kernel<<<dim3((T + kFinTokens - 1) / kFinTokens), dim3(kFinTokens * kFinSlices), 0, s>>>(p.pmax, p.psum, tgt, T, p.n_blocks,
                                                                                                           logprob);
    return check_hip(hipGetLastError(), "lse_finalize_kernel");
}

// ---- the library's own scratch for callers that cannot allocate.  One copy of the array exists on every GPU
// the library's code object is loaded on, at that GPU's own address.  In host code the array's NAME is only a
// handle for the symbol lookup below, never a device address: everything that touches the memory (kernel
// arguments, copies, fills) takes the pointer this function returns.
static __device__ __align__(256) unsigned char scratch[kLogprobScratchBytes];
static std::atomic<void *> g_scratch_ptr[64];   // per device, filled on the first call with that device current

int logprob_static_scratch(void **ptr)
{
    int dev = -1;
    int rc = check_hip(hipGetDevice(&dev), "hipGetDevice");
    if (rc) return rc;
    if (dev < 0 || dev >= 64) {
        set_error("logprob (library scratch): device index %d outside the table of 64", dev);
        return QARL_ERR_UNSUPPORTED;
    }
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        rc = check_hip(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)), "hipGetSymbolAddress(scratch)");
        if (rc) return rc;
        if (!p) {
            set_error("logprob (library scratch): symbol lookup returned a null address");
            return QARL_ERR_HIP;
        }
        g_scratch_ptr[dev].store(p, std::memory_order_release);
    }
    *ptr = p;
    return QARL_OK;
}

}  // namespace qarl
