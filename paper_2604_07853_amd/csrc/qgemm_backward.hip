// Backward of the rollout-aligned W4A16 forward under the straight-through estimator (section 3.1, item 2: the
// forward runs on the low-bit weights; gradients are computed as if Quant were the identity, in the trainer's
// 16-bit precision, and applied to the BF16 masters).  For Y[i] = What_e x[row(i)] (eq. (1), What = s*q):
//     dX[i][k]    = sum_n dY[i][n] * What_e[n][k]                -> qgemm_dx_kernel
//     dW[e][n][k] = sum_{i in expert e} dY[i][n] * x[row(i)][k]  -> grouped_dw_kernel
// Both are dense contractions on v_mfma_f32_32x32x16_bf16 with fp32 accumulation.  In both the contraction index
// is the one the operands do NOT store contiguously (n for dX: the codes are packed along k; the token index for
// dW), while the matrix instruction wants 8 consecutive contraction elements per lane.  The tiles go to LDS as
// they are stored (rows = contraction index, 16-byte pieces) and are read with the transposing LDS read
// ds_read_b64_tr_b16, which hands a lane four consecutive ROWS of one column: within each group of 16 lanes, lane
// 4 a + b receives element b of the 8 bytes addressed by lanes a, a + 4, a + 8 and a + 12 of the group.
//
// dX.  A workgroup owns 128 rows x 128 output columns k, i.e. exactly one scale group g of every weight row, so
// the scale s[n][g] depends on the contraction index alone and is folded into the gradient operand:
// A'[i][n] = bf16(dY[i][n] * s[n][g]), rounded once (the 16-bit backward; a one-hot dY and the exact-integer
// regime stay exact).  The codes go through the same exponent trick as in the forward, (q+24)/16 as an exact
// bf16, written row by row ([n][k]) into LDS; the offset is removed at the end with the row sums of A' (fp32,
// accumulated while A' is staged): dX = 16 * acc - 24 * rowsum.
#include <type_traits>

#include "common.hpp"

namespace qarl {

namespace {

constexpr int kBwThreads = 512;
constexpr int kTM = 128;   // rows (dX) / weight rows n (dW) per workgroup
constexpr int kTK = 128;   // output columns k per workgroup
constexpr int kStageN = 128;   // dX: contraction elements n per stage
constexpr int kStageM = 64;    // dW: contraction elements (token rows) per stage

struct DxParams {
    const uint32_t *codes;    // 1 KiB blocks [E * N / 16][K / 128][256 words]
    const uint16_t *scales;   // bf16 [E][N][K / 128]
    const uint16_t *dy;       // bf16 [M][N], rows grouped by expert
    const int32_t *offsets;
    const int32_t *out_row_map;
    void *out;                // [M][K]
    int E, N, K, out_f32;
    int m_slots, total;
};

// 16-byte chunk swizzles of 256-byte LDS rows.  As: rows are gradient rows, read by 32 consecutive rows at once.
// Tiles read by the transposing read: a 32-lane pass touches four consecutive rows (from a multiple of four) and 64
// bytes of each, so the rows go to different quarters of the 256 bytes; the second term spreads the sixteen rows a
// code block is written to.
__device__ __forceinline__ int swz_a(int m) { return m & 15; }
__device__ __forceinline__ int swz_tr(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// MFMA operand of lane `lane` (row or column l % 32, contraction elements 8 (l / 32) .. + 7) from a tile stored
// [contraction index][128 columns] bf16 in 256-byte rows with swz_tr chunks: columns col0 .. col0 + 31 (col0 a
// multiple of 32), contraction rows 16 st .. 16 st + 15.  The two addresses a lane passes are its base offsets
// (computed once: the swizzle of row 16 st + c does not depend on st) plus 4096 st, an immediate of the read.
struct TrBase {
    int lo, hi;
};
__device__ __forceinline__ TrBase tr_base(int col0, int lane)
{
    const int r16 = lane & 15, g = lane >> 4;
    const int row = 8 * (g >> 1) + (r16 >> 2);                // the row this lane ADDRESSES (second read: + 4)
    const int colq = col0 + 16 * (g & 1) + 4 * (r16 & 3);     // first of the four columns it addresses
    TrBase b;
    b.lo = row * 256 + (((colq >> 3) ^ swz_tr(row)) << 4) + (colq & 4) * 2;
    b.hi = (row + 4) * 256 + (((colq >> 3) ^ swz_tr(row + 4)) << 4) + (colq & 4) * 2;
    return b;
}
template <int ST>
__device__ __forceinline__ bf16x8 read_operand_tr(const unsigned char *tile, const TrBase &b)
{
    struct {
        s16x4 lo, hi;
    } v;
    v.lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(tile + b.lo + ST * 4096));
    v.hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(tile + b.hi + ST * 4096));
    return __builtin_bit_cast(bf16x8, v);
}

// compile-time loop over the 16-element contraction steps of a stage
template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>());
        static_for<I + 1, N>(f);
    }
}

__global__ __launch_bounds__(kBwThreads, 4) void qgemm_dx_kernel(DxParams p)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    __shared__ __attribute__((aligned(16))) int s_orow[kTM];
    __shared__ __attribute__((aligned(16))) float s_rs[kTM];
    unsigned char *As = smem;                       // [kTM][kStageN] bf16, 256-byte rows
    unsigned char *Bs = smem + kTM * kStageN * 2;   // [kStageN n][kTK k] bf16 (q+24)/16, 256-byte rows
    float *sc = (float *)(smem + (kTM + kTK) * kStageN * 2);   // [N] scales of group g as fp32

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int N = p.N, K = p.K, G = K / kGroup;

    const int per_xcd = p.total / 8;
    const int v = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
    const int g = v % G;   // output column block = scale group
    const int slot = v / G;
    if (slot >= p.m_slots) return;
    // slot -> (expert, row tile): wavefront-level scan of the per-expert tile counts (four experts per lane)
    int e, mtile;
    {
        int cnt[4], sum = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int ex = lane * 4 + q;
            cnt[q] = ex < p.E ? (p.offsets[ex + 1] - p.offsets[ex] + kTM - 1) / kTM : 0;
            sum += cnt[q];
        }
        int incl = sum;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int up = __shfl_up(incl, o, 64);
            if (lane >= o) incl += up;
        }
        int base = incl - sum, found = -1, mt = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (slot >= base && slot < base + cnt[q]) {
                found = lane * 4 + q;
                mt = slot - base;
            }
            base += cnt[q];
        }
        const unsigned long long hit = __ballot(found >= 0);
        if (hit == 0) return;
        const int src = __ffsll((long long)hit) - 1;
        e = __builtin_amdgcn_readfirstlane(__shfl(found, src, 64));
        mtile = __builtin_amdgcn_readfirstlane(__shfl(mt, src, 64));
    }
    const int row0 = p.offsets[e] + mtile * kTM;
    const int mrem = min(kTM, p.offsets[e + 1] - row0);
    if (tid < kTM) s_orow[tid] = tid < mrem ? (p.out_row_map ? p.out_row_map[row0 + tid] : row0 + tid) : -1;
    for (int n = tid; n < N; n += kBwThreads) sc[n] = bf16_bits_to_f32(p.scales[((int64_t)e * N + n) * G + g]);

    // gradient staging: chunk id = tid + 512 u -> row id >> 4, 16-byte piece id & 15 of the stage's 128 n
    const int am = tid >> 4, acn = tid & 15;
    float rowsum[4] = {0.f, 0.f, 0.f, 0.f};
    const bf16x2 ones2 = __builtin_bit_cast(bf16x2, 0x3f803f80u);
    // weight staging: this wavefront expands the block of rows n0 + 16 wave .. + 15; lane = (k range q, row c)
    const int bq = lane >> 4, bc = lane & 15;
    // matrix phase: wavefront (wm, wk) owns rows 32 wm .. + 31, columns 64 wk .. + 63
    const int wm = wave >> 1, wk = wave & 1, m32 = lane & 31, h = lane >> 5;
    f32x16 acc[2];
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[kt][i] = 0.f;

    const TrBase tb[2] = {tr_base(wk * 64, lane), tr_base(wk * 64 + 32, lane)};
    // The global loads of a stage are issued one stage ahead, right after the previous stage's operands have
    // been written to LDS, so they travel during that stage's matrix phase.
    u32x4 gv[4], wv;
    const uint16_t *gbase = p.dy + (int64_t)(row0 + am) * N + acn * 8;                      // row am of the tile; row am + 32 u: + 32 u N
    const uint32_t *cbase = p.codes + (((int64_t)e * N / 16 + wave) * G + g) * 256 + lane * 4;   // tile of rows n0 + 16 wave ..: + (n0 / 16) G blocks
    auto load_stage = [&](int n0) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            gv[u] = u32x4{0, 0, 0, 0};
            if (am + 32 * u < mrem) gv[u] = *(const u32x4 *)(gbase + (uint32_t)(32 * u) * (uint32_t)N + n0);
        }
        wv = *(const u32x4 *)(cbase + (uint32_t)(n0 / 16) * (uint32_t)(G * 256));
    };
    load_stage(0);
    for (int n0 = 0; n0 < N; n0 += kStageN) {
        lds_barrier();   // the matrix phase of the previous stage is done (first trip: the scales are written)
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int m = am + 32 * u;
            const f32x4 s_lo = *(const f32x4 *)(sc + n0 + acn * 8), s_hi = *(const f32x4 *)(sc + n0 + acn * 8 + 4);
            u32x4 o;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float s0 = i < 2 ? s_lo[2 * i] : s_hi[2 * i - 4], s1 = i < 2 ? s_lo[2 * i + 1] : s_hi[2 * i - 3];
                bf16x2 pr;
                pr[0] = (__bf16)(__uint_as_float(gv[u][i] << 16) * s0);
                pr[1] = (__bf16)(__uint_as_float(gv[u][i] & 0xffff0000u) * s1);
                // row sum of the ROUNDED values: both halves times 1.0, added to the running sum in one operation
                rowsum[u] = __builtin_amdgcn_fdot2_f32_bf16(pr, ones2, rowsum[u], false);
                o[i] = __builtin_bit_cast(uint32_t, pr);
            }
            *(u32x4 *)(As + m * 256 + ((acn ^ swz_a(m)) << 4)) = o;
        }
        {
            const int nl = wave * 16 + bc;   // row of the stage; word j of the lane = columns 32 bq + 8 j .. + 7
#pragma unroll
            for (int j = 0; j < 4; ++j)
                *(u32x4 *)(Bs + nl * 256 + (((bq * 4 + j) ^ swz_tr(nl)) << 4)) = __builtin_bit_cast(u32x4, unpack_int4_word(wv[j]));
        }
        if (n0 + kStageN < N) load_stage(n0 + kStageN);
        lds_barrier();
        static_for<0, kStageN / 16>([&](auto st_c) {
            constexpr int st = decltype(st_c)::value;
            const int ch = 2 * st + h;
            const int m = wm * 32 + m32;
            const bf16x8 a = *(const bf16x8 *)(As + m * 256 + ((ch ^ swz_a(m)) << 4));
#pragma unroll
            for (int kt = 0; kt < 2; ++kt) {
                const bf16x8 b = read_operand_tr<st>(Bs, tb[kt]);
                acc[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[kt], 0, 0, 0);
            }
        });
    }
    // row sums of A': the 16 threads of a row sit in 16 consecutive lanes
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        float r = rowsum[u];
#pragma unroll
        for (int o = 1; o < 16; o <<= 1) r += __shfl_xor(r, o, 64);
        if (acn == 0) s_rs[am + 32 * u] = r;
    }
    lds_barrier();
    // lane (column m32 of tile kt, half h), register i -> row 32 wm + 8 (i / 4) + 4 h + i % 4
#pragma unroll
    for (int i4 = 0; i4 < 4; ++i4) {
        const int r0 = wm * 32 + 8 * i4 + 4 * h;
        const i32x4 orow4 = *(const i32x4 *)(s_orow + r0);
        const f32x4 rs4 = *(const f32x4 *)(s_rs + r0);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int64_t orow = orow4[i];
            if (orow < 0) continue;
#pragma unroll
            for (int kt = 0; kt < 2; ++kt) {
                const float val = fmaf(16.f, acc[kt][i4 * 4 + i], -24.f * rs4[i]);
                const int64_t col = g * kTK + wk * 64 + kt * 32 + m32;
                if (p.out_f32) ((float *)p.out)[orow * K + col] = val;
                else ((uint16_t *)p.out)[orow * K + col] = f32_to_bf16_hw(val);
            }
        }
    }
}

struct DwParams {
    const uint16_t *dy;   // bf16 [M][N], rows grouped by expert
    const uint16_t *x;    // bf16 [x_rows][K]
    const int32_t *row_map;
    const int32_t *offsets;
    void *out;            // [E][N][K]
    int E, N, K, out_f32;
};

__global__ __launch_bounds__(kBwThreads, 4) void grouped_dw_kernel(DwParams p)
{
    __shared__ __attribute__((aligned(16))) unsigned char Ys[kStageM * kTM * 2];   // [64 token rows][128 n] bf16
    __shared__ __attribute__((aligned(16))) unsigned char Xs[kStageM * kTK * 2];   // [64 token rows][128 k] bf16
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int N = p.N, K = p.K;
    const int nbk = K / kTK, nbn = N / kTM;
    const int kb = blockIdx.x % nbk, nb = (blockIdx.x / nbk) % nbn, e = blockIdx.x / (nbk * nbn);
    if (e >= p.E) return;
    const int row0 = p.offsets[e], Me = p.offsets[e + 1] - row0;

    // staging: thread -> token rows tid / 16 and tid / 16 + 32 of the stage, 16-byte piece tid % 16 of their 128
    // columns (16 lanes take 256 contiguous bytes of a row)
    const int sr = tid >> 4, sc = tid & 15;
    const int wn = wave >> 1, wk = wave & 1, m32 = lane & 31, h = lane >> 5;
    f32x16 acc[2];
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[kt][i] = 0.f;

    const TrBase ta = tr_base(wn * 32, lane), tb[2] = {tr_base(wk * 64, lane), tr_base(wk * 64 + 32, lane)};
    // The global loads of a stage (row ids first, then the two tiles) are issued one stage ahead, right after the
    // previous stage's tiles have been written to LDS, so they travel during that stage's matrix phase.
    // (addresses: one pointer per tile and one widening multiply-add per load)
    u32x4 yv[2], xv[2];
    const uint16_t *ybase = p.dy + (int64_t)row0 * N + nb * kTM + sc * 8;
    const uint16_t *xbase = p.x + kb * kTK + sc * 8;
    const int32_t *mbase = p.row_map ? p.row_map + row0 : nullptr;
    auto load_stage = [&](int m0) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int r = m0 + sr + 32 * u;
            yv[u] = u32x4{0, 0, 0, 0};
            xv[u] = u32x4{0, 0, 0, 0};
            if (r < Me) {   // rows past the expert's end contribute zeros
                const uint32_t xrow = mbase ? (uint32_t)mbase[r] : (uint32_t)(row0 + r);
                yv[u] = *(const u32x4 *)(ybase + (uint64_t)(uint32_t)r * (uint32_t)N);
                xv[u] = *(const u32x4 *)(xbase + (uint64_t)xrow * (uint32_t)K);
            }
        }
    };
    load_stage(0);
    for (int m0 = 0; m0 < Me; m0 += kStageM) {
        lds_barrier();   // the matrix phase of the previous stage is done
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int r = sr + 32 * u;
            const int off = r * 256 + ((sc ^ swz_tr(r)) << 4);
            *(u32x4 *)(Ys + off) = yv[u];
            *(u32x4 *)(Xs + off) = xv[u];
        }
        if (m0 + kStageM < Me) load_stage(m0 + kStageM);
        lds_barrier();
        static_for<0, kStageM / 16>([&](auto st_c) {
            constexpr int st = decltype(st_c)::value;
            const bf16x8 a = read_operand_tr<st>(Ys, ta);
#pragma unroll
            for (int kt = 0; kt < 2; ++kt) {
                const bf16x8 b = read_operand_tr<st>(Xs, tb[kt]);
                acc[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[kt], 0, 0, 0);
            }
        });
    }
    // lane (column m32 of tile kt, half h), register i -> weight row 32 wn + 8 (i / 4) + 4 h + i % 4
    const int64_t obase = ((int64_t)e * N + nb * kTM + wn * 32 + 4 * h) * K + kb * kTK + wk * 64 + m32;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const uint32_t orow = (uint32_t)(8 * (i >> 2) + (i & 3)) * (uint32_t)K;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) {
            if (p.out_f32) ((float *)p.out + obase)[orow + kt * 32] = acc[kt][i];
            else ((uint16_t *)p.out + obase)[orow + kt * 32] = f32_to_bf16_hw(acc[kt][i]);
        }
    }
}

}  // namespace

int launch_qgemm_dx(const GemmArgs &a, hipStream_t s)
{
    if (a.E > 256 || a.N % kStageN != 0 || a.K % kTK != 0 || a.N > 8192) {
        set_error("qgemm dx: needs E <= 256, N %% 128 == 0, N <= 8192, K %% 128 == 0 (got E=%d N=%d K=%d)", a.E, a.N, a.K);
        return QARL_ERR_UNSUPPORTED;
    }
    DxParams p;
    p.codes = (const uint32_t *)a.codes;
    p.scales = (const uint16_t *)a.scales;
    p.dy = (const uint16_t *)a.x;
    p.offsets = a.offsets;
    p.out_row_map = a.out_row_map;
    p.out = a.out;
    p.E = a.E;
    p.N = a.N;
    p.K = a.K;
    p.out_f32 = a.out_f32;
    const int64_t slots = (a.M + kTM - 1) / kTM + a.E;
    const int64_t total = ((slots * (a.K / kTK) + 7) / 8) * 8;
    if (total > 0x7fffffffLL) {
        set_error("qgemm dx: grid too large");
        return QARL_ERR_UNSUPPORTED;
    }
    p.m_slots = (int)slots;
    p.total = (int)total;
    const size_t lds = (size_t)(kTM + kTK) * kStageN * 2 + (size_t)a.N * 4;
    static LdsLimitOnce once;
    if (int rc = raise_lds_limit((const void *)qgemm_dx_kernel, once, "hipFuncSetAttribute(qgemm dx)")) return rc;
    qgemm_dx_kernel<<<dim3((unsigned)total), dim3(kBwThreads), lds, s>>>(p);
    return check_hip(hipGetLastError(), "qgemm_dx_kernel");
}

int launch_grouped_dw(const void *dy, const void *x, const int32_t *row_map, const int32_t *offsets, int E, int N, int K,
                      void *out, int out_f32, hipStream_t s)
{
    if (N % kTM != 0 || K % kTK != 0) {
        set_error("grouped dw: needs N %% 128 == 0 and K %% 128 == 0 (got N=%d K=%d)", N, K);
        return QARL_ERR_UNSUPPORTED;
    }
    const int64_t grid = (int64_t)E * (N / kTM) * (K / kTK);
    if (grid > 0x7fffffffLL) {
        set_error("grouped dw: grid too large");
        return QARL_ERR_UNSUPPORTED;
    }
    DwParams p;
    p.dy = (const uint16_t *)dy;
    p.x = (const uint16_t *)x;
    p.row_map = row_map;
    p.offsets = offsets;
    p.out = out;
    p.E = E;
    p.N = N;
    p.K = K;
    p.out_f32 = out_f32;
    grouped_dw_kernel<<<dim3((unsigned)grid), dim3(kBwThreads), 0, s>>>(p);
    return check_hip(hipGetLastError(), "grouped_dw_kernel");
}

}  // namespace qarl
