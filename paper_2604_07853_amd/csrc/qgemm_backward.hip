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


// ---- dW on 256 x 256 tiles: the structure of the LM head kernel (logprob.hip) with the token index as the
// contraction.  A stage holds 64 token rows of both operands as they are stored, Ys [64][256 n] and Xs [64][256 k]
// (512-byte rows, 64 KiB per stage, two stages), filled by asynchronous global -> LDS copies: a wavefront instruction
// moves two rows; chunk q (16 bytes) of row r sits at position q ^ ((r & 3) << 2) of the row, so that the four rows
// a transposing read touches at once lie in different quarters of the 256 bytes the LDS serves per clock.  Rows past
// the expert's end are copied from a row of zeros.  Eight wavefronts of 128 n x 64 k (4 x 2 MFMA tiles, 128
// accumulator registers); the twelve transposing reads of a 16-token slice go out one pair behind each of the first
// six MFMAs of the slice before, the eight copies of the next stage one behind every second MFMA of the first two
// slices, the last slice's MFMAs run behind the stage barrier.  The x rows are gathered through row_map; the ids
// are the same for all lanes of a wavefront and are read with scalar loads (vector loads would share the counter
// the copies are waited on with) one stage before they are turned into addresses.
constexpr int kDwWTile = 256;                       // n rows and k columns per workgroup
constexpr int kDwWRowB = kDwWTile * 2;              // bytes of an LDS row
constexpr int kDwWTileB = kStageM * kDwWRowB;       // one operand tile of a stage: 32 KiB
constexpr int kDwWStageB = 2 * kDwWTileB;           // Ys, then Xs
__device__ __attribute__((aligned(256))) const unsigned char kDwZeroRow[kDwWRowB] = {0};

__device__ __forceinline__ TrBase tr_base_512(int col0, int lane)
{
    const int r16 = lane & 15, g = lane >> 4;
    const int row = 8 * (g >> 1) + (r16 >> 2);                // the row this lane ADDRESSES (second read: + 4)
    const int colq = col0 + 16 * (g & 1) + 4 * (r16 & 3);     // first of the four columns it addresses
    TrBase b;
    b.lo = row * kDwWRowB + (((colq >> 3) ^ ((row & 3) << 2)) << 4) + (colq & 4) * 2;
    b.hi = b.lo + 4 * kDwWRowB;                               // row + 4: same row & 3, same swizzle
    return b;
}

__global__ __launch_bounds__(kBwThreads, 2) void grouped_dw_wide_kernel(DwParams p, const int32_t *__restrict__ row_map)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wn = wave >> 2, wk = wave & 3;   // 128 n x 64 k per wavefront
    const int m32 = lane & 31, h = lane >> 5;
    const int N = p.N, K = p.K;
    const int nbn = N / kDwWTile, nbk = K / kDwWTile, tiles = nbn * nbk;
    // Every expert's tiles are spread over all eight XCDs (consecutive workgroup ids go round-robin over them), so a
    // skewed router loads the XCDs alike; where the tile grid allows it an XCD takes half of the n blocks and a
    // quarter of the k blocks of every expert, i.e. its L2 fetches a fifth of the expert's operand bytes, not all.
    int e, nb, kb;
    if (nbn % 2 == 0 && nbk % 4 == 0) {
        const int xcd = blockIdx.x % 8, idx = blockIdx.x / 8, per = tiles / 8, hn = nbn / 2;
        e = idx / per;
        nb = (xcd & 1) * hn + (idx % per) % hn;
        kb = (xcd >> 1) * (nbk / 4) + (idx % per) / hn;
    } else {
        e = blockIdx.x / tiles;
        nb = (blockIdx.x % tiles) / nbk;
        kb = (blockIdx.x % tiles) % nbk;
    }
    if (e >= p.E) return;
    const int row0 = p.offsets[e], Me = p.offsets[e + 1] - row0;
    const int stages = (Me + kStageM - 1) / kStageM;

    // ---- copies: instruction i (0..3) of this wavefront moves rows 8 w + 2 i and 8 w + 2 i + 1 of a tile; lane L
    // fills position L % 32 of row 8 w + 2 i + L / 32 with the chunk that belongs there
    int rrow[4];
    uint32_t chunkb[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        rrow[i] = wave * 8 + 2 * i + h;
        chunkb[i] = (uint32_t)(((lane & 31) ^ ((rrow[i] & 3) << 2)) << 4);
    }
    const unsigned char *ybase = (const unsigned char *)p.dy + ((int64_t)row0 * N + nb * kDwWTile) * 2;
    const unsigned char *xbase = (const unsigned char *)p.x + (int64_t)kb * kDwWTile * 2;
    const int32_t *mbase = row_map ? row_map + row0 : nullptr;
    int32_t ids[8];                       // x rows of the wavefront's eight token rows of the stage addressed next
    const unsigned char *ysrc[4], *xsrc[4];
    auto load_ids = [&](int s) {
        const int m0 = s * kStageM + wave * 8;
        if (mbase) {
#pragma unroll
            for (int r = 0; r < 8; ++r) ids[r] = mbase[min(m0 + r, Me - 1)];
        } else {
#pragma unroll
            for (int r = 0; r < 8; ++r) ids[r] = row0 + m0 + r;
        }
    };
    auto form_addresses = [&](int s) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int m = s * kStageM + rrow[i];
            const bool valid = m < Me;
            const int id = h ? ids[2 * i + 1] : ids[2 * i];
            ysrc[i] = valid ? ybase + (uint64_t)(uint32_t)m * (uint32_t)(N * 2) + chunkb[i] : kDwZeroRow + chunkb[i];
            xsrc[i] = valid ? xbase + (uint64_t)(uint32_t)id * (uint32_t)(K * 2) + chunkb[i] : kDwZeroRow + chunkb[i];
        }
    };
    auto copy_one = [&](int buf, int i) {   // i = 0..3: Ys, 4..7: Xs
        unsigned char *dst = smem + buf * kDwWStageB + (wave * 8 + 2 * (i & 3)) * kDwWRowB;
        if (i < 4) copy16_to_lds(ysrc[i], dst);
        else copy16_to_lds(xsrc[i - 4], dst + kDwWTileB);
    };

    // ---- operands: transposing reads, n columns 128 wn + 32 ms of Ys and k columns 64 wk + 32 nt of Xs
    TrBase ta[4], tb[2];
#pragma unroll
    for (int ms = 0; ms < 4; ++ms) ta[ms] = tr_base_512(wn * 128 + ms * 32, lane);
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
        tb[nt] = tr_base_512(wk * 64 + nt * 32, lane);
        tb[nt].lo += kDwWTileB;
        tb[nt].hi += kDwWTileB;
    }
    struct Frags {
        bf16x8 a[4], b[2];
    };
    // The transposing reads are written as asm: in front of a read the compiler can see it drains the asynchronous
    // copies in flight (it cannot tell that they fill the other stage buffer).  The results are therefore waited for
    // by hand: wait_frags() in front of the slice that multiplies them.
    const uint32_t lds0 = (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void *)smem;
    auto read_tr = [&](uint32_t base, const TrBase &t, auto off_c) -> bf16x8 {
        constexpr int off = decltype(off_c)::value;
        struct {
            s16x4 lo, hi;
        } v;
        asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v.lo) : "v"(base + (uint32_t)t.lo), "n"(off));
        asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v.hi) : "v"(base + (uint32_t)t.hi), "n"(off));
        return __builtin_bit_cast(bf16x8, v);
    };
    auto wait_frags = [&](Frags &f) {
        asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f.a[0]), "+v"(f.a[1]), "+v"(f.a[2]), "+v"(f.a[3]), "+v"(f.b[0]), "+v"(f.b[1]));
    };
    f32x16 acc[4][2];
#pragma unroll
    for (int ms = 0; ms < 4; ++ms)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[ms][nt][i] = 0.f;
    // Slice j (16 token rows) of stage ks: the eight MFMAs on `cur`, behind each of the first six one operand of
    // `nxt` (two transposing reads), in slices 0 and 1 behind every second MFMA one copy of the next stage.
    auto slice = [&](Frags &cur, Frags &nxt, int ks, auto j_c, auto more_t) {
        constexpr int j = decltype(j_c)::value;
        const int buf = ks & 1;
        const uint32_t base = lds0 + buf * kDwWStageB;
        constexpr std::integral_constant<int, j * 16 * kDwWRowB> off{};
        wait_frags(cur);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int ms = i >> 1, nt = i & 1;
            acc[ms][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur.a[ms], cur.b[nt], acc[ms][nt], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            if (i < 4) nxt.a[i] = read_tr(base, ta[i], off);
            else if (i < 6) nxt.b[i - 4] = read_tr(base, tb[i - 4], off);
            if (decltype(more_t)::value && j < 2 && (i & 1)) copy_one(buf ^ 1, 4 * j + (i >> 1));
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    auto stage_barrier = [&]() {   // own copies landed, own operand reads done; then everybody's
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    };

    if (stages > 0) {
        Frags last, f0, f1, f2, f3;
#pragma unroll
        for (int i = 0; i < 4; ++i) last.a[i] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int i = 0; i < 2; ++i) last.b[i] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
        load_ids(0);
        form_addresses(0);
#pragma unroll
        for (int i = 0; i < 8; ++i) copy_one(0, i);
        load_ids(1);
        stage_barrier();
        auto stage = [&](int ks, auto more_t) {
            if (decltype(more_t)::value) {
                form_addresses(ks + 1);   // from the ids loaded during the stage before
                load_ids(ks + 2);
            }
            slice(last, f0, ks, std::integral_constant<int, 0>{}, more_t);
            slice(f0, f1, ks, std::integral_constant<int, 1>{}, more_t);
            slice(f1, f2, ks, std::integral_constant<int, 2>{}, more_t);
            slice(f2, f3, ks, std::integral_constant<int, 3>{}, more_t);
            stage_barrier();
            last = f3;
        };
        for (int ks = 0; ks + 1 < stages; ++ks) stage(ks, std::true_type{});
        stage(stages - 1, std::false_type{});
        wait_frags(last);
#pragma unroll
        for (int ms = 0; ms < 4; ++ms)
#pragma unroll
            for (int nt = 0; nt < 2; ++nt)
                acc[ms][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(last.a[ms], last.b[nt], acc[ms][nt], 0, 0, 0);
    }

    // ---- epilogue: lane (k column m32 of tile nt, half h), register i -> weight row 32 ms + 8 (i / 4) + 4 h + i % 4.
    // Every 32 x 32 tile turns through this wavefront's own piece of the first stage buffer (rows of 36 floats) and
    // leaves as 16-byte (fp32) or 8-byte (bf16) pieces of whole 128-byte / 64-byte row segments.
    constexpr int kORow = 36 * 4;
    unsigned char *ot = smem + wave * (32 * kORow);
    const int64_t obase = ((int64_t)e * N + nb * kDwWTile + wn * 128) * K + kb * kDwWTile + wk * 64;
#pragma unroll
    for (int ms = 0; ms < 4; ++ms)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
#pragma unroll
            for (int i = 0; i < 16; ++i)
                *(float *)(ot + (8 * (i >> 2) + 4 * h + (i & 3)) * kORow + m32 * 4) = acc[ms][nt][i];
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
            for (int pass = 0; pass < 4; ++pass) {
                const int row = pass * 8 + (lane >> 3);
                const f32x4 v4 = *(const f32x4 *)(ot + row * kORow + (lane & 7) * 16);
                const int64_t o = obase + (int64_t)(ms * 32 + row) * K + nt * 32 + (lane & 7) * 4;
                if (p.out_f32) {
                    *(f32x4 *)((float *)p.out + o) = v4;
                } else {
                    u32x2 ob;
                    ob[0] = (uint32_t)f32_to_bf16_hw(v4[0]) | ((uint32_t)f32_to_bf16_hw(v4[1]) << 16);
                    ob[1] = (uint32_t)f32_to_bf16_hw(v4[2]) | ((uint32_t)f32_to_bf16_hw(v4[3]) << 16);
                    *(u32x2 *)((uint16_t *)p.out + o) = ob;
                }
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
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
    if (N % kDwWTile == 0 && K % kDwWTile == 0 && (int64_t)N * 2 < (1LL << 31) && (int64_t)K * 2 < (1LL << 31)) {
        const int64_t total = (int64_t)E * (N / kDwWTile) * (K / kDwWTile);
        static LdsLimitOnce once;
        if (int rc = raise_lds_limit((const void *)grouped_dw_wide_kernel, once, "hipFuncSetAttribute(grouped dw)")) return rc;
        grouped_dw_wide_kernel<<<dim3((unsigned)total), dim3(kBwThreads), 2 * kDwWStageB, s>>>(p, row_map);
        return check_hip(hipGetLastError(), "grouped_dw_wide_kernel");
    }
    grouped_dw_kernel<<<dim3((unsigned)grid), dim3(kBwThreads), 0, s>>>(p);
    return check_hip(hipGetLastError(), "grouped_dw_kernel");
}

}  // namespace qarl
