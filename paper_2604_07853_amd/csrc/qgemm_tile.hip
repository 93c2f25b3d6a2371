// Grouped quantized GEMM, MFMA-tiled ("prefill" / training-forward) path for W4A16: the same
// contraction as the weight-streaming path (eq. (1) of section 2.2), on the same codes and
// scales and with the same exact dequantized weight s*q, for experts that see hundreds to
// thousands of token rows, where the path is a dense contraction.  (FP8: qgemm_tile_fp8.hip.)
//
// A workgroup owns a (32*MS)-token x 256-column tile of one expert.  Its eight wavefronts split
// the columns: each owns 32 of them as MS v_mfma_f32_32x32x16 tiles, so no packed weight is read
// or expanded twice in a workgroup.  Token rows are gathered once per workgroup into a
// double-buffered LDS tile (one 128-k scale group per step) by asynchronous global -> LDS copies,
// 16-byte chunks XOR-swizzled with the row so that copies and operand reads are free of bank
// conflicts; packed weights go global ->
// registers and are expanded there, so the LDS only carries the activation operand.  Small
// wavefront tiles keep the register count at 128, four wavefronts per SIMD from two workgroups
// that run out of step: global-load latency and the VALU work of the expansion are hidden by the
// other wavefronts' MFMAs rather than by a deep software pipeline.  The kernel is bound by VALU
// issue next to the MFMAs, so everything outside the k loop is kept short: the expert lookup is a
// wavefront-level scan, output rows wait in LDS, SiLU uses the hardware
// exp2 / rcp, and gate and up meet through one 16-lane row swap.
//
// The group handling is the one described in qgemm_stream_w4.hip: codes become the exact bf16
// values (q+24)/16, every scale group accumulates in its own fp32 accumulator that starts at
// -1.5 * sum_k x (the sums come from a small pre-pass over the activations, once per call), and
// is folded in with one FMA by 16*s.
#include "common.hpp"

namespace qarl {

constexpr int kBN = 256;
constexpr int kTileWaves = kBN / 32;          // each wavefront owns 32 columns
constexpr int kTileThreads = 64 * kTileWaves;
constexpr int kARowB = kGroup * 2;            // bytes per LDS row: 128 bf16, no padding (chunks are swizzled)

struct TileParams {
    const uint32_t *codes;
    const void *scales;
    const void *x;
    const float *x_group_sums;
    const float *x_scales;   // W4A8: scale of each activation row (x then holds e4m3 values as bf16), else null
    const int32_t *row_map;
    const int32_t *out_row_map;
    const int32_t *offsets;
    void *out;
    int E, N, K, out_f32;
    int n_blocks;   // column blocks per expert
    int m_slots;    // upper bound of token tiles over all experts
    int total;      // n_blocks * m_slots rounded up to a multiple of 8
};

// MS: 32-row token tiles per wavefront (workgroup tile = 32 MS tokens x 256 columns).
template <int EPI, int MS>
__global__ __launch_bounds__(kTileThreads, MS == 2 ? 4 : 2) void qgemm_tile_kernel(TileParams p)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr bool kSilu = (EPI == QARL_EPI_SILU_MUL);
    constexpr int kBM = 32 * MS;
    constexpr int kThreads = kTileThreads;
    constexpr int kStride = kARowB;
    constexpr int kBufBytes = kBM * kStride + kBM * 4;  // tile + per-row group sums
    __shared__ __attribute__((aligned(16))) int s_rows[kBM];   // activation row of each tile row (clamped to a valid one)
    __shared__ __attribute__((aligned(16))) int s_orow[kBM];   // output row, -1 past the expert's last row
    __shared__ __attribute__((aligned(16))) float s_xsc[kBM];  // W4A8: row scale s_x (1 otherwise)

    const int tid = threadIdx.x, lane = tid & 63, wn = tid >> 6;
    const int c = lane & 31, h = lane >> 5;

    // workgroup id -> (m slot, column block): consecutive ids go round-robin over the 8 XCDs, so
    // give every XCD a contiguous range of tiles: column blocks of one token tile share its L2.
    const int per_xcd = p.total / 8;
    const int v = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
    const int nb = v % p.n_blocks;
    const int slot = v / p.n_blocks;
    if (slot >= p.m_slots) return;

    // slot -> (expert, tile within expert): every wavefront scans the per-expert tile counts itself
    // (four experts per lane, prefix sum across lanes), so no barrier is needed to agree on it.
    int e, mtile;
    {
        int cnt[4], sum = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int ex = lane * 4 + q;
            cnt[q] = ex < p.E ? (p.offsets[ex + 1] - p.offsets[ex] + kBM - 1) / kBM : 0;
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
    const int row0 = p.offsets[e] + mtile * kBM;
    const int mrem = min(kBM, p.offsets[e + 1] - row0);
    if (tid < kBM) {
        // rows past the expert's end read the tile's first row (valid data, results never stored)
        const int i = row0 + (tid < mrem ? tid : 0);
        const int xrow = p.row_map ? p.row_map[i] : i;
        s_rows[tid] = xrow;
        s_orow[tid] = tid < mrem ? (p.out_row_map ? p.out_row_map[i] : i) : -1;
        s_xsc[tid] = p.x_scales ? p.x_scales[xrow] : 1.f;
    }
    lds_barrier();

    const int N = p.N, K = p.K, G = K / kGroup;
    // Weight row of this lane (any row may feed any lane of the B operand).  SILU_MUL: lanes c < 16
    // take 16 gate rows, lanes c >= 16 the matching 16 up rows, so gate j and up j sit 16 lanes apart.
    int nrow, ocol;
    bool tile_ok;
    if (kSilu) {
        ocol = nb * (kBN / 2) + wn * 16 + (c & 15);
        nrow = (c < 16 ? 0 : N / 2) + ocol;
        tile_ok = ocol - (c & 15) + 16 <= N / 2;
    } else {
        ocol = nrow = nb * kBN + wn * 32 + c;
        tile_ok = nrow - c + 32 <= N;
    }
    // columns past N read row 0 of the expert (valid data, results never stored)
    const int64_t wr = (int64_t)e * N + (tile_ok ? nrow : 0);
    // Byte offsets from the (uniform) array bases; the launcher checks that every array is below 4 GiB.
    //   codes: block (16-row tile, group g) is 1 KiB; this lane's row is wr % 16 of tile wr / 16 and it
    //   takes the 16-byte pieces q = 2h + u (k in [32 q, +32)).
    const uint32_t woff = (uint32_t)((wr / 16) * G * 1024 + (wr % 16) * 16 + h * 512);
    const uint32_t soff = (uint32_t)(wr * G * 2);   // the row's bf16 scales

    // ---- activation tile: kBM rows x 128 k by asynchronous copies.  A wavefront instruction moves 4 rows x 256
    // bytes (lane L: row L / 16, LDS chunk L % 16); chunk q of row r sits at r * 256 + (q ^ (r & 15)) * 16, so
    // the lane fetches the chunk that belongs there.
    constexpr int kARegs = (kBM * 16) / kThreads;
    const unsigned char *arow[kARegs];
#pragma unroll
    for (int u = 0; u < kARegs; ++u) {
        const int r = u * (kThreads / 16) + (tid >> 4);
        const int q = (lane & 15) ^ (r & 15);
        arow[u] = (const unsigned char *)p.x + (int64_t)s_rows[r] * K * 2 + q * 16;
    }
    const float *gsrow = p.x_group_sums + (int64_t)s_rows[tid % kBM] * G;
    auto copy_a = [&](int g, int buf) {
        unsigned char *xs = smem + buf * kBufBytes;
#pragma unroll
        for (int u = 0; u < kARegs; ++u)
            copy16_to_lds(arow[u] + g * kGroup * 2, xs + (u * (kThreads / 16) + wn * 4) * kStride);
        if (tid < kBM)   // whole wavefronts: kBM is a multiple of 64
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(gsrow + g),
                                             (__attribute__((address_space(3))) void *)(xs + kBM * kStride + (tid & ~63) * 4), 4, 0, 0);
    };

    // ---- packed weights of one group
    constexpr int kWRegs = 2;  // 16-byte loads per lane
    struct BRegs {
        u32x4 w[kWRegs];
        uint32_t s;
    };
    auto load_b = [&](BRegs &dst, int g) {
        const unsigned char *wb = (const unsigned char *)p.codes;
        const uint32_t o = woff + (uint32_t)g * 1024u;
#pragma unroll
        for (int u = 0; u < kWRegs; ++u) dst.w[u] = *(const u32x4 *)(wb + (o + u * 256u));
        dst.s = *(const uint16_t *)((const unsigned char *)p.scales + (soff + (uint32_t)g * 2u));
    };

    f32x16 acc[MS];
#pragma unroll
    for (int ms = 0; ms < MS; ++ms)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[ms][i] = 0.f;

    // One 128-k step on the LDS buffer `buf` with the weights in `b`.
    const int afrag = c * kStride;   // this lane's operand read: row c (+32 ms); chunk 8 h + j, swizzled
    auto step = [&](const BRegs &b, int buf) {
        const unsigned char *xs = smem + buf * kBufBytes + afrag;
        const float *sx = (const float *)(smem + buf * kBufBytes + kBM * kStride);
        f32x16 ag[MS];
#pragma unroll
        for (int ms = 0; ms < MS; ++ms)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                const f32x4 init = *(const f32x4 *)(sx + ms * 32 + 8 * i4 + 4 * h);
#pragma unroll
                for (int i = 0; i < 4; ++i) ag[ms][i4 * 4 + i] = init[i];
            }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const bf16x8 bw = unpack_int4_word(b.w[j >> 2][j & 3]);
#pragma unroll
            for (int ms = 0; ms < MS; ++ms) {
                const bf16x8 a = *(const bf16x8 *)(xs + ms * 32 * kStride + (((8 * h + j) ^ (c & 15)) << 4));
                ag[ms] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bw, ag[ms], 0, 0, 0);
            }
        }
        const float s16 = 16.f * bf16_bits_to_f32(b.s);
#pragma unroll
        for (int ms = 0; ms < MS; ++ms)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[ms][i] = fmaf(s16, ag[ms][i], acc[ms][i]);
    };

    // Two steps per trip so that the two weight register sets swap roles without copies.  The weight registers
    // of a step are touched before the next copies and loads go out: the compiler waits for every outstanding
    // vector load at the first use of a loaded register while asynchronous copies are in flight, and at that
    // point nothing is.
    BRegs b0, b1;
    b0.s = 0;
    b1.s = 0;
    copy_a(0, 0);
    load_b(b0, 0);
    copy_barrier();
    for (int g = 0; g < G; g += 2) {
        asm volatile("" : "+v"(b0.w[0]), "+v"(b0.w[1]), "+v"(b0.s));
        if (g + 1 < G) {
            copy_a(g + 1, 1);
            load_b(b1, g + 1);
        }
        step(b0, 0);
        copy_barrier();
        if (g + 1 >= G) break;
        asm volatile("" : "+v"(b1.w[0]), "+v"(b1.w[1]), "+v"(b1.s));
        if (g + 2 < G) {
            copy_a(g + 2, 0);
            load_b(b0, g + 2);
        }
        step(b1, 1);
        copy_barrier();
    }

    // ---- epilogue: lane (c,h), register i -> token row 8*(i/4) + 4h + i%4, column c of the tile.
    // A lane holds one column of 16 rows, so a direct store would move 4 (or 2) bytes per lane.  The results
    // take a turn through the activation buffers, which are free after the loop's last barrier, and leave as
    // 16-byte pieces of whole 128-byte row segments.
    static_assert(2 * kBufBytes >= kBM * (kBN / 2) * 2 && 2 * kBufBytes >= (kThreads / 64) * 32 * 32 * 4, "epilogue tile does not fit");
    if (kSilu) {
        // workgroup tile [kBM rows][128 columns] bf16 in LDS
        uint16_t *ot = (uint16_t *)smem;
#pragma unroll
        for (int ms = 0; ms < MS; ++ms) {
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                f32x4 vv;
#pragma unroll
                for (int i = 0; i < 4; ++i) vv[i] = acc[ms][i4 * 4 + i];
                // Registers i and i+1 trade 16-lane rows: afterwards every lane holds a gate value
                // and the up value of the same column; lanes c < 16 for row i, lanes c >= 16 for row i+1.
#pragma unroll
                for (int ip = 0; ip < 2; ++ip) {
                    const u32x2 sw = __builtin_amdgcn_permlane16_swap(__float_as_uint(vv[2 * ip]),
                                                                      __float_as_uint(vv[2 * ip + 1]), false, false);
                    const int row = ms * 32 + 8 * i4 + 4 * h + 2 * ip + (c >> 4);
                    const float rs = s_xsc[row];
                    const float a = silu_mul_f32(__uint_as_float(sw[0]) * rs, __uint_as_float(sw[1]) * rs);
                    ot[row * (kBN / 2) + wn * 16 + (c & 15)] = f32_to_bf16_hw(a);
                }
            }
        }
        lds_barrier();
        constexpr int kPieces = kBM * (kBN / 2) * 2 / 16;   // 16 pieces per row
        const uint32_t rstride = (uint32_t)(N / 2) * 2u;    // bytes per output row (< 2^31: checked by the launcher)
#pragma unroll
        for (int q0 = 0; q0 < kPieces; q0 += kThreads) {
            const int q = q0 + tid, row = q >> 4, piece = q & 15;
            const int orow = s_orow[row];
            const int oc = nb * (kBN / 2) + piece * 8;
            const u32x4 v4 = *(const u32x4 *)(ot + row * (kBN / 2) + piece * 8);
            if (orow >= 0 && oc + 8 <= N / 2)
                *(u32x4 *)((unsigned char *)p.out + ((uint64_t)(uint32_t)orow * rstride + (uint32_t)oc * 2u)) = v4;
        }
    } else {
        // per wavefront [32 rows][32 columns] fp32 in LDS, one 32-row tile after the other; only the wavefront
        // itself touches its region, and the LDS operations of a wavefront execute in order
        float *ot = (float *)smem + wn * (32 * 32);
        const int esz = p.out_f32 ? 4 : 2;
        const uint32_t rstride = (uint32_t)N * (uint32_t)esz;   // bytes per output row (< 2^31: checked by the launcher)
        const int oc = nb * kBN + wn * 32 + (lane & 7) * 4;      // first of this lane's four columns
        unsigned char *obase = (unsigned char *)p.out + (int64_t)oc * esz;
#pragma unroll
        for (int ms = 0; ms < MS; ++ms) {
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                f32x4 vv;
#pragma unroll
                for (int i = 0; i < 4; ++i) vv[i] = acc[ms][i4 * 4 + i];
                const f32x4 rs4 = *(const f32x4 *)(s_xsc + ms * 32 + 8 * i4 + 4 * h);
#pragma unroll
                for (int i = 0; i < 4; ++i) ot[(8 * i4 + 4 * h + i) * 32 + c] = vv[i] * rs4[i];
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
            for (int pass = 0; pass < 4; ++pass) {
                const int row = pass * 8 + (lane >> 3);
                const f32x4 v4 = *(const f32x4 *)(ot + row * 32 + (lane & 7) * 4);
                const int orow = s_orow[ms * 32 + row];
                if (orow >= 0 && tile_ok) {
                    unsigned char *dst = obase + (uint64_t)(uint32_t)orow * rstride;
                    if (p.out_f32) {
                        __builtin_nontemporal_store(v4, (f32x4 *)dst);
                    } else {
                        u32x2 o;
                        o[0] = (uint32_t)f32_to_bf16_hw(v4[0]) | ((uint32_t)f32_to_bf16_hw(v4[1]) << 16);
                        o[1] = (uint32_t)f32_to_bf16_hw(v4[2]) | ((uint32_t)f32_to_bf16_hw(v4[3]) << 16);
                        __builtin_nontemporal_store(o, (u32x2 *)dst);
                    }
                }
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        }
    }
}

template <int EPI, int MS>
static int launch_cfg(const GemmArgs &a, hipStream_t s)
{
    constexpr int kBM = 32 * MS;
    if (a.E > 256) {
        set_error("qgemm (prefill path): at most 256 experts (got %d)", a.E);
        return QARL_ERR_UNSUPPORTED;
    }
    if (a.N % 32 != 0 || a.N > (1 << 28)) {
        set_error("qgemm (prefill path): N %% 32 == 0 and N <= 2^28 required (got %d)", a.N);
        return QARL_ERR_UNSUPPORTED;
    }
    const int64_t n_w = (int64_t)a.E * a.N * a.K;
    if (n_w / 2 >= (1LL << 32)) {
        set_error("qgemm (prefill path): quantized weights of one call must stay below 4 GiB");
        return QARL_ERR_UNSUPPORTED;
    }
    TileParams p;
    p.codes = (const uint32_t *)a.codes;
    p.scales = a.scales;
    p.x = a.x;
    p.x_group_sums = a.x_group_sums;
    p.x_scales = a.fmt == QARL_W4A8_G128 ? a.x_scales : nullptr;
    p.row_map = a.row_map;
    p.out_row_map = a.out_row_map;
    p.offsets = a.offsets;
    p.out = a.out;
    p.E = a.E;
    p.N = a.N;
    p.K = a.K;
    p.out_f32 = a.out_f32;
    p.n_blocks = (EPI == QARL_EPI_SILU_MUL) ? (a.N / 2 + kBN / 2 - 1) / (kBN / 2) : (a.N + kBN - 1) / kBN;
    const int64_t slots = (a.M + kBM - 1) / kBM + a.E;
    const int64_t total = ((slots * p.n_blocks + 7) / 8) * 8;
    if (total > 0x7fffffffLL) {
        set_error("qgemm (prefill path): grid too large");
        return QARL_ERR_UNSUPPORTED;
    }
    p.m_slots = (int)slots;
    p.total = (int)total;
    const size_t lds = 2 * ((size_t)kBM * kARowB + kBM * 4);
    static LdsLimitOnce once;
    auto kern = qgemm_tile_kernel<EPI, MS>;
    if (int rc = raise_lds_limit((const void *)kern, once, "hipFuncSetAttribute(tile)")) return rc;
    kern<<<dim3((unsigned)total), dim3(kTileThreads), lds, s>>>(p);
    return check_hip(hipGetLastError(), "qgemm_tile_kernel");
}

template <int EPI>
static int launch_one(const GemmArgs &a, hipStream_t s)
{
    return launch_cfg<EPI, 2>(a, s);
}

// sums[row][g] = -1.5 * sum over the 128 k of group g of x[row][k]: the start value of a group's
// accumulator (it cancels the +24/16 offset of the expanded codes).  16 lanes own a group.
__global__ __launch_bounds__(256) void group_sums_kernel(const u32x4 *__restrict__ x, int64_t n_chunks,
                                                         float *__restrict__ sums)
{
    const int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x;  // 16-byte chunk = 8 elements
    u32x4 v = {0, 0, 0, 0};
    if (c < n_chunks) v = x[c];
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) s += __uint_as_float(v[i] << 16) + __uint_as_float(v[i] & 0xffff0000u);
#pragma unroll
    for (int o = 1; o < 16; o <<= 1) s += __shfl_xor(s, o, 64);
    if (c < n_chunks && (c & 15) == 0) sums[c >> 4] = -1.5f * s;
}

int launch_group_sums(const void *x_bf16, int64_t rows, int K, float *sums, hipStream_t s)
{
    const int64_t n_chunks = rows * (int64_t)(K / 8);
    if (n_chunks == 0) return QARL_OK;
    const int64_t blocks = (n_chunks + 255) / 256;
    if (blocks > 0x7fffffffLL) {
        set_error("group sums: grid too large");
        return QARL_ERR_UNSUPPORTED;
    }
    group_sums_kernel<<<dim3((unsigned)blocks), dim3(256), 0, s>>>((const u32x4 *)x_bf16, n_chunks, sums);
    return check_hip(hipGetLastError(), "group_sums_kernel");
}

int launch_qgemm_tile(const GemmArgs &a, hipStream_t s)
{
    if (a.fmt == QARL_W4A16_G128 || a.fmt == QARL_W4A8_G128)
        return a.epilogue == QARL_EPI_SILU_MUL ? launch_one<QARL_EPI_SILU_MUL>(a, s) : launch_one<QARL_EPI_NONE>(a, s);
    return launch_qgemm_tile_fp8(a, s);
}

}  // namespace qarl
