// Grouped quantized GEMM, MFMA-tiled ("prefill" / training-forward) path: the same
// contraction as the weight-streaming path (eq. (1) / eq. (2) of section 2.2), on the same
// codes and scales and with the same exact dequantized weight s*q, for experts that see
// hundreds to thousands of token rows, where the path is a dense contraction.
//
// A workgroup owns a (32*MS)-token x 256-column tile of one expert.  Its wavefronts split the
// columns: each owns 32*NT of them as MS x NT v_mfma_f32_32x32x16 tiles, so no packed weight is
// read or expanded twice in a workgroup.  Token rows are gathered once per workgroup into a
// double-buffered LDS tile (one 128-k scale group per step); packed weights go global ->
// registers and are expanded there, so the LDS only carries the activation operand.  Small
// wavefront tiles (NT = 1) keep the register count at 128, four wavefronts per SIMD from two
// workgroups that run out of step: global-load latency and the VALU work of the expansion are
// hidden by the other wavefronts' MFMAs rather than by a deep software pipeline.
//
// W4A16 group handling is the one described in qgemm_stream.hip: codes become the exact bf16
// values (q+24)/16, every scale group accumulates in its own fp32 accumulator that starts at
// -1.5 * sum_k x (the sums come from a small pre-pass over the activations, once per call), and
// is folded in with one FMA by 16*s.
#include "common.hpp"

namespace qarl {

constexpr int kBN = 256;
constexpr int kAStrideB16 = kGroup * 2 + 16;  // bytes per LDS row, bf16 activations
constexpr int kAStrideF8 = kGroup + 16;       // bytes per LDS row, e4m3 activations

struct TileParams {
    const uint32_t *codes;
    const void *scales;
    const void *x;
    const float *x_scales;
    const float *x_group_sums;
    const int32_t *row_map;
    const int32_t *out_row_map;
    const int32_t *offsets;
    void *out;
    int E, N, K, out_f32;
    int n_blocks;   // column blocks per expert
    int m_slots;    // upper bound of token tiles over all experts
    int total;      // n_blocks * m_slots rounded up to a multiple of 8
};

// MS: 32-row token tiles per wavefront; NT: 32-column tiles per wavefront (256/(32 NT) wavefronts).
template <int FMT, int EPI, int MS, int NT>
__global__ __launch_bounds__(64 * (kBN / (32 * NT)), (NT == 1 ? 4 : 2)) void qgemm_tile_kernel(TileParams p)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr bool kInt4 = (FMT == QARL_W4A16_G128);
    constexpr bool kSilu = (EPI == QARL_EPI_SILU_MUL);
    constexpr int kWaves = kBN / (32 * NT);
    constexpr int kThreads = 64 * kWaves;
    constexpr int kBM = 32 * MS;
    constexpr int kStride = kInt4 ? kAStrideB16 : kAStrideF8;
    constexpr int kBufBytes = kBM * kStride + kBM * 4;  // tile + per-row group sums
    __shared__ int s_rows[kBM];
    __shared__ int s_scan[256];
    __shared__ int s_expert, s_mtile;

    const int tid = threadIdx.x, lane = tid & 63, wn = tid >> 6;
    const int c = lane & 31, h = lane >> 5;

    // workgroup id -> (m slot, column block): consecutive ids go round-robin over the 8 XCDs, so
    // give every XCD a contiguous range of tiles: column blocks of one token tile share its L2.
    const int per_xcd = p.total / 8;
    const int v = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
    const int nb = v % p.n_blocks;
    const int slot = v / p.n_blocks;
    if (slot >= p.m_slots) return;

    // slot -> (expert, tile within expert) by a scan over the per-expert tile counts
    if (tid < 256) {
        int t = 0;
        if (tid < p.E) t = (p.offsets[tid + 1] - p.offsets[tid] + kBM - 1) / kBM;
        s_scan[tid] = t;
    }
    if (tid == 0) s_expert = -1;
    lds_barrier();
    for (int o = 1; o < 256; o <<= 1) {
        int add = 0;
        if (tid < 256 && tid >= o) add = s_scan[tid - o];
        lds_barrier();
        if (tid < 256) s_scan[tid] += add;
        lds_barrier();
    }
    if (tid < p.E) {
        const int incl = s_scan[tid];
        const int excl = tid ? s_scan[tid - 1] : 0;
        if (slot >= excl && slot < incl) {
            s_expert = tid;
            s_mtile = slot - excl;
        }
    }
    lds_barrier();
    const int e = s_expert;
    if (e < 0) return;
    const int row0 = p.offsets[e] + s_mtile * kBM;
    const int mrem = min(kBM, p.offsets[e + 1] - row0);
    if (tid < kBM) {
        const int i = row0 + tid;
        s_rows[tid] = (tid < mrem) ? (p.row_map ? p.row_map[i] : i) : -1;
    }
    lds_barrier();

    const int N = p.N, K = p.K, G = K / kGroup;
    // Weight row of this lane in each of its column tiles (any row may feed any lane of the B
    // operand).  SILU_MUL: gate row j and up row N/2 + j must meet in one lane or in lanes 16 apart:
    //   NT = 2: tile 0 = 32 gate rows, tile 1 = the matching 32 up rows (same lane);
    //   NT = 1: lanes c < 16 take 16 gate rows, lanes c >= 16 the matching up rows (lane ^ 16).
    int nrow[NT];
    bool tile_ok[NT];
    if (kSilu) {
        if (NT == 2) {
            nrow[0] = nb * (kBN / 2) + wn * 32 + c;
            nrow[NT - 1] = N / 2 + nrow[0];
            tile_ok[0] = tile_ok[NT - 1] = nrow[0] - c + 32 <= N / 2;
        } else {
            const int j = nb * (kBN / 2) + wn * 16 + (c & 15);
            nrow[0] = (c < 16 ? 0 : N / 2) + j;
            tile_ok[0] = j - (c & 15) + 16 <= N / 2;
        }
    } else {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            nrow[nt] = nb * kBN + wn * 32 * NT + nt * 32 + c;
            tile_ok[nt] = nrow[nt] - c + 32 <= N;
        }
    }
    const int words_per_row = kInt4 ? K / 8 : K / 4;
    const uint32_t *wrow[NT], *wblk[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int64_t r = (int64_t)e * N + (tile_ok[nt] ? nrow[nt] : 0);
        wrow[nt] = p.codes + r * words_per_row;                      // fp8: row-major
        wblk[nt] = p.codes + (r / 16) * G * 256 + (r % 16) * 4;      // int4: first block of the row's tile
    }

    // ---- activation tile: kBM rows x 128 k, 16-byte blocks; consecutive lanes cover one row
    constexpr int kBlkPerRow = kInt4 ? 16 : 8;
    constexpr int kARegs = (kBM * kBlkPerRow + kThreads - 1) / kThreads;
    u32x4 ar[kARegs];
    float gsum = 0.f;  // W4A16: -1.5 * sum of this thread's row over the group (threads < kBM)
    auto load_a = [&](int g) {
        if (kInt4 && tid < kBM) {
            const int xrow = s_rows[tid];
            gsum = xrow >= 0 ? p.x_group_sums[(int64_t)xrow * G + g] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < kARegs; ++u) {
            const int idx = u * kThreads + tid;
            const int r = idx / kBlkPerRow, b = idx % kBlkPerRow;
            ar[u] = u32x4{0, 0, 0, 0};
            if (r < kBM) {
                const int xrow = s_rows[r];
                if (xrow >= 0)
                    ar[u] = *(const u32x4 *)((const unsigned char *)p.x +
                                             ((int64_t)xrow * K + g * kGroup) * (kInt4 ? 2 : 1) + b * 16);
            }
        }
    };
    auto store_a = [&](int buf) {
        unsigned char *xs = smem + buf * kBufBytes;
        float *sx = (float *)(xs + kBM * kStride);
        if (kInt4 && tid < kBM) sx[tid] = gsum;
#pragma unroll
        for (int u = 0; u < kARegs; ++u) {
            const int idx = u * kThreads + tid;
            const int r = idx / kBlkPerRow, b = idx % kBlkPerRow;
            if (r < kBM) *(u32x4 *)(xs + r * kStride + b * 16) = ar[u];
        }
    };

    // ---- packed weights of one group: lane (c,h) reads k in [128 g + 64 h, +64) of its rows
    constexpr int kWRegs = kInt4 ? 2 : 4;  // 16-byte loads per lane and column tile
    struct BRegs {
        u32x4 w[NT][kWRegs];
        uint32_t s[NT];
    };
    auto load_b = [&](BRegs &dst, int g) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
#pragma unroll
            for (int u = 0; u < kWRegs; ++u) {
                dst.w[nt][u] = u32x4{0, 0, 0, 0};
                if (tile_ok[nt]) {
                    // int4: block (16-row tile, group g) is 1 KiB; this lane's row is r % 16 of tile r / 16 and
                    // it takes the 16-byte pieces q = 2h + u (k in [32 q, +32)).  fp8: row-major bytes.
                    const uint32_t *src = kInt4 ? wblk[nt] + ((int64_t)g * 64 + (2 * h + u) * 16) * 4
                                                : wrow[nt] + (g * 32 + h * 16 + u * 4);
                    dst.w[nt][u] = *(const u32x4 *)src;
                }
            }
            dst.s[nt] = 0;
            if (kInt4 && tile_ok[nt]) dst.s[nt] = ((const uint16_t *)p.scales)[((int64_t)e * N + nrow[nt]) * G + g];
        }
    };

    f32x16 acc[MS][NT];
#pragma unroll
    for (int ms = 0; ms < MS; ++ms)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[ms][nt][i] = 0.f;

    BRegs bcur, bnxt;
    load_a(0);
    load_b(bcur, 0);
    store_a(0);
    lds_barrier();
    for (int g = 0; g < G; ++g) {
        if (g + 1 < G) {
            load_a(g + 1);
            load_b(bnxt, g + 1);
        }
        const unsigned char *xs = smem + (g & 1) * kBufBytes;
        const float *sx = (const float *)(xs + kBM * kStride);
        if (kInt4) {
            f32x16 ag[MS][NT];
#pragma unroll
            for (int ms = 0; ms < MS; ++ms) {
#pragma unroll
                for (int i4 = 0; i4 < 4; ++i4) {
                    const f32x4 init = *(const f32x4 *)(sx + ms * 32 + 8 * i4 + 4 * h);
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                        for (int i = 0; i < 4; ++i) ag[ms][nt][i4 * 4 + i] = init[i];
                }
            }
            if (NT == 1) {
                // four wavefronts per SIMD: the other wavefronts cover LDS latency and code expansion
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const bf16x8 b = unpack_int4_word(bcur.w[0][j >> 2][j & 3]);
#pragma unroll
                    for (int ms = 0; ms < MS; ++ms) {
                        const bf16x8 a = *(const bf16x8 *)(xs + (ms * 32 + c) * kStride + (h * 64 + j * 8) * 2);
                        ag[ms][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, ag[ms][0], 0, 0, 0);
                    }
                }
            } else {
            // Software pipeline over the eight 16-k slices: the LDS reads and the code expansion of
            // slice j+1 are issued under the MFMAs of slice j; the group barriers pin that
            // interleaving (MFMA, LDS read, VALU, MFMA, ...) in the machine schedule.
            bf16x8 a_c[MS], b_c[NT];
#pragma unroll
            for (int ms = 0; ms < MS; ++ms) a_c[ms] = *(const bf16x8 *)(xs + (ms * 32 + c) * kStride + (h * 64) * 2);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) b_c[nt] = unpack_int4_word(bcur.w[nt][0][0]);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                bf16x8 a_n[MS], b_n[NT];
                if (j < 7) {
#pragma unroll
                    for (int ms = 0; ms < MS; ++ms)
                        a_n[ms] = *(const bf16x8 *)(xs + (ms * 32 + c) * kStride + (h * 64 + (j + 1) * 8) * 2);
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt) b_n[nt] = unpack_int4_word(bcur.w[nt][(j + 1) >> 2][(j + 1) & 3]);
                }
#pragma unroll
                for (int ms = 0; ms < MS; ++ms)
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
                        ag[ms][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_c[ms], b_c[nt], ag[ms][nt], 0, 0, 0);
                if (j < 7) {
#pragma unroll
                    for (int t = 0; t < MS * NT; ++t) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                        // MFMA
                        if (t < MS) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);            // LDS read
                        __builtin_amdgcn_sched_group_barrier(0x002, (8 * NT) / (MS * NT), 0);     // VALU
                    }
#pragma unroll
                    for (int ms = 0; ms < MS; ++ms) a_c[ms] = a_n[ms];
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt) b_c[nt] = b_n[nt];
                }
            }
            }
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const float s16 = 16.f * bf16_bits_to_f32(bcur.s[nt]);
#pragma unroll
                for (int ms = 0; ms < MS; ++ms)
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc[ms][nt][i] = fmaf(s16, ag[ms][nt][i], acc[ms][nt][i]);
            }
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                long b[NT];
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    const u32x4 w = bcur.w[nt][j >> 1];
                    b[nt] = (long)(((uint64_t)w[(j & 1) * 2 + 1] << 32) | w[(j & 1) * 2]);
                }
#pragma unroll
                for (int ms = 0; ms < MS; ++ms) {
                    const long a = *(const long *)(xs + (ms * 32 + c) * kStride + h * 64 + j * 8);
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
                        acc[ms][nt] = __builtin_amdgcn_mfma_f32_32x32x16_fp8_fp8(a, b[nt], acc[ms][nt], 0, 0, 0);
                }
            }
        }
        if (g + 1 < G) {
            store_a((g + 1) & 1);
            bcur = bnxt;
        }
        lds_barrier();
    }

    // ---- epilogue: lane (c,h), register i -> token row 8*(i/4) + 4h + i%4, column c of each tile
    float swn[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
        swn[nt] = (!kInt4 && tile_ok[nt]) ? ((const float *)p.scales)[(int64_t)e * N + nrow[nt]] : 1.f;
#pragma unroll
    for (int ms = 0; ms < MS; ++ms) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int r = ms * 32 + 8 * (i >> 2) + 4 * h + (i & 3);
            const bool row_ok = r < mrem;
            const int64_t srow = (int64_t)row0 + (row_ok ? r : 0);
            const int64_t orow = p.out_row_map ? (int64_t)p.out_row_map[srow] : srow;
            float vv[NT];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                vv[nt] = acc[ms][nt][i];
                if (!kInt4) vv[nt] *= (row_ok ? p.x_scales[s_rows[r]] : 0.f) * swn[nt];
            }
            if (kSilu) {
                // gate and up value of the same column: tile 0 / tile 1 (NT = 2) or lanes 16 apart (NT = 1)
                const float gate = vv[0];
                const float up = (NT == 2) ? vv[NT - 1] : __shfl_xor(vv[0], 16, 64);
                const bool writer = (NT == 2) || c < 16;
                if (row_ok && tile_ok[0] && writer) {
                    const float a = gate / (1.f + expf(-gate)) * up;
                    ((uint16_t *)p.out)[orow * (N / 2) + nrow[0]] = (uint16_t)f32_to_bf16_bits(a);
                }
            } else {
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    if (row_ok && tile_ok[nt]) {
                        if (p.out_f32) ((float *)p.out)[orow * N + nrow[nt]] = vv[nt];
                        else ((uint16_t *)p.out)[orow * N + nrow[nt]] = (uint16_t)f32_to_bf16_bits(vv[nt]);
                    }
                }
            }
        }
    }
}

template <int FMT, int EPI, int MS, int NT>
static int launch_cfg(const GemmArgs &a, hipStream_t s)
{
    constexpr bool kInt4 = (FMT == QARL_W4A16_G128);
    constexpr int kBM = 32 * MS;
    constexpr int kThreads = 64 * (kBN / (32 * NT));
    if (a.E > 256) {
        set_error("qgemm (prefill path): at most 256 experts (got %d)", a.E);
        return QARL_ERR_UNSUPPORTED;
    }
    if (a.N % 32 != 0) {
        set_error("qgemm (prefill path): N %% 32 == 0 required (got %d)", a.N);
        return QARL_ERR_UNSUPPORTED;
    }
    TileParams p;
    p.codes = (const uint32_t *)a.codes;
    p.scales = a.scales;
    p.x = a.x;
    p.x_scales = a.x_scales;
    p.x_group_sums = a.x_group_sums;
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
    const int stride = kInt4 ? kAStrideB16 : kAStrideF8;
    const size_t lds = 2 * ((size_t)kBM * stride + kBM * 4);
    static bool attr_done = false;
    auto kern = qgemm_tile_kernel<FMT, EPI, MS, NT>;
    if (!attr_done) {
        int rc = check_hip(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds),
                           "hipFuncSetAttribute(tile)");
        if (rc) return rc;
        attr_done = true;
    }
    kern<<<dim3((unsigned)total), dim3(kThreads), lds, s>>>(p);
    return check_hip(hipGetLastError(), "qgemm_tile_kernel");
}

template <int FMT, int EPI>
static int launch_one(const GemmArgs &a, hipStream_t s)
{
    return launch_cfg<FMT, EPI, 2, 1>(a, s);
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
    if (a.fmt == QARL_W4A16_G128)
        return a.epilogue == QARL_EPI_SILU_MUL ? launch_one<QARL_W4A16_G128, QARL_EPI_SILU_MUL>(a, s)
                                               : launch_one<QARL_W4A16_G128, QARL_EPI_NONE>(a, s);
    return a.epilogue == QARL_EPI_SILU_MUL ? launch_one<QARL_FP8_E4M3_CH, QARL_EPI_SILU_MUL>(a, s)
                                           : launch_one<QARL_FP8_E4M3_CH, QARL_EPI_NONE>(a, s);
}

}  // namespace qarl
