// Grouped quantized GEMM, weight-streaming ("decode") path: eq. (1) / eq. (2) of
// section 2.2 when every expert sees only a few token rows, so the kernel is bound by
// reading each expert's packed weights from HBM exactly once.
//
// Layout of the work: a workgroup of 4 wavefronts owns (expert, block of weight rows);
// each wavefront owns two 16-row weight tiles for the whole K and up to 64 token rows.
// Packed codes go global -> registers (one 16-byte load per lane and scale group, 64
// contiguous bytes per weight row), are expanded in registers to bf16 MFMA operands, and
// meet the token rows, staged once per workgroup in LDS, in v_mfma_f32_16x16x32.
//
// W4A16 numerics: the dequantized weight is s*q exactly.  The nibble u = q+8 is placed in
// the top mantissa bits of bf16 1.0, giving the exact bf16 value (q+24)/16 with one shift
// and one and-or per two codes.  Each 128-k scale group accumulates in its own fp32 MFMA
// accumulator, started at -1.5 * sum_k x (which cancels the +24/16 offset), and is folded
// into the running sum with one fp32 FMA by 16*s.  A one-hot activation row therefore
// reproduces s*q bit for bit.
#include <math.h>

#include "common.hpp"

namespace qarl {

constexpr int kSThreads = 256;
constexpr int kSWaves = 4;
constexpr int kMT = 4;                 // 16-row token tiles per pass (64 rows)
constexpr int kRows = kMT * 16;
constexpr int kMaxGC = 4;              // scale groups (128 k) per staged chunk, at most
// LDS row stride in bytes: the chunk's k plus 16 bytes, so consecutive rows skew by 4 banks
__host__ __device__ constexpr int x_stride(bool int4, int gc) { return gc * kGroup * (int4 ? 2 : 1) + 16; }

struct StreamParams {
    const uint32_t *codes;   // int4: [E][N][K/8] words; fp8: bytes viewed as words [E][N][K/4]
    const void *scales;      // int4: bf16 [E][N][K/128]; fp8: float [E][N]
    const void *x;           // bf16 or e4m3 rows
    const float *x_scales;   // fp8 only
    const int32_t *row_map;
    const int32_t *out_row_map;
    const int32_t *offsets;
    void *out;
    int N, K, out_f32, n_units;  // n_units: wave work items per expert (tile pairs)
};

__device__ __forceinline__ bf16x8 unpack_int4_word(uint32_t w)
{
    // -> bf16 pairs (c0,c4) (c1,c5) (c2,c6) (c3,c7), each (q+24)/16
    u32x4 d;
    d[0] = ((w << 3) & 0x00780078u) | 0x3f803f80u;
    d[1] = ((w >> 1) & 0x00780078u) | 0x3f803f80u;
    d[2] = ((w >> 5) & 0x00780078u) | 0x3f803f80u;
    d[3] = ((w >> 9) & 0x00780078u) | 0x3f803f80u;
    return __builtin_bit_cast(bf16x8, d);
}

template <int GC, int WH>
struct WRegs {
    u32x4 w[2][GC][WH];  // [tile][group in chunk][16-byte part]
    uint32_t s[2][GC];   // int4: bf16 scale bits
};

// One pass over the whole K for up to MTC*16 token rows of expert e, GC scale groups per chunk.
template <int FMT, int EPI, int MTC, int GC>
__device__ __forceinline__ void stream_pass(const StreamParams &p, unsigned char *smem, int e, int row0, int m0,
                                            int mrem, const int (&nrow)[2], const bool (&tile_ok)[2],
                                            const uint32_t *const (&wrow)[2])
{
    constexpr bool kInt4 = (FMT == QARL_W4A16_G128);
    constexpr int kKC = GC * kGroup;
    constexpr int kStride = x_stride(kInt4, GC);
    constexpr int kWH = kInt4 ? 1 : 2;
    int *s_row = (int *)smem;                                       // [kRows] activation row ids
    float *sx = (float *)(smem + kRows * 4);                        // int4: [GC][kRows]  -1.5 * group sums
    unsigned char *xs = smem + kRows * 4 + kMaxGC * kRows * 4;      // [MTC*16][kStride]

    const int tid = threadIdx.x, lane = tid & 63;
    const int c = lane & 15, q = lane >> 4;
    const int N = p.N, K = p.K;
    const int G = K / kGroup;
    const int n_chunks = (K + kKC - 1) / kKC;

    __syncthreads();
    if (tid < kRows) {
        int i = row0 + m0 + tid;
        s_row[tid] = (tid < mrem) ? (p.row_map ? p.row_map[i] : i) : -1;
    }
    __syncthreads();

    f32x4 acc[2][MTC];
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int mt = 0; mt < MTC; ++mt) acc[nt][mt] = f32x4{0.f, 0.f, 0.f, 0.f};

    // activation chunk: 16-byte blocks, row-major, prefetched into registers
    constexpr int kBlkPerRow = kInt4 ? kKC / 8 : kKC / 16;        // 64 or 32
    constexpr int kXRegs = MTC * 16 * kBlkPerRow / kSThreads;     // 4*MTC or 2*MTC
    u32x4 xr[kXRegs];
    auto load_x = [&](int kc) {
        const int nblk = min(kBlkPerRow, (K - kc * kKC) / (kInt4 ? 8 : 16));
#pragma unroll
        for (int u = 0; u < kXRegs; ++u) {
            const int idx = u * kSThreads + tid;
            const int r = idx / kBlkPerRow, b = idx % kBlkPerRow;
            const int xrow = s_row[r];
            xr[u] = u32x4{0, 0, 0, 0};
            if (xrow >= 0 && b < nblk) {
                const unsigned char *src =
                    (const unsigned char *)p.x + ((int64_t)xrow * K + kc * kKC) * (kInt4 ? 2 : 1) + b * 16;
                xr[u] = *(const u32x4 *)src;
            }
        }
    };
    auto store_x = [&]() {
#pragma unroll
        for (int u = 0; u < kXRegs; ++u) {
            const int idx = u * kSThreads + tid;
            const int r = idx / kBlkPerRow, b = idx % kBlkPerRow;
            u32x4 v = xr[u];
            if (kInt4) {
                // sum of the 8 values, then over the 16 lanes that hold one scale group of one row
                float sum = 0.f;
#pragma unroll
                for (int i = 0; i < 4; ++i) sum += __uint_as_float(v[i] << 16) + __uint_as_float(v[i] & 0xffff0000u);
#pragma unroll
                for (int o = 1; o < 16; o <<= 1) sum += __shfl_xor(sum, o, 64);
                if ((b & 15) == 0) sx[(b >> 4) * kRows + r] = -1.5f * sum;
                // element order inside an 8-block follows the unpacked code order 0,4,1,5,2,6,3,7
                u32x4 o4;
                o4[0] = (v[0] & 0xffffu) | (v[2] << 16);
                o4[1] = (v[0] >> 16) | (v[2] & 0xffff0000u);
                o4[2] = (v[1] & 0xffffu) | (v[3] << 16);
                o4[3] = (v[1] >> 16) | (v[3] & 0xffff0000u);
                v = o4;
            }
            *(u32x4 *)(xs + r * kStride + b * 16) = v;
        }
    };
    // packed weights (+ scales) of one chunk: lane (c,q) reads k in [128 g + 32 q, +32) of its rows
    auto load_w = [&](WRegs<GC, kWH> &dst, int kc) {
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
            for (int gl = 0; gl < GC; ++gl) {
                const int g = kc * GC + gl;
                const bool ok = tile_ok[nt] && g < G;
#pragma unroll
                for (int h = 0; h < kWH; ++h) {
                    dst.w[nt][gl][h] = u32x4{0, 0, 0, 0};
                    if (ok) {
                        const uint32_t *src = wrow[nt] + (kInt4 ? (g * 16 + q * 4) : (g * 32 + q * 8 + h * 4));
                        dst.w[nt][gl][h] = __builtin_nontemporal_load((const u32x4 *)src);
                    }
                }
                if (kInt4) {
                    dst.s[nt][gl] = 0;
                    if (ok) dst.s[nt][gl] = ((const uint16_t *)p.scales)[((int64_t)e * N + nrow[nt]) * G + g];
                }
            }
    };

    WRegs<GC, kWH> wcur, wnxt;
    load_x(0);
    load_w(wcur, 0);
    for (int kc = 0; kc < n_chunks; ++kc) {
        __syncthreads();  // the previous chunk's LDS readers are done
        store_x();
        __syncthreads();
        if (kc + 1 < n_chunks) {
            load_x(kc + 1);
            load_w(wnxt, kc + 1);
        }
        const int ng = min(GC, G - kc * GC);
#pragma unroll
        for (int gl = 0; gl < GC; ++gl) {
            if (gl < ng) {
                f32x4 ag[2][MTC];
                if (kInt4) {
#pragma unroll
                    for (int mt = 0; mt < MTC; ++mt) {
                        const f32x4 init = *(const f32x4 *)(sx + gl * kRows + mt * 16 + 4 * q);
                        ag[0][mt] = init;
                        ag[1][mt] = init;
                    }
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (kInt4) {
                        const bf16x8 b0 = unpack_int4_word(wcur.w[0][gl][0][j]);
                        const bf16x8 b1 = unpack_int4_word(wcur.w[1][gl][0][j]);
#pragma unroll
                        for (int mt = 0; mt < MTC; ++mt) {
                            const bf16x8 a =
                                *(const bf16x8 *)(xs + (mt * 16 + c) * kStride + (gl * 128 + q * 32 + j * 8) * 2);
                            ag[0][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b0, ag[0][mt], 0, 0, 0);
                            ag[1][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b1, ag[1][mt], 0, 0, 0);
                        }
                    } else {
                        const u32x4 w0 = wcur.w[0][gl][j >> 1], w1 = wcur.w[1][gl][j >> 1];
                        const long b0 = (long)(((uint64_t)w0[(j & 1) * 2 + 1] << 32) | w0[(j & 1) * 2]);
                        const long b1 = (long)(((uint64_t)w1[(j & 1) * 2 + 1] << 32) | w1[(j & 1) * 2]);
#pragma unroll
                        for (int mt = 0; mt < MTC; ++mt) {
                            const long a = *(const long *)(xs + (mt * 16 + c) * kStride + gl * 128 + q * 32 + j * 8);
                            acc[0][mt] = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(a, b0, acc[0][mt], 0, 0, 0);
                            acc[1][mt] = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(a, b1, acc[1][mt], 0, 0, 0);
                        }
                    }
                }
                if (kInt4) {
#pragma unroll
                    for (int nt = 0; nt < 2; ++nt) {
                        const float s16 = 16.f * bf16_bits_to_f32(wcur.s[nt][gl]);
#pragma unroll
                        for (int mt = 0; mt < MTC; ++mt)
#pragma unroll
                            for (int i = 0; i < 4; ++i) acc[nt][mt][i] = fmaf(s16, ag[nt][mt][i], acc[nt][mt][i]);
                    }
                }
            }
        }
        if (kc + 1 < n_chunks) wcur = wnxt;
    }

    // epilogue: lane (c,q) holds rows 4q..4q+3 of each token tile, column c of each weight tile
    float swn[2] = {1.f, 1.f};
    if (!kInt4) {
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) swn[nt] = tile_ok[nt] ? ((const float *)p.scales)[(int64_t)e * N + nrow[nt]] : 0.f;
    }
#pragma unroll
    for (int mt = 0; mt < MTC; ++mt) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int r = mt * 16 + 4 * q + i;
            if (r < mrem) {
                const int64_t srow = (int64_t)row0 + m0 + r;
                const int64_t orow = p.out_row_map ? (int64_t)p.out_row_map[srow] : srow;
                float v0 = acc[0][mt][i], v1 = acc[1][mt][i];
                if (!kInt4) {
                    const float sxr = p.x_scales[s_row[r]];
                    v0 *= sxr * swn[0];
                    v1 *= sxr * swn[1];
                }
                if (EPI == QARL_EPI_SILU_MUL) {
                    if (tile_ok[0]) {
                        const float a = v0 / (1.f + expf(-v0)) * v1;
                        ((uint16_t *)p.out)[orow * (N / 2) + nrow[0]] = (uint16_t)f32_to_bf16_bits(a);
                    }
                } else if (p.out_f32) {
                    if (tile_ok[0]) ((float *)p.out)[orow * N + nrow[0]] = v0;
                    if (tile_ok[1]) ((float *)p.out)[orow * N + nrow[1]] = v1;
                } else {
                    if (tile_ok[0]) ((uint16_t *)p.out)[orow * N + nrow[0]] = (uint16_t)f32_to_bf16_bits(v0);
                    if (tile_ok[1]) ((uint16_t *)p.out)[orow * N + nrow[1]] = (uint16_t)f32_to_bf16_bits(v1);
                }
            }
        }
    }
}

// MT = 16-row token tiles held per pass.  The host picks it from the mean rows per expert; an
// expert with more rows than 16*MT takes further passes over its weights.
template <int FMT, int EPI, int MT>
__global__ __launch_bounds__(kSThreads, 2) void qgemm_stream_kernel(StreamParams p)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr bool kInt4 = (FMT == QARL_W4A16_G128);
    constexpr int GC = (MT <= 2) ? 4 : 2;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 15;
    const int e = blockIdx.y;
    const int row0 = p.offsets[e];
    const int Me = p.offsets[e + 1] - row0;
    if (Me <= 0) return;

    const int N = p.N;
    const int unit = blockIdx.x * kSWaves + wave;
    const bool active = unit < p.n_units;
    int nrow[2];  // weight rows of this lane's two tiles
    if (EPI == QARL_EPI_SILU_MUL) {
        nrow[0] = unit * 16 + c;
        nrow[1] = N / 2 + unit * 16 + c;
    } else {
        nrow[0] = unit * 32 + c;
        nrow[1] = unit * 32 + 16 + c;
    }
    bool tile_ok[2];
    tile_ok[0] = active && nrow[0] - c + 16 <= N;
    tile_ok[1] = active && nrow[1] - c + 16 <= N;
    const int words_per_row = kInt4 ? p.K / 8 : p.K / 4;
    const uint32_t *wrow[2];
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
        wrow[nt] = p.codes + ((int64_t)e * N + (tile_ok[nt] ? nrow[nt] : 0)) * words_per_row;

    for (int m0 = 0; m0 < Me; m0 += MT * 16)
        stream_pass<FMT, EPI, MT, GC>(p, smem, e, row0, m0, min(MT * 16, Me - m0), nrow, tile_ok, wrow);
}

template <int FMT, int EPI, int MT>
static int launch_mt(const StreamParams &p, int E, hipStream_t s)
{
    constexpr bool kInt4 = (FMT == QARL_W4A16_G128);
    constexpr int GC = (MT <= 2) ? 4 : 2;
    const size_t lds = (size_t)MT * 16 * x_stride(kInt4, GC) + (size_t)kMaxGC * kRows * 4 + kRows * 4;
    static bool attr_done = false;
    auto kern = qgemm_stream_kernel<FMT, EPI, MT>;
    if (!attr_done) {
        int rc = check_hip(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds),
                           "hipFuncSetAttribute(stream)");
        if (rc) return rc;
        attr_done = true;
    }
    dim3 grid((p.n_units + kSWaves - 1) / kSWaves, E);
    kern<<<grid, dim3(kSThreads), lds, s>>>(p);
    return check_hip(hipGetLastError(), "qgemm_stream_kernel");
}

template <int FMT, int EPI>
static int launch_one(const GemmArgs &a, hipStream_t s)
{
    StreamParams p;
    p.codes = (const uint32_t *)a.codes;
    p.scales = a.scales;
    p.x = a.x;
    p.x_scales = a.x_scales;
    p.row_map = a.row_map;
    p.out_row_map = a.out_row_map;
    p.offsets = a.offsets;
    p.out = a.out;
    p.N = a.N;
    p.K = a.K;
    p.out_f32 = a.out_f32;
    p.n_units = (EPI == QARL_EPI_SILU_MUL) ? (a.N / 2) / 16 : (a.N + 31) / 32;
    // token tiles per pass from the mean rows per expert (mean + 4 sigma of a uniform router fits)
    const double mean = (double)a.M / (double)a.E;
    const double need = mean + 4.0 * sqrt(mean);
    if (need <= 16.0) return launch_mt<FMT, EPI, 1>(p, a.E, s);
    if (need <= 32.0) return launch_mt<FMT, EPI, 2>(p, a.E, s);
    return launch_mt<FMT, EPI, 4>(p, a.E, s);
}

int launch_qgemm_stream(const GemmArgs &a, hipStream_t s)
{
    if (a.fmt == QARL_W4A16_G128)
        return a.epilogue == QARL_EPI_SILU_MUL ? launch_one<QARL_W4A16_G128, QARL_EPI_SILU_MUL>(a, s)
                                               : launch_one<QARL_W4A16_G128, QARL_EPI_NONE>(a, s);
    return a.epilogue == QARL_EPI_SILU_MUL ? launch_one<QARL_FP8_E4M3_CH, QARL_EPI_SILU_MUL>(a, s)
                                           : launch_one<QARL_FP8_E4M3_CH, QARL_EPI_NONE>(a, s);
}

}  // namespace qarl
