// Grouped quantized GEMM, weight-streaming ("decode") path for the FP8 format: eq. (2) of
// section 2.2 when every expert sees only a few token rows, so the kernel is bound by
// reading each expert's e4m3 weights from HBM exactly once (the regime the paper's
// appendix on quantization schemes calls memory-bound).  The W4A16 format has its own
// kernel (qgemm_stream_w4.hip); this file also holds the dispatch between the two.
//
// Work layout.  A workgroup of 8 wavefronts owns (expert, slice of its weight rows, block
// of <= 16*MT token rows).  It gathers its e4m3 token rows ONCE into LDS for the whole K;
// after that single barrier every wavefront runs on its own: it walks its pairs of 16-row
// weight tiles and, per pair, K in steps of 128, with the codes of the next R steps always
// in flight in a register ring (global -> registers, two 16-byte loads per lane, tile and
// step: lane (c, q) reads k in [128 g + 32 q, +32) of row c).  Codes and token rows meet as
// stored in v_mfma_f32_16x16x32_fp8_fp8; the row scale s_x and the channel scale s_w are
// applied to the fp32 sums in the epilogue.
//
// Experts with more than 16*MT rows: the grid carries m_split row blocks per (expert,
// slice), mapped to consecutive workgroups of the same XCD so that their identical weight
// reads meet in that XCD's L2; rows beyond 16*MT*m_split take further passes.
//
// Routed mode (QX): the kernel is driven by the router's ids and by 16-bit activations.  Every
// workgroup lists its expert's (token, slot) pairs itself and quantizes the token rows it
// gathers with the row quantizer's own arithmetic (one wavefront per row: absmax, s_x =
// absmax / 448, e4m3 codes of x / s_x), so a decode step needs neither a grouping pass nor an
// activation-quantizer launch between the router and the two expert GEMMs, and its results
// equal theirs bit for bit.
#include <math.h>

#include <type_traits>

#include "common.hpp"

namespace qarl {

namespace {

constexpr int kSThreads = 512;
constexpr int kSWaves = 8;

struct StreamParams {
    const uint32_t *codes;   // e4m3 bytes viewed as words [E][N][K/4]
    const float *scales;     // [E][N]
    const void *x;           // e4m3 rows
    const float *x_scales;
    const int32_t *row_map;
    const int32_t *out_row_map;
    const int32_t *offsets;
    void *out;
    int E, N, K, out_f32;
    int n_units;     // pairs of 16-row weight tiles per expert
    int n_slices;    // workgroups along the weight rows of one expert
    int m_split;     // row blocks per (expert, slice) in the grid
    int w4;          // weights are packed e2m1 codes [E][N][K/8] words
    // routed mode: x is bf16; row = pair id t * topk + slot of expert ids[row], activation row t (x_per_token)
    // or the pair id, output row = pair id
    const int32_t *ids;
    int n_ids, topk, x_per_token;
};

constexpr int kIdsMax = 4096;    // pairs a workgroup scans (8 per thread)
constexpr int kIdsRows = 512;    // rows of one expert it can list: one per token, T <= 512

// LDS bytes per activation row: the row plus 16 bytes, so consecutive rows skew by 4 banks.
__host__ __device__ constexpr int x_stride(int K) { return K + 16; }

// Dynamic LDS of a workgroup: row ids, output rows, row scales, pair counter, token tile.
size_t stream_lds_bytes(int K, int MT, bool routed = false)
{
    const size_t rows = (size_t)MT * 16;
    return rows * 12 + 16 + rows * x_stride(K) + (routed ? 8 * (size_t)kIdsRows + 4 * kSWaves : 0);
}

// e2m1 magnitude code (3 bits) -> e4m3 byte of the same value: 0, 0.5, 1, 1.5 | 2, 3, 4, 6.  Every e2m1 value is
// an e4m3 value, so FP4 weights are widened in registers (one byte permute per four codes) and meet the e4m3
// token rows in the same matrix instruction as FP8 weights do.
constexpr uint32_t kE2m1LutLo = 0x3c383000u, kE2m1LutHi = 0x4c484440u;

// A word of eight packed e2m1 codes (byte b: element b in the low nibble, element 4 + b in the high nibble)
// -> the eight e4m3 bytes in element order.
__device__ __forceinline__ u32x2 widen_e2m1_word(uint32_t w)
{
    u32x2 o;
    o[0] = __builtin_amdgcn_perm(kE2m1LutHi, kE2m1LutLo, w & 0x07070707u) | ((w & 0x08080808u) << 4);
    o[1] = __builtin_amdgcn_perm(kE2m1LutHi, kE2m1LutLo, (w >> 4) & 0x07070707u) | (w & 0x80808080u);
    return o;
}

// EPI: NONE or SILU_MUL; MT: 16-row token tiles per block; R: ring depth in 128-k steps (must divide K/128);
// W4: the weights are packed e2m1 codes (half a byte per weight) instead of e4m3 bytes; QX: routed mode.
template <int EPI, int MT, int R, bool W4, bool QX>
__global__ __launch_bounds__(kSThreads, 1) void qgemm_stream_fp8_kernel(StreamParams p)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr int kRowsMax = MT * 16;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, q = lane >> 4;
    const int N = p.N, K = p.K, G = K / kGroup;
    const int stride = x_stride(K);

    // workgroup id -> (expert, slice, row block).  Ids go round-robin over the 8 XCDs; the row
    // blocks of one (expert, slice) take consecutive positions on the same XCD.
    const int xcd = blockIdx.x & 7, pos = blockIdx.x >> 3;
    const int mh = pos % p.m_split;
    const int unit_id = (pos / p.m_split) * 8 + xcd;
    if (unit_id >= p.E * p.n_slices) return;
    const int e = unit_id / p.n_slices, slice = unit_id % p.n_slices;

    int *s_row = (int *)smem;                              // [kRowsMax] activation row of each tile row
    int *s_orow = (int *)(smem + kRowsMax * 4);            // [kRowsMax] output row, -1 past the expert's last row
    float *s_xs = (float *)(smem + kRowsMax * 8);          // [kRowsMax] activation scale of the row
    int *s_next = (int *)(smem + kRowsMax * 12);           // next undrawn pair
    unsigned char *xs = smem + kRowsMax * 12 + 16;         // [kRowsMax][stride]

    // this workgroup's pairs of weight tiles: units u_lo .. u_hi-1
    const int per_slice = (p.n_units + p.n_slices - 1) / p.n_slices;
    const int u_lo = slice * per_slice, u_hi = min(p.n_units, u_lo + per_slice);
    const int n_pairs = max(0, u_hi - u_lo);  // pairs of this workgroup; wavefronts draw them from an LDS counter
    const int words_per_row = W4 ? K / 8 : K / 4;
    const int64_t ebase = (int64_t)e * N;

    auto tile_row = [&](int pi, int nt) -> int {  // weight row of this lane in tile nt of the slice's pi-th pair
        const int u = u_lo + pi;
        if (EPI == QARL_EPI_SILU_MUL) return (nt ? N / 2 : 0) + u * 16 + c;
        return u * 32 + nt * 16 + c;
    };

    constexpr int kH = W4 ? 1 : 2;   // 16-byte loads per lane, tile and 128-k step: 32 weights of one row
    struct Slot {
        u32x4 w[2][kH];
    };
    Slot ring[R];
    // Base pointer of the R-step batch (pair pi, steps g0..) of tile nt for this lane.  Past this
    // wavefront's work the pointer falls back to the start of the expert's codes: the ring is refilled
    // without a branch (a conditional refill turns every slot into a merge of old and new value and
    // doubles the registers the ring takes), and those few loads all hit one cached line.
    auto batch_src = [&](int pi, int g0, int nt) -> const uint32_t * {
        const bool ok = pi < n_pairs;
        const int64_t row = ebase + (ok ? tile_row(pi, nt) : c);
        return p.codes + row * words_per_row + (ok ? g0 * (8 * kH * 2) + q * (4 * kH) : 0);
    };
    // Plain (temporal) loads on purpose: with row-major codes one load instruction takes half of each
    // 128-byte line it touches and the h = 1 load the other half.  A nontemporal load drops the line
    // after the first half and fetches it again for the second (measured: 7 % of the 256-token layer,
    // 16 % at 512 tokens).
    auto fill = [&](Slot &dst, int r, const uint32_t *const (&src)[2]) {
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
            for (int h = 0; h < kH; ++h) dst.w[nt][h] = *(const u32x4 *)(src[nt] + r * (16 * kH) + h * 4);
    };
    auto fill_ring = [&](int pi, int g0) {
        const uint32_t *src[2] = {batch_src(pi, g0, 0), batch_src(pi, g0, 1)};
#pragma unroll
        for (int r = 0; r < R; ++r) fill(ring[r], r, src);
    };

    int row0, Me;
    int *tmp_map = (int *)(xs + kRowsMax * stride);   // routed mode: [kIdsRows] activation rows, [kIdsRows] pair ids, [kSWaves] counts
    if (QX) {
        // Thread tid looks at pairs 8 tid .. 8 tid + 7.  Matches keep their order: the rows of an expert are its
        // pairs by increasing pair id, the (token, slot) order a stable grouping gives.
        const int base = tid * 8;
        uint32_t hits = 0;
#pragma unroll
        for (int q4 = 0; q4 < 2; ++q4) {
            const int b4 = base + 4 * q4;
            i32x4 v4 = {-1, -1, -1, -1};
            if (b4 + 3 < p.n_ids) {
                v4 = *(const i32x4 *)(p.ids + b4);
            } else {
                for (int k = 0; b4 + k < p.n_ids; ++k) v4[k] = p.ids[b4 + k];
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) hits |= (v4[k] == e) ? (1u << (4 * q4 + k)) : 0u;
        }
        const int cnt = __popc(hits);
        int incl = cnt;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int up = __shfl_up(incl, o, 64);
            if (lane >= o) incl += up;
        }
        int *s_wcnt = tmp_map + 2 * kIdsRows;
        if (lane == 63) s_wcnt[wave] = incl;
        lds_barrier();
        int before = 0, total = 0;
#pragma unroll
        for (int w = 0; w < kSWaves; ++w) {
            const int cw = s_wcnt[w];
            before += w < wave ? cw : 0;
            total += cw;
        }
        int rank = before + incl - cnt;
        for (uint32_t hm = hits; hm; hm &= hm - 1) {
            const int pr = base + __builtin_ctz(hm);
            if (rank < kIdsRows) {
                tmp_map[rank] = p.x_per_token ? pr / p.topk : pr;
                tmp_map[kIdsRows + rank] = pr;
            }
            ++rank;
        }
        row0 = 0;
        Me = min(total, kIdsRows);
    } else {
        row0 = p.offsets[e];
        Me = p.offsets[e + 1] - row0;
    }
    if (Me <= mh * kRowsMax) return;

    for (int m0 = mh * kRowsMax; m0 < Me; m0 += kRowsMax * p.m_split) {
        const int mrem = min(kRowsMax, Me - m0);
        lds_barrier();  // the pair list is complete / the previous pass is done with the LDS tile
        if (tid < kRowsMax) {
            const int i = row0 + m0 + tid;
            if (QX) {
                s_row[tid] = (tid < mrem) ? tmp_map[i] : -1;
                s_orow[tid] = (tid < mrem) ? tmp_map[kIdsRows + i] : -1;
            } else {
                s_row[tid] = (tid < mrem) ? (p.row_map ? p.row_map[i] : i) : -1;
                s_orow[tid] = (tid < mrem) ? (p.out_row_map ? p.out_row_map[i] : i) : -1;
                s_xs[tid] = (tid < mrem) ? p.x_scales[p.row_map ? p.row_map[i] : i] : 0.f;
            }
        }
        if (tid == 0) *s_next = kSWaves;  // pairs 0..7 start on wavefronts 0..7, the rest are drawn
        lds_barrier();
        // ---- gather the token rows into LDS (whole K) in 16-byte blocks.  A thread keeps one block
        // column and walks down the rows (at most kBatch of them: the workgroup sweeps >= 2 rows at a
        // time), so the only index arithmetic is an add per block, and all its loads are in flight at
        // once.  Vector loads return in order: the token rows are requested first and the weight
        // stream right behind them, so it flows in while the tile is being built.
        if (QX) {
            // ---- routed mode: 16-bit token rows, quantized on their way into LDS.  One wavefront per row (rows
            // wave, wave + 8, ...): lane L holds the 16-byte chunks L, L + 64, ... of the row, the row's absmax is
            // a wavefront reduction, and the codes are the row quantizer's (same scale, same division, same
            // conversion).  Rows past the expert's end are left alone: a tile row feeds only its own output row,
            // which is never stored.
            const int n16 = K / 8;   // chunks of 8 values per row
            auto gather_q = [&](auto rows_c, auto kch_c, int rbase, bool first) {
                constexpr int ROWS = decltype(rows_c)::value, KCH = decltype(kch_c)::value;
                u32x4 v[ROWS][KCH];
                int xrow[ROWS];
#pragma unroll
                for (int rr = 0; rr < ROWS; ++rr) {
                    xrow[rr] = __builtin_amdgcn_readfirstlane(s_row[rbase + rr * kSWaves + wave]);
#pragma unroll
                    for (int u = 0; u < KCH; ++u) {
                        const int ch = lane + 64 * u;
                        v[rr][u] = u32x4{0, 0, 0, 0};
                        if (xrow[rr] >= 0 && ch < n16)
                            v[rr][u] = *(const u32x4 *)((const unsigned char *)p.x + ((int64_t)xrow[rr] * K + ch * 8) * 2);
                    }
                }
                if (first) fill_ring(wave, 0);   // the weight stream is requested right behind the token rows
#pragma unroll
                for (int rr = 0; rr < ROWS; ++rr) {
                    if (xrow[rr] < 0) continue;
                    const int r = rbase + rr * kSWaves + wave;
                    float am = 0.f;
#pragma unroll
                    for (int u = 0; u < KCH; ++u) am = absmax_bf16x8(v[rr][u], am);
                    am = wave_max(am);
                    const float sxr = am / 448.0f;
                    const RowScale rs(sxr);
#pragma unroll
                    for (int u = 0; u < KCH; ++u) {
                        const int ch = lane + 64 * u;
                        if (ch < n16) *(u32x2 *)(xs + r * stride + ch * 8) = e4m3_quantize_bf16x8(rs, v[rr][u]);
                    }
                    if (lane == 0) s_xs[r] = sxr;
                }
            };
            if (n16 <= 4 * 64) {
                gather_q(std::integral_constant<int, 2 * MT>(), std::integral_constant<int, 4>(), 0, true);
            } else {
#pragma unroll 1
                for (int i = 0; i < MT; ++i)
                    gather_q(std::integral_constant<int, 2>(), std::integral_constant<int, 8>(), i * 16, i == 0);   // rows 16 i + wave, + 8
            }
        } else {
            const int bpr = K / 16;                      // blocks per row
            const int rpp = kSThreads / bpr;             // rows covered per sweep of the workgroup
            const int rsub = tid / bpr, b = tid - rsub * bpr;
            const bool active = rsub < rpp;
            constexpr int kBatch = 16;
            u32x4 v[kBatch];
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                const int r = rsub + u * rpp;
                v[u] = u32x4{0, 0, 0, 0};
                if (active && r < kRowsMax) {
                    const int xrow = s_row[r];
                    if (xrow >= 0)
                        v[u] = *(const u32x4 *)((const unsigned char *)p.x + (int64_t)xrow * K + b * 16);
                }
            }
            fill_ring(wave, 0);
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                const int r = rsub + u * rpp;
                const u32x4 o4 = v[u];
                if (active && r < kRowsMax) *(u32x4 *)(xs + r * stride + b * 16) = o4;
            }
        }
        lds_barrier();

        // ---- stream this wavefront's weight tiles
        // Wavefronts draw pairs from the LDS counter one pair ahead, so the two wavefronts that share a
        // SIMD (one of which the arbiter favours) finish together instead of the slower one trailing.
        for (int pi = wave; pi < n_pairs;) {
            int npi = 0;
            if (lane == 0) npi = atomicAdd(s_next, 1);
            npi = __builtin_amdgcn_readfirstlane(npi);
            f32x4 acc[2][MT];
#pragma unroll
            for (int nt = 0; nt < 2; ++nt)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) acc[nt][mt] = f32x4{0.f, 0.f, 0.f, 0.f};
            for (int g0 = 0; g0 < G; g0 += R) {
                // the batch that refills the ring while this one is consumed: same pair or the next one
                const bool same = g0 + R < G;
                const uint32_t *nsrc[2] = {batch_src(same ? pi : npi, same ? g0 + R : 0, 0),
                                           batch_src(same ? pi : npi, same ? g0 + R : 0, 1)};
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    const int g = g0 + r;
                    Slot &cur = ring[r];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        long b0, b1;   // the 8 weights k = 8 j .. 8 j + 7 of this lane's row in either tile
                        if (W4) {
                            const u32x2 e0 = widen_e2m1_word(cur.w[0][0][j]), e1 = widen_e2m1_word(cur.w[1][0][j]);
                            b0 = (long)(((uint64_t)e0[1] << 32) | e0[0]);
                            b1 = (long)(((uint64_t)e1[1] << 32) | e1[0]);
                        } else {
                            const u32x4 w0 = cur.w[0][(j >> 1) % kH], w1 = cur.w[1][(j >> 1) % kH];
                            b0 = (long)(((uint64_t)w0[(j & 1) * 2 + 1] << 32) | w0[(j & 1) * 2]);
                            b1 = (long)(((uint64_t)w1[(j & 1) * 2 + 1] << 32) | w1[(j & 1) * 2]);
                        }
#pragma unroll
                        for (int mt = 0; mt < MT; ++mt) {
                            const long a = *(const long *)(xs + (mt * 16 + c) * stride + g * 128 + q * 32 + j * 8);
                            acc[0][mt] = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(a, b0, acc[0][mt], 0, 0, 0);
                            acc[1][mt] = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(a, b1, acc[1][mt], 0, 0, 0);
                        }
                    }
                    // refill this slot with the step R ahead
                    fill(cur, r, nsrc);
                }
            }
            // ---- epilogue of this pair: lane (c,q) holds rows 4q..4q+3 of each token tile, column c
            const int n0 = tile_row(pi, 0), n1 = tile_row(pi, 1);
            const float sw0 = p.scales[ebase + n0], sw1 = p.scales[ebase + n1];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int r = mt * 16 + 4 * q + i;
                    const int64_t orow = s_orow[r];
                    if (orow >= 0) {
                        const float sxr = s_xs[r];
                        const float v0 = acc[0][mt][i] * (sxr * sw0), v1 = acc[1][mt][i] * (sxr * sw1);
                        if (EPI == QARL_EPI_SILU_MUL) {
                            const float a = silu_mul_f32(v0, v1);
                            ((uint16_t *)p.out)[orow * (N / 2) + n0] = f32_to_bf16_hw(a);
                        } else if (p.out_f32) {
                            ((float *)p.out)[orow * N + n0] = v0;
                            ((float *)p.out)[orow * N + n1] = v1;
                        } else {
                            ((uint16_t *)p.out)[orow * N + n0] = f32_to_bf16_hw(v0);
                            ((uint16_t *)p.out)[orow * N + n1] = f32_to_bf16_hw(v1);
                        }
                    }
                }
            }
            pi = npi;
        }
    }
}

template <int EPI, int MT, int R, bool W4, bool QX>
int launch_cfg_w(const StreamParams &p, hipStream_t s)
{
    const size_t lds = stream_lds_bytes(p.K, MT, QX);
    if (lds > 160 * 1024) {
        set_error("qgemm (decode path): K=%d needs %zu bytes of LDS per workgroup, more than the 160 KiB of a CU", p.K, lds);
        return QARL_ERR_UNSUPPORTED;
    }
    static LdsLimitOnce once;
    auto kern = qgemm_stream_fp8_kernel<EPI, MT, R, W4, QX>;
    if (int rc = raise_lds_limit((const void *)kern, once, "hipFuncSetAttribute(stream fp8)")) return rc;
    const int64_t units = (int64_t)p.E * p.n_slices;
    const int64_t grid = ((units + 7) / 8) * 8 * p.m_split;
    kern<<<dim3((unsigned)grid), dim3(kSThreads), lds, s>>>(p);
    return check_hip(hipGetLastError(), "qgemm_stream_fp8_kernel");
}

template <int EPI, int MT, int R>
int launch_cfg(const StreamParams &p, hipStream_t s)
{
    if (p.ids) return p.w4 ? launch_cfg_w<EPI, MT, R, true, true>(p, s) : launch_cfg_w<EPI, MT, R, false, true>(p, s);
    return p.w4 ? launch_cfg_w<EPI, MT, R, true, false>(p, s) : launch_cfg_w<EPI, MT, R, false, false>(p, s);
}

template <int EPI, int MT>
int launch_ring(const StreamParams &p, hipStream_t s)
{
    const int G = p.K / kGroup;
    // ring depth (steps in flight per wavefront): 8 KiB per wavefront, i.e. two steps of e4m3 codes (4 KiB each: two
    // tiles, two 1 KiB loads per tile) or four steps of e2m1 codes, already saturate HBM with eight wavefronts per CU;
    // twice that measured 4 % slower on the gate_up launch, and a deeper ring would push the gather into spilling
    if (p.w4 && G % 4 == 0) return launch_cfg<EPI, MT, 4>(p, s);
    if (p.w4 && G % 3 == 0) return launch_cfg<EPI, MT, 3>(p, s);
    if (G % 2 == 0) return launch_cfg<EPI, MT, 2>(p, s);
    if (G % 3 == 0) return launch_cfg<EPI, MT, 3>(p, s);
    return launch_cfg<EPI, MT, 1>(p, s);
}

template <int EPI>
int launch_one(const GemmArgs &a, hipStream_t s)
{
    StreamParams p;
    p.codes = (const uint32_t *)a.codes;
    p.scales = (const float *)a.scales;
    p.x = a.x;
    p.x_scales = a.x_scales;
    p.row_map = a.row_map;
    p.out_row_map = a.out_row_map;
    p.offsets = a.offsets;
    p.out = a.out;
    p.E = a.E;
    p.N = a.N;
    p.K = a.K;
    p.out_f32 = a.out_f32;
    p.w4 = (a.fmt == QARL_FP4_E2M1_CH);
    p.ids = a.ids;
    p.n_ids = (int)a.M;
    p.topk = a.topk;
    p.x_per_token = a.x_per_token;
    const bool routed = a.ids != nullptr;
    if (routed && (a.M > kIdsMax || a.topk <= 0 || a.M % a.topk != 0 || a.M / a.topk > kIdsRows || ((uintptr_t)a.ids & 15) != 0)) {
        set_error("qgemm (routed decode path): needs T <= %d, T * topk <= %d and 16-byte aligned ids", kIdsRows, kIdsMax);
        return QARL_ERR_UNSUPPORTED;
    }
    p.n_units = (EPI == QARL_EPI_SILU_MUL) ? (a.N / 2) / 16 : a.N / 32;
    // rows per expert the grid should cover in one pass: mean + 4 sigma of a uniform router
    const double mean = (double)a.M / (double)a.E;
    const double need = mean + 4.0 * sqrt(mean);
    // token tiles per workgroup: limited by the LDS tile, which holds the whole K of every row
    const int mt_fit = stream_lds_bytes(a.K, 2, routed) <= 160 * 1024 ? 2 : (stream_lds_bytes(a.K, 1, routed) <= 160 * 1024 ? 1 : 0);
    if (mt_fit < 1) {
        set_error("qgemm (decode path): K=%d does not fit the LDS tile", a.K);
        return QARL_ERR_UNSUPPORTED;
    }
    int MT = need <= 16.0 ? 1 : 2;  // more rows per expert go to further row blocks (m_split)
    if (MT > mt_fit) MT = 1;
    const int ms = (int)ceil(need / (16.0 * MT));
    p.m_split = ms < 1 ? 1 : (ms > 8 ? 8 : ms);
    // slices per expert: aim at one workgroup per CU, at least one pair of tiles per wavefront
    int slices = (256 + a.E * p.m_split - 1) / (a.E * p.m_split);
    const int max_slices = (p.n_units + kSWaves - 1) / kSWaves;
    if (slices > max_slices) slices = max_slices;
    if (slices < 1) slices = 1;
    p.n_slices = slices;
    if (MT == 1) return launch_ring<EPI, 1>(p, s);
    return launch_ring<EPI, 2>(p, s);
}

}  // namespace

bool qgemm_stream_routed_supported(int fmt, int N, int K, int T, int topk)
{
    if (fmt == QARL_W4A16_G128 || fmt == QARL_W4A8_G128) return qgemm_stream_w4_routed_supported(N, K, T, topk);
    if (fmt != QARL_FP8_E4M3_CH && fmt != QARL_FP4_E2M1_CH) return false;
    if (!qgemm_stream_supported(fmt, N, K) || T <= 0 || topk <= 0) return false;
    if (T > kIdsRows || (int64_t)T * topk > kIdsMax) return false;
    return stream_lds_bytes(K, 1, true) <= 160 * 1024;
}

bool qgemm_stream_supported(int fmt, int N, int K)
{
    if (fmt == QARL_W4A16_G128 || fmt == QARL_W4A8_G128) return qgemm_stream_w4_supported(N, K);
    if (N % 32 != 0 || K % kGroup != 0 || K > 4096) return false;  // the gather sweeps >= 2 rows per step
    return stream_lds_bytes(K, 1) <= 160 * 1024;
}

int launch_qgemm_stream(const GemmArgs &a, hipStream_t s)
{
    if (!qgemm_stream_supported(a.fmt, a.N, a.K)) {
        set_error("qgemm (decode path): unsupported shape N=%d K=%d (needs N %% 32 == 0; W4A16: K %% 256 == 0, K <= 4096; "
                  "FP8: K %% 128 == 0, K <= 4096; the token tile of one row block must fit LDS)", a.N, a.K);
        return QARL_ERR_UNSUPPORTED;
    }
    if (a.fmt == QARL_W4A16_G128 || a.fmt == QARL_W4A8_G128) return launch_qgemm_stream_w4(a, s);
    return a.epilogue == QARL_EPI_SILU_MUL ? launch_one<QARL_EPI_SILU_MUL>(a, s) : launch_one<QARL_EPI_NONE>(a, s);
}

}  // namespace qarl
