// Grouped quantized GEMM, weight-streaming ("decode") path for the W4A16 format: eq. (1) of
// section 2.2 when every expert sees a few dozen token rows, so the kernel is bound by reading
// each expert's packed weights from HBM exactly once (the regime the paper's appendix on
// quantization schemes calls memory-bound).
//
// Work layout.  A workgroup of 8 wavefronts owns (expert, slice of its weight rows, block of
// 32*MT token rows).  It gathers its token rows ONCE into LDS for the whole K, and from then on
// every wavefront runs on its own: it walks pairs of 16-row weight tiles and, per pair, the
// K/128 scale groups, with the packed codes of the next R groups always in flight in a register
// ring (global -> registers, two 16-byte loads per lane and group).  The codes are stored in
// 1 KiB blocks of 16 rows x 128 k; a wavefront load takes the same half of the blocks of both
// tiles of the pair, so a tile's whole K is one contiguous stream.  The two tiles of a pair are
// the 32 columns of v_mfma_f32_32x32x16_bf16 (lanes 0-15 and 32-47 carry the first tile, 16-31
// and 48-63 the second), the token rows from LDS its 32 rows: one matrix instruction per 8
// packed words.  A matrix instruction holds the issue port of its SIMD for about two VALU slots
// whatever its shape, and the kernel is bound by issue (expansion of the codes) next to HBM, so
// the large shape leaves more slots to the expansion than twice as many 16x16x32 ones.
//
// Numerics: the dequantized weight is s*q exactly.  The nibble u = q+8 is placed in the top
// mantissa bits of bf16 1.0, giving the exact bf16 value (q+24)/16 with one shift and one
// and-or per two codes.  Each 128-k scale group accumulates in its own fp32 MFMA accumulator,
// started at -1.5 * sum_k x (which cancels the +24/16 offset), and is folded into the running
// sum with one fp32 FMA by 16*s.  A one-hot activation row therefore reproduces s*q bit for bit.
//
// Start-up.  Until the token tile stands in LDS no wavefront can use a weight, so the code in
// front of that point is kept short (every instruction costs a wavefront 4 cycles and two
// wavefronts share a SIMD): ids are split by shifts, the thread -> tile-block map uses a
// host-checked multiplication instead of a division, addresses are 32-bit offsets.  The chain
// expert offsets -> row ids -> token rows loses one link: the whole row map of a decode-sized
// batch is copied to LDS while the expert offsets are still on their way.  Rows past the
// expert's end are not loaded.
//
// Experts with more than 32*MT rows: the grid carries row blocks per (expert, slice), mapped to
// consecutive workgroups of the same XCD so that their identical weight reads meet in that
// XCD's L2; rows beyond that take further passes.
#include <math.h>

#include "common.hpp"

namespace qarl {

namespace {

constexpr int kThreads = 512;
constexpr int kWaves = 8;
constexpr int kMapMax = 4096;   // row-map entries a workgroup copies to LDS up front

struct W4Params {
    const uint32_t *codes;   // 1 KiB blocks [E*N/16][K/128][256 words]
    const uint16_t *scales;  // bf16 [E][N][K/128]
    const uint16_t *x;       // bf16 rows
    const float *x_scales;   // W4A8: scale of each activation row (the rows of x then hold e4m3 values), else null
    const int32_t *row_map;
    const int32_t *out_row_map;
    const int32_t *offsets;
    void *out;
    int E, N, K, out_f32;
    int M;           // rows over all experts (entries of the row maps)
    int n_units;     // pairs of 16-row weight tiles per expert
    int per_slice;   // pairs per workgroup (the last slice may hold fewer)
    int slice_sh;    // log2(workgroups along the weight rows of one expert)
    int msplit_sh;   // log2(row blocks per (expert, slice) in the grid)
    // gather of the token tile: thread -> (row rsub, 16-byte block b) = (tid / bpr, tid % bpr), the division
    // by a multiplication the host has checked for every tid
    int bpr, rpp;
    uint32_t bpr_magic;   // tid / bpr == (tid * bpr_magic) >> 20
    int map_mode;    // row maps copied to LDS up front: 0 no, 1 into the (still free) tile region, 2 into their own
    int half_tile;   // 16-row LDS tile (K beyond 2048)
    // Routed mode (ids != null; offsets and the row maps are unused): problem row = pair id pr = t * topk + slot,
    // expert ids[pr], activation row t or pr, output row pr.  Every workgroup finds its expert's pairs itself.
    const int32_t *ids;
    int n_ids;         // T * topk <= kIdsMax
    int topk;
    int x_per_token;   // activation row of pair pr: pr / topk if set, else pr
    // Routed W4A8: x holds 16-bit rows; the workgroup applies the activation quantizer of eq. (2) to the rows it
    // gathers (the row quantizer's arithmetic), keeps the e4m3 values as exact bf16 in the LDS tile and the row
    // scales in LDS for the epilogue.
    int qx;
};
constexpr int kQxScaleBytes = 4 * 64;   // LDS for the row scales of a block (up to 64 rows), routed mode

constexpr int kIdsMax = 4096;    // pairs a workgroup scans (8 per thread)
constexpr int kIdsRows = 512;    // rows of one expert it can list: one per token, T <= 512

// LDS bytes per activation row: the row plus 16 bytes, so consecutive rows skew by 4 banks.
__host__ __device__ constexpr int x_stride(int K) { return K * 2 + 16; }

// Dynamic LDS: row ids, output rows, pair counter, group sums, per-wavefront scale buffers, token tile.
// half: the 16-row variant for K beyond 2048 (one scale buffer per wavefront instead of two).
size_t lds_bytes(int K, int MT, bool half = false)
{
    const size_t G = K / kGroup, rows = half ? 16 : (size_t)MT * 32, idx = (size_t)MT * 32;
    return idx * 8 + 16 + G * rows * 4 + (size_t)kWaves * (half ? 1 : 2) * 32 * G * 2 + rows * x_stride(K);
}

// EPI: NONE or SILU_MUL; MT: 32-row token tiles per block; R: ring depth in scale groups (divides K/128);
// NT: the weight stream uses nontemporal loads (every line is read once).  With several row blocks per (expert,
// slice) the same lines are read by neighbouring workgroups of one XCD: there the loads stay temporal, so that the
// second reader finds them in that XCD's L2.
// HALF (with MT = 1): the LDS tile holds 16 token rows instead of 32, which is what fits for K up to 4096 (the
// hidden size of the dense models); the matrix instruction still takes 32 rows, its rows 16..31 re-read rows 0..15
// and their results are dropped.
template <int EPI, int MT, int R, bool NT, bool HALF = false>
__global__ __launch_bounds__(kThreads, 1) void qgemm_stream_w4_kernel(W4Params p)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    static_assert(!HALF || MT == 1, "the 16-row tile goes with one 32-row MFMA tile");
    constexpr int kRows = HALF ? 16 : MT * 32;   // token rows in LDS
    constexpr int kIdx = MT * 32;                // entries of the row-id arrays (rows of the MFMA tiles)
    constexpr int kScBufs = HALF ? 1 : 2;        // scale buffers per wavefront
    constexpr bool kSilu = (EPI == QARL_EPI_SILU_MUL);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // lane -> column 16 t + c of the pair's 32 weight rows, half h of every 16-k MFMA step
    const int c = lane & 15, t = (lane >> 4) & 1, h = lane >> 5, m32 = lane & 31;
    const int N = p.N, K = p.K, G = K / kGroup;
    const int stride = x_stride(K);

    // workgroup id -> (expert, slice, row block).  Ids go round-robin over the 8 XCDs; the row
    // blocks of one (expert, slice) take consecutive positions on the same XCD.
    const int xcd = blockIdx.x & 7, pos = blockIdx.x >> 3;
    const int m_split = 1 << p.msplit_sh;
    const int mh = pos & (m_split - 1);
    const int unit_id = (pos >> p.msplit_sh) * 8 + xcd;
    if (unit_id >= (p.E << p.slice_sh)) return;
    const int e = unit_id >> p.slice_sh, slice = unit_id & ((1 << p.slice_sh) - 1);

    int *s_row = (int *)smem;                              // [kIdx] activation row of each tile row (rows past the end repeat the last one)
    int *s_orow = (int *)(smem + kIdx * 4);                // [kIdx] output row, -1 past the expert's last row
    int *s_next = (int *)(smem + kIdx * 8);                // next undrawn pair
    float *sx = (float *)(smem + kIdx * 8 + 16);           // [G][kRows]  -1.5 * group sums
    // per wavefront two buffers of [32 rows of the pair][G] bf16 scales (this pair, next pair); one buffer in the
    // 16-row variant: the next pair's scales are parked after the last read of the current ones, and the LDS
    // operations of a wavefront execute in order
    uint16_t *ssc = (uint16_t *)(smem + kIdx * 8 + 16 + G * kRows * 4) + wave * kScBufs * 32 * G;
    unsigned char *xs = smem + kIdx * 8 + 16 + G * kRows * 4 + kWaves * kScBufs * 32 * G * 2;  // [kRows][stride]

    // this workgroup's pairs of weight tiles: units u_lo .. u_hi-1
    const int u_lo = slice * p.per_slice, u_hi = min(p.n_units, u_lo + p.per_slice);
    const int n_pairs = max(0, u_hi - u_lo);
    const int64_t ebase = (int64_t)e * N;

    // 16-row tile of this lane (its half t of the 32 MFMA columns) in the slice's pi-th pair
    auto pair_tile16 = [&](int pi) -> int {
        const int u = u_lo + pi;
        if (kSilu) return (t ? (N / 2) / 16 : 0) + u;   // gate tile | matching up tile
        return u * 2 + t;
    };
    // First word this lane loads of (pair pi, group g): block (tile, g) is 1 KiB = 4 k-ranges x 16 rows x 16 B;
    // the lane's load L takes k-range 2L + h of row c, so word j of load L holds k = 128 g + 64 L + 32 h + 8 j .. +8.
    // Past this wavefront's work the pointer falls back to the start of the expert's codes: the ring is
    // refilled without a branch (a conditional refill turns every slot into a merge of old and new value
    // and doubles the registers the ring takes), and those few loads all hit one cached line.
    auto batch_src = [&](int pi, int g0) -> const uint32_t * {
        const bool ok = pi < n_pairs;
        const int64_t tile = ebase / 16 + (ok ? pair_tile16(pi) : 0);
        return p.codes + (tile * G + (ok ? g0 : 0)) * 256 + h * 64 + c * 4;
    };
    struct Slot {
        u32x4 w[2];
    };
    Slot ring[R];
    auto fill = [&](Slot &dst, int r, const uint32_t *src) {
#pragma unroll
        for (int L = 0; L < 2; ++L) {
            const u32x4 *a = (const u32x4 *)(src + r * 256 + L * 128);
            dst.w[L] = NT ? __builtin_nontemporal_load(a) : *a;
        }
    };
    auto fill_ring = [&](int pi, int g0) {
        const uint32_t *src = batch_src(pi, g0);
#pragma unroll
        for (int r = 0; r < R; ++r) fill(ring[r], r, src);
    };
    // scales of a pair: [32 rows][G] bf16, G/2 dwords per row; lanes 2r and 2r+1 fetch row r (dwords of their
    // parity) and park them in the wavefront's LDS buffer one pair ahead.
    constexpr int kScRegs = HALF ? 8 : 4;  // dwords per lane: covers G <= 16 (32 in the 16-row variant)
    uint32_t scr[kScRegs];
    const int sc_row = lane >> 1, sc_par = lane & 1, sc_half = G / 2;
    auto load_scales = [&](int pi) {
        const int uu = u_lo + (pi < n_pairs ? pi : 0);
        const int nt = sc_row >> 4;
        const int tile = kSilu ? (nt ? (N / 2) / 16 : 0) + uu : uu * 2 + nt;
        const uint32_t *src = (const uint32_t *)p.scales + ((ebase + tile * 16 + (sc_row & 15)) * G) / 2;
#pragma unroll
        for (int u = 0; u < kScRegs; ++u) {
            const int dw = 2 * u + sc_par;
            scr[u] = dw < sc_half ? src[dw] : 0;
        }
    };
    auto park_scales = [&](int buf) {
        uint32_t *dst = (uint32_t *)(ssc + (buf % kScBufs) * 32 * G) + sc_row * sc_half;
#pragma unroll
        for (int u = 0; u < kScRegs; ++u) {
            const int dw = 2 * u + sc_par;
            if (dw < sc_half) dst[dw] = scr[u];
        }
    };

    // ---- start-up: the whole row maps go to LDS while the expert offsets are on their way: 16-byte loads;
    // the last, partial quad of a map is fetched entry by entry
    const bool routed = p.ids != nullptr;
    const bool map_in_lds = p.map_mode != 0;
    // [M rounded up to 4] row_map, then the same for out_row_map; routed mode: [kIdsRows] activation rows of
    // this expert's pairs, [kIdsRows] pair ids, then the pair count of every wavefront's share of the ids
    int *tmp_map = (int *)(p.map_mode == 2 ? xs + kRows * stride : xs);
    const int m4 = routed ? kIdsRows : (p.M + 3) & ~3;
    float *s_rsc = (float *)(xs + kRows * stride + 8 * kIdsRows + 4 * kWaves);   // [kIdx] row scales (routed W4A8)
    int row0, Me;
    if (routed) {
        // Thread tid looks at pairs 8 tid .. 8 tid + 7.  Matches keep their order: the rows of an expert are its
        // pairs by increasing pair id, the (token, slot) order a stable grouping gives.
        const int base = tid * 8;
        int idv[8];
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
            for (int k = 0; k < 4; ++k) idv[4 * q4 + k] = v4[k];
        }
        uint32_t hits = 0;
#pragma unroll
        for (int k = 0; k < 8; ++k) hits |= (idv[k] == e) ? (1u << k) : 0u;
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
        for (int w = 0; w < kWaves; ++w) {
            const int cw = s_wcnt[w];
            before += w < wave ? cw : 0;
            total += cw;
        }
        int rank = before + incl - cnt;
        for (uint32_t hm = hits; hm; hm &= hm - 1) {
            const int pr = base + __builtin_ctz(hm);
            if (rank < kIdsRows) {
                tmp_map[rank] = p.x_per_token ? pr / p.topk : pr;
                tmp_map[m4 + rank] = pr;
            }
            ++rank;
        }
        row0 = 0;
        Me = min(total, kIdsRows);
    } else {
    if (map_in_lds) {
        constexpr int kPer = kMapMax / (4 * kThreads);
#pragma unroll
        for (int u = 0; u < kPer; ++u) {
            const int i = (u * kThreads + tid) * 4;
            if (i < p.M) {
                i32x4 a = {i, i + 1, i + 2, i + 3}, b = a;
                if (i + 3 < p.M) {
                    if (p.row_map) a = *(const i32x4 *)(p.row_map + i);
                    if (p.out_row_map) b = *(const i32x4 *)(p.out_row_map + i);
                } else {
                    for (int k = 0; i + k < p.M; ++k) {
                        if (p.row_map) a[k] = p.row_map[i + k];
                        if (p.out_row_map) b[k] = p.out_row_map[i + k];
                    }
                }
                *(i32x4 *)(tmp_map + i) = a;
                *(i32x4 *)(tmp_map + m4 + i) = b;
            }
        }
    }
    row0 = p.offsets[e];
    Me = p.offsets[e + 1] - row0;
    }
    if (Me <= mh * kRows) return;

    bool first_pass = true;
    for (int m0 = mh * kRows; m0 < Me; m0 += kRows * m_split) {
        const int mrem = min(kRows, Me - m0);
        lds_barrier();  // the row map copy is complete / the previous pass is done with the LDS tile
        const bool use_tmp = map_in_lds && (first_pass || routed);   // the routed list has its own LDS region
        if (tid < kIdx) {
            // rows past the expert's end take the id of its last row (never loaded, results never stored)
            const int i = row0 + m0 + min(tid, mrem - 1);
            int xr, orow;
            if (use_tmp) {
                xr = tmp_map[i];
                orow = tmp_map[m4 + i];
            } else {
                xr = p.row_map ? p.row_map[i] : i;
                orow = p.out_row_map ? p.out_row_map[i] : i;
            }
            s_row[tid] = xr;
            s_orow[tid] = tid < mrem ? orow : -1;
        }
        if (tid == 0) *s_next = kWaves;  // pairs 0..7 start on wavefronts 0..7, the rest are drawn
        if (!use_tmp) lds_barrier();
        if (p.qx) {
            // ---- routed W4A8: one wavefront per row (rows wave, wave + 8, ...), four rows in flight: lane L holds
            // the 16-byte chunks L, L + 64, ... of the row; absmax by a wavefront reduction, s_x = absmax / 448,
            // e4m3 codes of x / s_x (the row quantizer's arithmetic), kept as the bf16 values they stand for.
            const int n16 = K / 8;
            bool first = true;
#pragma unroll 1
            for (int rb = 0; rb < kRows; rb += 4 * kWaves) {
                u32x4 v[4][4];
                int xrow[4];
#pragma unroll
                for (int rr = 0; rr < 4; ++rr) {
                    const int r = rb + rr * kWaves + wave;
                    xrow[rr] = r < mrem ? __builtin_amdgcn_readfirstlane(tmp_map[row0 + m0 + r]) : -1;
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int ch = lane + 64 * u;
                        v[rr][u] = u32x4{0, 0, 0, 0};
                        if (xrow[rr] >= 0 && ch < n16)
                            v[rr][u] = *(const u32x4 *)((const unsigned char *)p.x + ((uint32_t)xrow[rr] * (uint32_t)K + ch * 8) * 2u);
                    }
                }
                if (first) {
                    load_scales(wave);
                    fill_ring(wave, 0);
                    first = false;
                }
#pragma unroll
                for (int rr = 0; rr < 4; ++rr) {
                    const int r = rb + rr * kWaves + wave;
                    if (r >= kRows) continue;
                    if (xrow[rr] < 0) {   // past the expert's end: a row of zeros
#pragma unroll
                        for (int u = 0; u < 4; ++u)
                            if (lane + 64 * u < n16) *(u32x4 *)(xs + r * stride + (lane + 64 * u) * 16) = u32x4{0, 0, 0, 0};
                        if (lane == 0) s_rsc[r] = 0.f;
                        continue;
                    }
                    float am = 0.f;
#pragma unroll
                    for (int u = 0; u < 4; ++u) am = absmax_bf16x8(v[rr][u], am);
                    am = wave_max(am);
                    const float sxr = am / 448.0f;
                    const RowScale rs(sxr);
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int ch = lane + 64 * u;
                        if (ch < n16) {
                            const u32x2 q8 = e4m3_quantize_bf16x8(rs, v[rr][u]);
                            u32x4 o;   // e4m3 -> fp32 is exact, and so is its upper half as bf16 (four significant bits)
#pragma unroll
                            for (int i = 0; i < 2; ++i) {
                                const auto lo = __builtin_amdgcn_cvt_pk_f32_fp8((int)q8[i], false);
                                const auto hi = __builtin_amdgcn_cvt_pk_f32_fp8((int)q8[i], true);
                                o[2 * i] = (__float_as_uint(lo[0]) >> 16) | (__float_as_uint(lo[1]) & 0xffff0000u);
                                o[2 * i + 1] = (__float_as_uint(hi[0]) >> 16) | (__float_as_uint(hi[1]) & 0xffff0000u);
                            }
                            *(u32x4 *)(xs + r * stride + ch * 16) = o;
                        }
                    }
                    if (lane == 0) s_rsc[r] = sxr;
                }
            }
        } else
        // ---- gather the token rows into LDS (whole K) in 16-byte blocks.  A thread keeps one block column and
        // walks down the rows; the row ids are read first and then every load goes out at once, so no load
        // waits for a branch on an id.  Vector loads return in order: the token rows are requested first and the
        // weight stream right behind them, so it flows in while the tile is being built.
        {
            const int bpr = p.bpr;                      // blocks per row = K / 8
            const int rpp = p.rpp;                      // rows covered per sweep of the workgroup
            const int rsub = (int)(((uint32_t)tid * p.bpr_magic) >> 20), b = tid - rsub * bpr;
            const bool active = rsub < rpp;
            constexpr int kBatch = 16;
            u32x4 v[kBatch];
            int xr[kBatch];
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                const int r = min(min(rsub + u * rpp, kRows - 1), mrem - 1);
                xr[u] = use_tmp ? tmp_map[row0 + m0 + r] : s_row[r];
            }
            // byte offsets fit 32 bits (the launcher checks x_rows * K * 2 < 2^32)
            const uint32_t coff = (uint32_t)(b * 16), rbytes = (uint32_t)K * 2u;
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                v[u] = u32x4{0, 0, 0, 0};   // rows past the expert's end: no load
                if (rsub + u * rpp < mrem)
                    v[u] = *(const u32x4 *)((const unsigned char *)p.x + ((uint32_t)xr[u] * rbytes + coff));
            }
            load_scales(wave);
            fill_ring(wave, 0);
            if (use_tmp && p.map_mode == 1) lds_barrier();   // every thread has read its row ids: the map may be overwritten
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                const int r = rsub + u * rpp;
                const u32x4 o4 = v[u];
                if (active && r < kRows) *(u32x4 *)(xs + r * stride + b * 16) = o4;
            }
        }
        park_scales(0);
        lds_barrier();
        {
            // ---- group sums of the token rows, sx[g][m] = -1.5 * sum_k x[m][k], with the matrix core:
            // x times a matrix of ones; every column of the product holds the sums.
            const u32x4 ones4 = {0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};
            const bf16x8 ones = __builtin_bit_cast(bf16x8, ones4);
            const int q = lane >> 4;
            for (int g = wave; g < G; g += kWaves) {
#pragma unroll
                for (int mt = 0; mt < kRows / 16; ++mt) {
                    f32x4 d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const bf16x8 a = *(const bf16x8 *)(xs + (mt * 16 + c) * stride + (g * 128 + q * 32 + j * 8) * 2);
                        d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, ones, d, 0, 0, 0);
                    }
                    if (c == 0) {
#pragma unroll
                        for (int i = 0; i < 4; ++i) d[i] *= -1.5f;
                        *(f32x4 *)(sx + g * kRows + mt * 16 + 4 * q) = d;
                    }
                }
            }
            lds_barrier();
        }

        // ---- stream this wavefront's weight tiles.  Wavefronts draw pairs from the LDS counter one pair ahead.
        int it = 0;
        for (int pi = wave; pi < n_pairs; ++it) {
            int npi = 0;
            if (lane == 0) npi = atomicAdd(s_next, 1);
            npi = __builtin_amdgcn_readfirstlane(npi);
            load_scales(npi);
            f32x16 acc[MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[mt][i] = 0.f;
            for (int g0 = 0; g0 < G; g0 += R) {
                // the batch that refills the ring while this one is consumed: same pair or the next one
                const bool same = g0 + R < G;
                const uint32_t *nsrc = batch_src(same ? pi : npi, same ? g0 + R : 0);
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    const int g = g0 + r;
                    Slot &cur = ring[r];
                    // lane (m32, h), register i of a 32x32 result -> token row 8 (i / 4) + 4 h + i % 4
                    f32x16 ag[MT];
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                        for (int i4 = 0; i4 < 4; ++i4) {
                            const f32x4 init = *(const f32x4 *)(sx + g * kRows + (mt * 32 + 8 * i4 + 4 * h) % kRows);
#pragma unroll
                            for (int i = 0; i < 4; ++i) ag[mt][i4 * 4 + i] = init[i];
                        }
#pragma unroll
                    for (int L = 0; L < 2; ++L)
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const bf16x8 bw = unpack_int4_word(cur.w[L][j]);
#pragma unroll
                            for (int mt = 0; mt < MT; ++mt) {
                                const bf16x8 a = *(const bf16x8 *)(xs + ((mt * 32 + m32) % kRows) * stride +
                                                                   (g * 128 + L * 64 + h * 32 + j * 8) * 2);
                                ag[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bw, ag[mt], 0, 0, 0);
                            }
                        }
                    const float s16 = 16.f * bf16_bits_to_f32(ssc[((it & 1) % kScBufs) * 32 * G + m32 * G + g]);
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                        for (int i = 0; i < 16; ++i) acc[mt][i] = fmaf(s16, ag[mt][i], acc[mt][i]);
                    fill(cur, r, nsrc);   // refill this slot with the group R ahead
                }
            }
            // ---- epilogue of this pair
            const int u = u_lo + pi;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
                for (int i4 = 0; i4 < 4; ++i4) {
                    const i32x4 orow4 = *(const i32x4 *)(s_orow + mt * 32 + 8 * i4 + 4 * h);
                    if (p.qx) {   // routed W4A8: the row scales this workgroup computed
                        const f32x4 sc4 = *(const f32x4 *)(s_rsc + mt * 32 + 8 * i4 + 4 * h);
#pragma unroll
                        for (int i = 0; i < 4; ++i) acc[mt][i4 * 4 + i] *= sc4[i];
                    } else if (p.x_scales) {   // W4A8: the row scale s_x of eq. (2), in front of SiLU
                        const i32x4 xrow4 = *(const i32x4 *)(s_row + mt * 32 + 8 * i4 + 4 * h);
#pragma unroll
                        for (int i = 0; i < 4; ++i) acc[mt][i4 * 4 + i] *= p.x_scales[xrow4[i]];
                    }
                    if (kSilu) {
                        // Registers i and i+1 trade 16-lane rows: afterwards every lane holds a gate value and the
                        // up value of the same column; lanes of the first tile for row i, of the second for row i+1.
#pragma unroll
                        for (int ip = 0; ip < 2; ++ip) {
                            const u32x2 sw = __builtin_amdgcn_permlane16_swap(__float_as_uint(acc[mt][i4 * 4 + 2 * ip]),
                                                                              __float_as_uint(acc[mt][i4 * 4 + 2 * ip + 1]),
                                                                              false, false);
                            const int64_t orow = t ? orow4[2 * ip + 1] : orow4[2 * ip];
                            if (orow >= 0) {
                                const float a = silu_mul_f32(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
                                ((uint16_t *)p.out)[orow * (N / 2) + u * 16 + c] = f32_to_bf16_hw(a);
                            }
                        }
                    } else {
                        const int n = u * 32 + m32;
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const int64_t orow = orow4[i];
                            if (orow >= 0) {
                                if (p.out_f32) ((float *)p.out)[orow * N + n] = acc[mt][i4 * 4 + i];
                                else ((uint16_t *)p.out)[orow * N + n] = f32_to_bf16_hw(acc[mt][i4 * 4 + i]);
                            }
                        }
                    }
                }
            }
            park_scales((it + 1) & 1);
            pi = npi;
        }
        first_pass = false;
    }
}

// ---- 64 token rows per block where their whole K does not fit LDS (K = 2048: the gate_up projection of a batch
// with more than 32 rows per expert).  Two 32-row blocks would each pay a full pass over the expert's codes
// (expansion and matrix instructions are per weight, whatever the number of token rows).  Here K is walked in NC
// chunks: the LDS tile holds 64 rows x K / NC, every wavefront owns PW pairs of weight tiles for the whole kernel
// and keeps their accumulators (2 x 16 registers per pair) across the chunks, so the codes are expanded once and
// meet all 64 rows.  The weight ring runs through (chunk, pair, group) without a break; between two chunks the
// workgroup meets at a barrier and gathers the next K-range of its token rows.  Scales go from global memory
// straight to the lane that folds them (the 8 groups of a chunk are one 16-byte load).
template <int EPI, int PW, int NC>
__global__ __launch_bounds__(kThreads, 1) void qgemm_stream_w4_wide_kernel(W4Params p)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr int kRows = 64, R = 4, GC = 8;   // rows per block, ring depth, scale groups per chunk
    constexpr bool kSilu = (EPI == QARL_EPI_SILU_MUL);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, t = (lane >> 4) & 1, h = lane >> 5, m32 = lane & 31;
    const int N = p.N, K = p.K, G = K / kGroup, KC = K / NC;
    const int stride = x_stride(KC);

    const int xcd = blockIdx.x & 7, pos = blockIdx.x >> 3;
    const int m_split = 1 << p.msplit_sh;
    const int mh = pos & (m_split - 1);
    const int unit_id = (pos >> p.msplit_sh) * 8 + xcd;
    if (unit_id >= (p.E << p.slice_sh)) return;
    const int e = unit_id >> p.slice_sh, slice = unit_id & ((1 << p.slice_sh) - 1);

    int *s_row = (int *)smem;                              // [kRows]
    int *s_orow = (int *)(smem + kRows * 4);               // [kRows]
    float *sx = (float *)(smem + kRows * 8);               // [GC][kRows]  -1.5 * group sums of the chunk
    unsigned char *xs = smem + kRows * 8 + GC * kRows * 4;  // [kRows][stride]
    int *tmp_map = (int *)(xs + kRows * stride);           // routed mode: [kIdsRows] rows, [kIdsRows] pair ids, [kWaves] counts

    const int u_lo = slice * p.per_slice;                  // this workgroup's pairs: u_lo .. u_lo + 8 PW - 1
    const int64_t ebase = (int64_t)e * N;
    auto pair_tile16 = [&](int pi, int tt) -> int {
        const int u = u_lo + pi;
        if (kSilu) return (tt ? (N / 2) / 16 : 0) + u;
        return u * 2 + tt;
    };
    auto batch_src = [&](int pi, int g0) -> const uint32_t * {
        const int64_t tile = ebase / 16 + pair_tile16(pi, t);
        return p.codes + (tile * G + g0) * 256 + h * 64 + c * 4;
    };
    struct Slot {
        u32x4 w[2];
    };
    Slot ring[R];
    auto fill = [&](Slot &dst, int r, const uint32_t *src) {
#pragma unroll
        for (int L = 0; L < 2; ++L) dst.w[L] = __builtin_nontemporal_load((const u32x4 *)(src + r * 256 + L * 128));
    };
    // scales of this lane's output column (weight row) in pair pi, groups of chunk ch: 8 bf16 = one 16-byte load
    auto load_scales = [&](int pi, int ch) -> u32x4 {
        const int64_t row = ebase + pair_tile16(pi, m32 >> 4) * 16 + (m32 & 15);
        return *(const u32x4 *)(p.scales + row * G + ch * GC);
    };

    // ---- start-up: the expert's rows, from the router's ids (routed mode) or from offsets and row maps
    const bool routed = p.ids != nullptr;
    int row0, Me;
    if (routed) {
        const int base = tid * 8;
        int idv[8];
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
            for (int k = 0; k < 4; ++k) idv[4 * q4 + k] = v4[k];
        }
        uint32_t hits = 0;
#pragma unroll
        for (int k = 0; k < 8; ++k) hits |= (idv[k] == e) ? (1u << k) : 0u;
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
        for (int w = 0; w < kWaves; ++w) {
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
    if (Me <= mh * kRows) return;

    for (int m0 = mh * kRows; m0 < Me; m0 += kRows * m_split) {
        const int mrem = min(kRows, Me - m0);
        lds_barrier();  // the pair list is complete / the previous pass is done with the LDS tile
        if (tid < kRows) {
            const int i = row0 + m0 + min(tid, mrem - 1);
            int xr, orow;
            if (routed) {
                xr = tmp_map[i];
                orow = tmp_map[kIdsRows + i];
            } else {
                xr = p.row_map ? p.row_map[i] : i;
                orow = p.out_row_map ? p.out_row_map[i] : i;
            }
            s_row[tid] = xr;
            s_orow[tid] = tid < mrem ? orow : -1;
        }
        f32x16 acc[PW][2];
#pragma unroll
        for (int j = 0; j < PW; ++j)
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[j][mt][i] = 0.f;
        u32x4 sc_cur = load_scales(wave, 0), sc_nxt = sc_cur;

#pragma unroll 1
        for (int ch = 0; ch < NC; ++ch) {
            lds_barrier();  // row ids are written / every wavefront has left the previous chunk's tile
            // ---- gather the K-range of the token rows by asynchronous global -> LDS copies (no registers: the
            // accumulators of all pairs stay live across this point): a wavefront instruction moves 1 KiB, half of a
            // row's KC * 2 = 2 KiB; wavefront w copies rows 8 w .. 8 w + 7.  Rows past the expert's end repeat its
            // last row (their results are never stored).
            {
#pragma unroll
                for (int u = 0; u < 16; ++u) {
                    const int r = wave * 8 + (u >> 1), hh = u & 1;
                    const int xr = __builtin_amdgcn_readfirstlane(s_row[min(r, mrem - 1)]);
                    const unsigned char *src = (const unsigned char *)p.x + ((uint32_t)xr * (uint32_t)K * 2u +
                                                                              (uint32_t)(ch * KC * 2 + hh * 1024 + lane * 16));
                    copy16_to_lds(src, xs + r * stride + hh * 1024);
                }
                if (ch == 0) {   // the weight stream starts right behind the first gather
                    const uint32_t *src = batch_src(wave, 0);
#pragma unroll
                    for (int r = 0; r < R; ++r) fill(ring[r], r, src);
                }
            }
            copy_barrier();
            {
                // group sums of the chunk, sx[g][m] = -1.5 * sum_k x[m][k]: x times a matrix of ones
                const u32x4 ones4 = {0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};
                const bf16x8 ones = __builtin_bit_cast(bf16x8, ones4);
                const int q = lane >> 4;
                for (int unit = wave; unit < GC * 4; unit += kWaves) {
                    const int g = unit >> 2, mt = unit & 3;
                    f32x4 d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const bf16x8 a = *(const bf16x8 *)(xs + (mt * 16 + c) * stride + (g * 128 + q * 32 + j * 8) * 2);
                        d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, ones, d, 0, 0, 0);
                    }
                    if (c == 0) {
#pragma unroll
                        for (int i = 0; i < 4; ++i) d[i] *= -1.5f;
                        *(f32x4 *)(sx + g * kRows + mt * 16 + 4 * q) = d;
                    }
                }
                lds_barrier();
            }
            // ---- this wavefront's pairs over the chunk's groups
#pragma unroll
            for (int j = 0; j < PW; ++j) {
                const int pi = wave + 8 * j;
                // what follows (chunk, pair) in the stream: the next pair of the chunk, the first pair of the next chunk,
                // or, at the very end, lines that are cached already
                const bool last_pair = (j == PW - 1);
                const int npi = last_pair ? wave : pi + 8;
                const int nch = last_pair ? (ch + 1 < NC ? ch + 1 : 0) : ch;
                sc_nxt = load_scales(npi, nch);
#pragma unroll 1
                for (int g0 = 0; g0 < GC; g0 += R) {
                    const bool same = g0 + R < GC;
                    const uint32_t *nsrc = batch_src(same ? pi : npi, same ? ch * GC + g0 + R : nch * GC);
#pragma unroll
                    for (int r = 0; r < R; ++r) {
                        const int g = g0 + r;   // group within the chunk
                        Slot &cur = ring[r];
                        f32x16 ag[2];
#pragma unroll
                        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                            for (int i4 = 0; i4 < 4; ++i4) {
                                const f32x4 init = *(const f32x4 *)(sx + g * kRows + mt * 32 + 8 * i4 + 4 * h);
#pragma unroll
                                for (int i = 0; i < 4; ++i) ag[mt][i4 * 4 + i] = init[i];
                            }
#pragma unroll
                        for (int L = 0; L < 2; ++L)
#pragma unroll
                            for (int jj = 0; jj < 4; ++jj) {
                                const bf16x8 bw = unpack_int4_word(cur.w[L][jj]);
#pragma unroll
                                for (int mt = 0; mt < 2; ++mt) {
                                    const bf16x8 a = *(const bf16x8 *)(xs + (mt * 32 + m32) * stride +
                                                                       (g * 128 + L * 64 + h * 32 + jj * 8) * 2);
                                    ag[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bw, ag[mt], 0, 0, 0);
                                }
                            }
                        // scale of group g0 + r: bf16 number 2 (g0 / 4) + r / 2 .. of the lane's eight (g0 is 0 or 4)
                        const uint32_t sw = g0 ? sc_cur[2 + (r >> 1)] : sc_cur[r >> 1];
                        const float s16 = 16.f * __uint_as_float((r & 1) ? (sw & 0xffff0000u) : (sw << 16));
#pragma unroll
                        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                            for (int i = 0; i < 16; ++i) acc[j][mt][i] = fmaf(s16, ag[mt][i], acc[j][mt][i]);
                        fill(cur, r, nsrc);
                        __builtin_amdgcn_sched_barrier(0);   // keep the groups apart: hoisted operand reads cost registers
                    }
                }
                sc_cur = sc_nxt;
            }
        }

        // ---- epilogue of the wavefront's pairs
#pragma unroll
        for (int j = 0; j < PW; ++j) {
            const int u = u_lo + wave + 8 * j;
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
#pragma unroll
                for (int i4 = 0; i4 < 4; ++i4) {
                    const i32x4 orow4 = *(const i32x4 *)(s_orow + mt * 32 + 8 * i4 + 4 * h);
                    if (p.x_scales) {
                        const i32x4 xrow4 = *(const i32x4 *)(s_row + mt * 32 + 8 * i4 + 4 * h);
#pragma unroll
                        for (int i = 0; i < 4; ++i) acc[j][mt][i4 * 4 + i] *= p.x_scales[xrow4[i]];
                    }
                    if (kSilu) {
#pragma unroll
                        for (int ip = 0; ip < 2; ++ip) {
                            // lanes of the gate tile (t = 0) finish row 2 ip, lanes of the up tile row 2 ip + 1: each
                            // sends the value of the row it does not finish to its partner 16 lanes away
                            const float v0 = acc[j][mt][i4 * 4 + 2 * ip], v1 = acc[j][mt][i4 * 4 + 2 * ip + 1];
                            const float recv = __shfl_xor(t ? v0 : v1, 16, 64);
                            const float gv = t ? recv : v0, uv = t ? v1 : recv;
                            const int64_t orow = t ? orow4[2 * ip + 1] : orow4[2 * ip];
                            if (orow >= 0) {
                                const float a = silu_mul_f32(gv, uv);
                                ((uint16_t *)p.out)[orow * (N / 2) + u * 16 + c] = f32_to_bf16_hw(a);
                            }
                        }
                    } else {
                        const int n = u * 32 + m32;
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const int64_t orow = orow4[i];
                            if (orow >= 0) {
                                if (p.out_f32) ((float *)p.out)[orow * N + n] = acc[j][mt][i4 * 4 + i];
                                else ((uint16_t *)p.out)[orow * N + n] = f32_to_bf16_hw(acc[j][mt][i4 * 4 + i]);
                            }
                        }
                    }
                }
            }
        }
    }
}

size_t wide_lds_bytes(int K, int NC, bool routed)
{
    return (size_t)64 * 8 + 8 * 64 * 4 + (size_t)64 * x_stride(K / NC) + (routed ? 8 * (size_t)kIdsRows + 4 * kWaves : 0);
}

template <int EPI, int PW>
int launch_wide(const W4Params &p, hipStream_t s)
{
    constexpr int NC = 2;
    const size_t lds = wide_lds_bytes(p.K, NC, p.ids != nullptr);
    static LdsLimitOnce once;
    auto kern = qgemm_stream_w4_wide_kernel<EPI, PW, NC>;
    if (int rc = raise_lds_limit((const void *)kern, once, "hipFuncSetAttribute(stream w4 wide)")) return rc;
    const int64_t units = (int64_t)p.E << p.slice_sh;
    const int64_t grid = (((units + 7) / 8) * 8) << p.msplit_sh;
    kern<<<dim3((unsigned)grid), dim3(kThreads), lds, s>>>(p);
    return check_hip(hipGetLastError(), "qgemm_stream_w4_wide_kernel");
}

template <int EPI, int MT, int R, bool NT, bool HALF = false>
int launch_cfg_nt(const W4Params &p, hipStream_t s)
{
    size_t lds = lds_bytes(p.K, MT, HALF);
    if (p.ids) lds += 8 * (size_t)kIdsRows + 4 * kWaves + kQxScaleBytes;
    else if (p.map_mode == 2) lds += 8 * (size_t)((p.M + 3) & ~3);
    if (lds > 160 * 1024) {
        set_error("qgemm (decode path): K=%d needs %zu bytes of LDS per workgroup, more than the 160 KiB of a CU", p.K, lds);
        return QARL_ERR_UNSUPPORTED;
    }
    static LdsLimitOnce once;
    auto kern = qgemm_stream_w4_kernel<EPI, MT, R, NT, HALF>;
    if (int rc = raise_lds_limit((const void *)kern, once, "hipFuncSetAttribute(stream w4)")) return rc;
    const int64_t units = (int64_t)p.E << p.slice_sh;
    const int64_t grid = (((units + 7) / 8) * 8) << p.msplit_sh;
    kern<<<dim3((unsigned)grid), dim3(kThreads), lds, s>>>(p);
    return check_hip(hipGetLastError(), "qgemm_stream_w4_kernel");
}

template <int EPI, int MT, int R>
int launch_cfg(const W4Params &p, hipStream_t s)
{
    if (MT == 1 && p.half_tile)
        return p.msplit_sh == 0 ? launch_cfg_nt<EPI, 1, R, true, true>(p, s) : launch_cfg_nt<EPI, 1, R, false, true>(p, s);
    return p.msplit_sh == 0 ? launch_cfg_nt<EPI, MT, R, true>(p, s) : launch_cfg_nt<EPI, MT, R, false>(p, s);
}

template <int EPI, int MT>
int launch_ring(const W4Params &p, hipStream_t s)
{
    const int G = p.K / kGroup;
    // ring depth (groups in flight per wavefront): four 2 KiB batches per wavefront already saturate HBM with
    // eight wavefronts per CU
    if (G % 4 == 0) return launch_cfg<EPI, MT, 4>(p, s);
    if (G % 3 == 0) return launch_cfg<EPI, MT, 3>(p, s);
    return launch_cfg<EPI, MT, 2>(p, s);
}

template <int EPI>
int launch_one(const GemmArgs &a, hipStream_t s)
{
    W4Params p;
    p.codes = (const uint32_t *)a.codes;
    p.scales = (const uint16_t *)a.scales;
    p.x = (const uint16_t *)a.x;
    p.x_scales = a.fmt == QARL_W4A8_G128 ? a.x_scales : nullptr;
    p.row_map = a.row_map;
    p.out_row_map = a.out_row_map;
    p.offsets = a.offsets;
    p.out = a.out;
    p.E = a.E;
    p.N = a.N;
    p.K = a.K;
    p.out_f32 = a.out_f32;
    p.M = (int)a.M;
    p.ids = a.ids;
    p.n_ids = a.ids ? (int)a.M : 0;
    p.topk = a.topk;
    p.x_per_token = a.x_per_token;
    p.qx = (a.ids && a.fmt == QARL_W4A8_G128) ? 1 : 0;
    p.n_units = (EPI == QARL_EPI_SILU_MUL) ? (a.N / 2) / 16 : a.N / 32;
    // rows per expert the grid should cover in one pass: mean + 4 sigma of a uniform router
    const double mean = (double)a.M / (double)a.E;
    const double need = mean + 4.0 * sqrt(mean);
    // 64-row blocks where the whole K of 64 rows fits the LDS tile, 32-row blocks otherwise, 16-row blocks for K
    // beyond 2048
    const int MT = (need > 32.0 && lds_bytes(a.K, 2) <= 160 * 1024) ? 2 : 1;
    p.half_tile = lds_bytes(a.K, 1) > 160 * 1024;
    // row blocks per (expert, slice) and slices per expert are powers of two (the kernel splits ids by shifts)
    const int ms = (int)ceil(need / (p.half_tile ? 16.0 : 32.0 * MT));
    int msh = 0;
    while ((1 << msh) < ms && msh < 3) ++msh;
    p.msplit_sh = msh;
    // slices per expert: aim at one workgroup per CU, at least one pair of tiles per wavefront
    const int max_slices = (p.n_units + kWaves - 1) / kWaves;
    int ssh = 0;
    while (((int64_t)a.E << msh << (ssh + 1)) <= 256 && (2 << ssh) <= max_slices) ++ssh;
    p.slice_sh = ssh;
    p.per_slice = (p.n_units + (1 << ssh) - 1) >> ssh;
    // 64-row blocks over a K-chunked tile: K = 2048 (two chunks of eight scale groups), more than 32 rows per expert
    // to expect, and a slice that gives every wavefront the same one to three pairs
    static_assert(kWaves * 8 == 64, "the wide kernel's gather: eight rows per wavefront");
    if (MT == 1 && !p.half_tile && need > 32.0 && a.K == 2048 && !p.qx) {   // (its gather is an asynchronous copy: no quantizer)
        const int ms_w = (int)ceil(need / 64.0);
        int msh_w = 0;
        while ((1 << msh_w) < ms_w && msh_w < 3) ++msh_w;
        int ssh_w = 0;
        while (((int64_t)a.E << msh_w << (ssh_w + 1)) <= 256 && (2 << ssh_w) <= max_slices) ++ssh_w;
        const int per_w = p.n_units >> ssh_w;
        if ((per_w << ssh_w) == p.n_units && per_w % kWaves == 0 && per_w / kWaves >= 1 && per_w / kWaves <= 3 &&
            (int64_t)a.x_rows * a.K * 2 < (1LL << 32) &&
            (!a.ids || (a.M <= kIdsMax && a.topk > 0 && a.M % a.topk == 0 && a.M / a.topk <= kIdsRows && ((uintptr_t)a.ids & 15) == 0))) {
            p.msplit_sh = msh_w;
            p.slice_sh = ssh_w;
            p.per_slice = per_w;
            p.map_mode = 0;
            if (a.ids) p.row_map = p.out_row_map = p.offsets = nullptr;
            switch (per_w / kWaves) {
            case 1: return launch_wide<EPI, 1>(p, s);
            case 2: return launch_wide<EPI, 2>(p, s);
            default: return launch_wide<EPI, 3>(p, s);
            }
        }
    }
    p.bpr = a.K / 8;
    p.rpp = kThreads / p.bpr;
    p.bpr_magic = ((1u << 20) + p.bpr - 1) / p.bpr;
    if (16 * p.rpp < (p.half_tile ? 16 : 32 * MT)) {   // the gather keeps 16 blocks per thread in flight
        set_error("qgemm (decode path): K=%d: the token tile does not fit one sweep of the gather", a.K);
        return QARL_ERR_UNSUPPORTED;
    }
    for (uint32_t tid = 0; tid < (uint32_t)kThreads; ++tid)
        if (((tid * p.bpr_magic) >> 20) != tid / p.bpr) {
            set_error("qgemm (decode path): internal: bad division constant for K=%d", a.K);
            return QARL_ERR_UNSUPPORTED;
        }
    if ((int64_t)a.x_rows * a.K * 2 >= (1LL << 32)) {
        set_error("qgemm (decode path): activations of one call must stay below 4 GiB");
        return QARL_ERR_UNSUPPORTED;
    }
    if (a.ids) {
        if (a.M > kIdsMax || a.topk <= 0 || a.M % a.topk != 0 || a.M / a.topk > kIdsRows || ((uintptr_t)a.ids & 15) != 0) {
            set_error("qgemm (routed decode path): needs T <= %d, T * topk <= %d and 16-byte aligned ids", kIdsRows, kIdsMax);
            return QARL_ERR_UNSUPPORTED;
        }
        p.row_map = p.out_row_map = p.offsets = nullptr;
        p.map_mode = 2;
        if (MT == 1) return launch_ring<EPI, 1>(p, s);
        return launch_ring<EPI, 2>(p, s);
    }
    // decode-sized batches: the row maps go to LDS while the expert offsets are still on their way
    p.map_mode = 0;
    if (!p.half_tile && a.M <= kMapMax && (a.row_map || a.out_row_map) &&
        (((uintptr_t)a.row_map | (uintptr_t)a.out_row_map) & 15) == 0) {
        const size_t maps = 8 * (size_t)((a.M + 3) & ~3);
        if (lds_bytes(a.K, MT) + maps <= 160 * 1024) p.map_mode = 2;
        else if (maps <= (size_t)MT * 32 * x_stride(a.K)) p.map_mode = 1;
    }
    if (MT == 1) return launch_ring<EPI, 1>(p, s);
    return launch_ring<EPI, 2>(p, s);
}

}  // namespace

bool qgemm_stream_w4_supported(int N, int K)
{
    // the per-pair scale fetch is sized for K/128 <= 16 groups (32 with the 16-row tile) and moves pairs of scales;
    // the gather sweeps whole rows (K / 8 blocks of 16 bytes per row, at most one sweep of the workgroup)
    if (N % 32 != 0 || K % 256 != 0 || K > 4096) return false;
    return lds_bytes(K, 1) <= 160 * 1024 || lds_bytes(K, 1, true) <= 160 * 1024;
}

bool qgemm_stream_w4_routed_supported(int N, int K, int T, int topk)
{
    if (!qgemm_stream_w4_supported(N, K) || K > 2048 || T <= 0 || topk <= 0) return false;
    if (T > kIdsRows || (int64_t)T * topk > kIdsMax) return false;
    return lds_bytes(K, 1) + 8 * (size_t)kIdsRows + 4 * kWaves + kQxScaleBytes <= 160 * 1024;
}

int launch_qgemm_stream_w4(const GemmArgs &a, hipStream_t s)
{
    return a.epilogue == QARL_EPI_SILU_MUL ? launch_one<QARL_EPI_SILU_MUL>(a, s) : launch_one<QARL_EPI_NONE>(a, s);
}

}  // namespace qarl
