// Grouped quantized GEMM, MFMA-tiled ("prefill" / training-forward) path for the FP8 W8A8 format:
// eq. (2) of section 2.2 with e4m3 activations (one scale per token row) and e4m3 weights (one scale
// per output channel), Y = s_x s_w (X_q W_q^T), on the same codes and scales as the streaming path.
//
// Both operands are MFMA inputs as stored, so the kernel is a plain dense contraction: a workgroup owns
// 128 token rows x 256 weight rows of one expert; its eight wavefronts (2 x 4) own 64 x 64 each as 2 x 2
// v_mfma_f32_32x32x64_f8f6f4 tiles (e4m3 x e4m3, unit block scales).  The weight rows are the MFMA's row
// operand and the tokens its column operand, so a lane ends up with four consecutive output columns of ONE
// token per register quad: results leave in 16-byte (fp32) or 8-byte (bf16) stores, and the gate and up value
// of a column meet in the same lane.  Token rows (gathered through row_map) and weight rows reach LDS by
// asynchronous global -> LDS copies, three 128-k stages deep; 16-byte chunks of a row are XOR-swizzled with
// the row index so that the copies (8 rows x 128 bytes per wavefront instruction) and the operand reads
// (32 rows, one chunk) are free of bank conflicts.  The operand reads of half a stage run under the MFMAs
// of the half before, across the stage barrier as well; the six (four) copy instructions of a stage are
// issued one by one between its MFMAs, so that a wavefront that waits for room in the memory pipeline
// waits while its matrix instructions execute.
//
// FP4 weights (W4 = true) take the same kernel: the instruction reads e2m1 codes natively in its first
// operand (format select 4), 16 bytes per lane instead of 32.  A weight row then has 64 bytes per stage
// (four chunks, swizzled with (row >> 2) & 3), a stage is 32 KiB instead of 48, and no e4m3 copy of the
// weights is ever written.  The library packs the eight codes of a word as (element b, element 4 + b) in
// byte b; the instruction pairs nibble n of its first operand with byte n of the second within a group of
// 16 k, so the token bytes of every 8-byte group are put into the order 0 4 1 5 2 6 3 7 after their LDS
// read (two byte permutes per 8 bytes).  Across groups it pairs the 2 x 16 codes of first-operand lane h
// (k-half h of the 64) with bytes [16 h, 16 h + 16) of second-operand lanes 0 and 1: the token lanes
// therefore read the 16-byte chunks h and 2 + h of a half stage instead of 2 h and 2 h + 1.
#include "common.hpp"

namespace qarl {

constexpr int kFThreads = 512;
constexpr int kFTM = 128, kFTN = 256;        // token rows, weight rows per workgroup
constexpr int kFKS = 128;                    // k per stage (= bytes of an e4m3 row; an e2m1 row has 64)
constexpr int kFStages = 3;
__host__ __device__ constexpr int stage_bytes(bool w4) { return kFTM * kFKS + kFTN * (w4 ? kFKS / 2 : kFKS); }

struct Tile8Params {
    const unsigned char *codes;   // [E][N][K] e4m3, or [E][N][K/2] packed e2m1
    const float *scales;          // [E][N]
    const unsigned char *x;       // [x_rows][K] e4m3
    const float *x_scales;        // [x_rows]
    const int32_t *row_map;
    const int32_t *out_row_map;
    const int32_t *offsets;
    void *out;
    int E, N, K, out_f32;
    int n_blocks;   // column blocks per expert
    int bpw;        // consecutive column blocks one workgroup computes
    int n_bgroups;  // ceil(n_blocks / bpw)
    int m_slots, total;
};

template <int EPI, bool W4>
__global__ __launch_bounds__(kFThreads, 2) void qgemm_tile_fp8_kernel(Tile8Params p)
{
    constexpr int kFStageB = stage_bytes(W4);
    constexpr int kWRowB = W4 ? kFKS / 2 : kFKS;   // bytes of a weight row per stage
    constexpr int kWCopies = W4 ? 2 : 4;           // copy instructions per wavefront and stage for the weight rows
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr bool kSilu = (EPI == QARL_EPI_SILU_MUL);
    __shared__ __attribute__((aligned(16))) int s_rows[kFTM];
    __shared__ __attribute__((aligned(16))) int s_orow[kFTM];
    __shared__ __attribute__((aligned(16))) float s_xs[kFTM];
    __shared__ __attribute__((aligned(16))) float s_wn[2][kFTN];   // channel scale of every LDS weight row, per column block parity

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 2, wn = wave & 3;
    const int c = lane & 31, h = lane >> 5;

    // workgroup id -> (m slot, column block); XCD-contiguous ranges, column blocks of a token tile adjacent
    const int per_xcd = p.total / 8;
    const int v = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
    const int nb0 = (v % p.n_bgroups) * p.bpw;
    const int slot = v / p.n_bgroups;
    if (slot >= p.m_slots) return;

    // slot -> (expert, tile within expert): wavefront-level scan of the per-expert tile counts
    int e, mtile;
    {
        int cnt[4], sum = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int ex = lane * 4 + q;
            cnt[q] = ex < p.E ? (p.offsets[ex + 1] - p.offsets[ex] + kFTM - 1) / kFTM : 0;
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
    const int row0 = p.offsets[e] + mtile * kFTM;
    const int mrem = min(kFTM, p.offsets[e + 1] - row0);
    if (tid < kFTM) {
        // rows past the expert's end read the tile's first row (valid data, results never stored)
        const int i = row0 + (tid < mrem ? tid : 0);
        const int xrow = p.row_map ? p.row_map[i] : i;
        s_rows[tid] = xrow;
        s_orow[tid] = tid < mrem ? (p.out_row_map ? p.out_row_map[i] : i) : -1;
        s_xs[tid] = p.x_scales[xrow];
    }
    lds_barrier();

    const int N = p.N, K = p.K;
    // LDS weight row rho (0..255) of this workgroup -> weight row of the expert.  SILU_MUL: every 32-row
    // tile holds 16 gate rows then the 16 matching up rows, so gate j and up j sit 16 lanes apart in the
    // MFMA result.  Rows past N read row 0 (valid data, results never stored).
    auto weight_row = [&](int nb, int rho) -> int {
        int n;
        bool ok;
        if (kSilu) {
            const int j = nb * (kFTN / 2) + (rho >> 5) * 16 + (rho & 15);
            n = ((rho & 16) ? N / 2 : 0) + j;
            ok = j - (rho & 15) + 16 <= N / 2;
        } else {
            n = nb * kFTN + rho;
            ok = n - (rho & 31) + 32 <= N;
        }
        return ok ? n : 0;
    };

    // ---- copies: a wavefront instruction moves 8 rows x 128 bytes.  Chunk q of row r sits at
    // r * 128 + (q ^ ((r >> 1) & 7)) * 16.  This wavefront copies token rows [16 w, 16 w + 16) and weight
    // rows [32 w, 32 w + 32) of the tile.
    const unsigned char *aptr[2];
    uint32_t boff[kWCopies];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int r = wave * 16 + i * 8 + (lane >> 3);
        const int q = (lane & 7) ^ ((r >> 1) & 7);
        aptr[i] = p.x + (int64_t)s_rows[r] * K + q * 16;
    }
    uint32_t soff = 0;   // weight row whose scale this lane copies: LDS row 64 (wave % 4) + lane
    auto set_block = [&](int nb) {
#pragma unroll
        for (int i = 0; i < kWCopies; ++i) {
            if (W4) {   // 16 rows x 64 bytes per instruction
                const int r = wave * 32 + i * 16 + (lane >> 2);
                const int q = (lane & 3) ^ ((r >> 2) & 3);
                boff[i] = (uint32_t)weight_row(nb, r) * (uint32_t)(K / 2) + q * 16;
            } else {
                const int r = wave * 32 + i * 8 + (lane >> 3);
                const int q = (lane & 7) ^ ((r >> 1) & 7);
                boff[i] = (uint32_t)weight_row(nb, r) * (uint32_t)K + q * 16;
            }
        }
        soff = (uint32_t)weight_row(nb, (wave & 3) * 64 + lane);
    };
    set_block(nb0);
    const unsigned char *wbase = p.codes + (int64_t)e * N * (W4 ? K / 2 : K);
    const float *sbase = p.scales + (int64_t)e * N;
    // copy number j (0 .. 1 + kWCopies) of stage ks into buffer buf: two token copies, then the weight copies
    auto copy_one = [&](int ks, int buf, int j) {
        unsigned char *dst = smem + buf * kFStageB;
        if (j < 2) copy16_to_lds(aptr[j] + ks * kFKS, dst + (wave * 16 + j * 8) * kFKS);
        else copy16_to_lds(wbase + (int64_t)ks * kWRowB + boff[j - 2], dst + kFTM * kFKS + (wave * 32) * kWRowB + (j - 2) * 1024);
    };
    auto copy_stage = [&](int ks, int buf) {
#pragma unroll
        for (int j = 0; j < 2 + kWCopies; ++j) copy_one(ks, buf, j);
    };

    // ---- operand reads: v_mfma_f32_32x32x64_f8f6f4 takes 32 bytes per lane and operand: lane (c,h), half t of
    // the stage -> row c, bytes [64 t + 32 h, +32) = chunks 4t + 2h and 4t + 2h + 1 (both operands split k alike)
    // e2m1 weights: 16 bytes per lane, chunk 2 t + h of the row's four
    int foff[4], woff[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            // e2m1 first operand: the instruction pairs its lane h with bytes [16 h, 16 h + 16) of the second operand's
            // lanes 0 and 1 (measured), so the token lanes take the 16-byte chunks h and 2 + h of the half stage
            const int chunk = W4 ? 4 * t + h + 2 * u : 4 * t + 2 * h + u;
            foff[t * 2 + u] = c * kFKS + ((chunk ^ ((c >> 1) & 7)) * 16);
        }
        woff[t] = c * (kFKS / 2) + (((2 * t + h) ^ ((c >> 2) & 3)) * 16);
    }
    const int a_wave = wm * 64 * kFKS, b_wave = kFTM * kFKS + wn * 64 * kWRowB;
    struct Frags {
        i32x8 a[2], b[2];
    };
    auto read_frags = [&](Frags &f, int buf, int t) {
        const unsigned char *base = smem + buf * kFStageB;
#pragma unroll
        for (int ms = 0; ms < 2; ++ms) {
            const u32x4 lo = *(const u32x4 *)(base + foff[t * 2] + a_wave + ms * 32 * kFKS);
            const u32x4 hi = *(const u32x4 *)(base + foff[t * 2 + 1] + a_wave + ms * 32 * kFKS);
            f.a[ms] = i32x8{(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3], (int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
        }
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
            if (W4) {
                const u32x4 lo = *(const u32x4 *)(base + woff[t] + b_wave + nt * 32 * kWRowB);
                f.b[nt] = i32x8{(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3], 0, 0, 0, 0};
            } else {
                const u32x4 lo = *(const u32x4 *)(base + foff[t * 2] + b_wave + nt * 32 * kFKS);
                const u32x4 hi = *(const u32x4 *)(base + foff[t * 2 + 1] + b_wave + nt * 32 * kFKS);
                f.b[nt] = i32x8{(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3], (int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
            }
        }
    };
    // e2m1 weights: token bytes 0..7 of every 8-byte group -> order 0 4 1 5 2 6 3 7 (nibble n of a packed word
    // holds element n / 2 + 4 (n % 2))
    auto pair_tokens = [&](Frags &f) {
        if (!W4) return;
#pragma unroll
        for (int ms = 0; ms < 2; ++ms)
#pragma unroll
            for (int d = 0; d < 8; d += 2) {
                const uint32_t lo = (uint32_t)f.a[ms][d], hi = (uint32_t)f.a[ms][d + 1];
                f.a[ms][d] = (int)__builtin_amdgcn_perm(hi, lo, 0x05010400u);
                f.a[ms][d + 1] = (int)__builtin_amdgcn_perm(hi, lo, 0x07030602u);
            }
    };
    f32x16 acc[2][2];
#pragma unroll
    for (int ms = 0; ms < 2; ++ms)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[ms][nt][i] = 0.f;
    // e4m3 (or e2m1: format 4) x e4m3, no block scales
    auto mfma1 = [&](const Frags &f, int ms, int nt) {
        acc[ms][nt] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(f.b[nt], f.a[ms], acc[ms][nt], W4 ? 4 : 0, 0, 0, 0, 0, 0);
    };
    auto mfma4 = [&](const Frags &f) {
#pragma unroll
        for (int ms = 0; ms < 2; ++ms)
#pragma unroll
            for (int nt = 0; nt < 2; ++nt) mfma1(f, ms, nt);
    };

    // Rotated loop (see logprob.hip): the MFMAs of a stage's last group run in the next trip, behind the
    // stage barrier and under the first operand reads of the next stage.  The copies of stage s + 2 are
    // issued during stage s into the buffer stage s - 1 has just left; the wait before the barrier
    // leaves exactly those six (e2m1 weights: four) copies in flight.
    constexpr int kCopies = 2 + kWCopies;
    auto wait_stage = [&]() {   // all but the newest stage's copies have landed, own LDS reads are done; then the barrier
        if (W4) asm volatile("s_waitcnt vmcnt(4) lgkmcnt(0)\n\ts_barrier" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(6) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    };
    const int stages = K / kFKS;
    Frags last, g0, g1;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        last.a[i] = i32x8{0, 0, 0, 0, 0, 0, 0, 0};
        last.b[i] = i32x8{0, 0, 0, 0, 0, 0, 0, 0};
    }
    // First two stages of a column block into buffers 0 and 1; in front of them the block's 256 channel
    // scales, 4 bytes per lane (wavefronts w and w + 4 copy the same 64), into the half of s_wn the block's
    // parity selects.  They are older than every stage copy, so each counted wait below covers them.
    auto start_block = [&](int par) {
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(sbase + soff),
                                         (__attribute__((address_space(3))) void *)(&s_wn[par][(wave & 3) * 64]), 4, 0, 0);
        copy_stage(0, 0);
        if (stages > 1) copy_stage(1, 1);
    };
    start_block(0);
  for (int bi = 0; bi < p.bpw && nb0 + bi < p.n_blocks; ++bi) {
    const int nb = nb0 + bi;
    if (stages > 1)
        wait_stage();   // stage 0 has landed (stores of the block before too)
    else
        copy_barrier();
#pragma unroll
    for (int ms = 0; ms < 2; ++ms)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[ms][nt][i] = 0.f;
    int buf = 0;
    for (int ks = 0; ks < stages; ++ks) {
        const bool more = ks + 2 < stages;
        const int nbuf = buf == 0 ? 2 : buf - 1;
        // one MFMA, the operand reads of the next half, then MFMA and copy in turns
        read_frags(g0, buf, 0);
        mfma1(last, 0, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, W4 ? 6 : 8, 0);
        __builtin_amdgcn_sched_barrier(0);
        mfma1(last, 0, 1);
        if (more) copy_one(ks + 2, nbuf, 0);
        __builtin_amdgcn_sched_barrier(0);
        mfma1(last, 1, 0);
        if (more) copy_one(ks + 2, nbuf, 1);
        __builtin_amdgcn_sched_barrier(0);
        mfma1(last, 1, 1);
        if (more) copy_one(ks + 2, nbuf, 2);
        pair_tokens(g0);
        __builtin_amdgcn_sched_barrier(0);
        read_frags(g1, buf, 1);
        mfma1(g0, 0, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, W4 ? 6 : 8, 0);
        __builtin_amdgcn_sched_barrier(0);
        mfma1(g0, 0, 1);
        if (more) copy_one(ks + 2, nbuf, 3);
        __builtin_amdgcn_sched_barrier(0);
        mfma1(g0, 1, 0);
        if (more && kCopies > 4) copy_one(ks + 2, nbuf, 4);
        __builtin_amdgcn_sched_barrier(0);
        mfma1(g0, 1, 1);
        if (more && kCopies > 4) copy_one(ks + 2, nbuf, 5);
        pair_tokens(g1);
        __builtin_amdgcn_sched_barrier(0);
        if (more)
            wait_stage();
        else
            copy_barrier();
        last = g1;
        buf = buf == 2 ? 0 : buf + 1;
    }
    mfma4(last);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        last.a[i] = i32x8{0, 0, 0, 0, 0, 0, 0, 0};
        last.b[i] = i32x8{0, 0, 0, 0, 0, 0, 0, 0};
    }

    // ---- epilogue: lane (c,h), register i of acc[ms][nt] -> token row 64 wm + 32 ms + c, LDS weight row
    // 64 wn + 32 nt + 8 (i/4) + 4 h + i%4: four consecutive rows, i.e. output columns, per register quad.
    // The first copies of the next column block are issued first (every buffer is free after the last
    // barrier), so they travel while this block's results are scaled and stored.
    if (bi + 1 < p.bpw && nb + 1 < p.n_blocks) {
        set_block(nb + 1);
        start_block((bi + 1) & 1);
    }
    const float *wsc = s_wn[bi & 1];
    const int ncols = kSilu ? N / 2 : N;
    const int esz = (kSilu || !p.out_f32) ? 2 : 4;
    const uint32_t rstride = (uint32_t)ncols * (uint32_t)esz;
#pragma unroll
    for (int ms = 0; ms < 2; ++ms) {
        const int trow = wm * 64 + ms * 32 + c;
        const int orow = s_orow[trow];
        const float xs = s_xs[trow];
        unsigned char *orow_base = (unsigned char *)p.out + (uint64_t)(uint32_t)max(orow, 0) * rstride;
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
            const int rho0 = wn * 64 + nt * 32;
            if (kSilu) {
                // rows rho0 .. +15 are gate rows, rho0 + 16 .. +31 the matching up rows: registers i and i + 8
                const int ocol0 = nb * (kFTN / 2) + (rho0 >> 5) * 16;
                const bool tile_ok = ocol0 + 16 <= N / 2;
#pragma unroll
                for (int a4 = 0; a4 < 2; ++a4) {
                    const int r = 8 * a4 + 4 * h;
                    const f32x4 sg = *(const f32x4 *)(wsc + rho0 + r), su = *(const f32x4 *)(wsc + rho0 + 16 + r);
                    u32x2 o;
#pragma unroll
                    for (int b2 = 0; b2 < 2; ++b2) {
                        uint32_t pk = 0;
#pragma unroll
                        for (int q = 0; q < 2; ++q) {
                            const int i = 2 * b2 + q;
                            const float g = acc[ms][nt][4 * a4 + i] * (xs * sg[i]);
                            const float u = acc[ms][nt][8 + 4 * a4 + i] * (xs * su[i]);
                            pk |= (uint32_t)f32_to_bf16_hw(silu_mul_f32(g, u)) << (16 * q);
                        }
                        o[b2] = pk;
                    }
                    if (orow >= 0 && tile_ok) *(u32x2 *)(orow_base + (ocol0 + r) * 2) = o;
                }
            } else {
                const int ocol0 = nb * kFTN + rho0;
                const bool tile_ok = ocol0 + 32 <= N;
                // The 32 x 32 tile (lane: one token, four consecutive columns per register quad) turns through
                // this wavefront's 4 KiB of the third stage buffer, which the next block's first copies leave
                // alone, and leaves as 16-byte pieces of whole 128-byte row segments.  Chunks are XOR-swizzled
                // with the row; the stores are written so that the compiler does not see them (in front of a
                // visible LDS store it would drain the copies in flight for the next block).
                unsigned char *ot = smem + 2 * kFStageB + wave * 4096;   // 32 KiB: fits the third stage buffer of either format
                const uint32_t ot_a = (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void *)ot;
#pragma unroll
                for (int a4 = 0; a4 < 4; ++a4) {
                    const int r = 8 * a4 + 4 * h;
                    const f32x4 sw = *(const f32x4 *)(wsc + rho0 + r);
                    f32x4 vv;
#pragma unroll
                    for (int i = 0; i < 4; ++i) vv[i] = acc[ms][nt][4 * a4 + i] * (xs * sw[i]);
                    const uint32_t dst = ot_a + (uint32_t)(c * 128 + (((2 * a4 + h) ^ (c & 7)) << 4));
                    asm volatile("ds_write_b128 %0, %1" ::"v"(dst), "v"(vv) : "memory");
                }
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
                for (int pass = 0; pass < 4; ++pass) {
                    const int row = pass * 8 + (lane >> 3);
                    const f32x4 v4 = *(const f32x4 *)(ot + row * 128 + (lane & 7) * 16);
                    const int orow_r = s_orow[wm * 64 + ms * 32 + row];
                    const int col = ocol0 + (((lane & 7) ^ (row & 7)) << 2);
                    if (orow_r >= 0 && tile_ok) {
                        unsigned char *dstp = (unsigned char *)p.out + (uint64_t)(uint32_t)orow_r * rstride;
                        if (p.out_f32) {
                            __builtin_nontemporal_store(v4, (f32x4 *)(dstp + col * 4));   // fp32 rows for the combine: written once, read once by another kernel
                        } else {
                            u32x2 o;
                            o[0] = (uint32_t)f32_to_bf16_hw(v4[0]) | ((uint32_t)f32_to_bf16_hw(v4[1]) << 16);
                            o[1] = (uint32_t)f32_to_bf16_hw(v4[2]) | ((uint32_t)f32_to_bf16_hw(v4[3]) << 16);
                            *(u32x2 *)(dstp + col * 2) = o;
                        }
                    }
                }
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            }
        }
    }
  }
}

template <int EPI, bool W4>
static int launch_fp8_cfg(const GemmArgs &a, hipStream_t s)
{
    if (a.E > 256) {
        set_error("qgemm (prefill path): at most 256 experts (got %d)", a.E);
        return QARL_ERR_UNSUPPORTED;
    }
    if (a.N % 32 != 0 || a.N > (1 << 28) || (int64_t)a.N * a.K >= (1LL << 32)) {
        set_error("qgemm (prefill path): N %% 32 == 0 and N * K < 2^32 required (got N=%d K=%d)", a.N, a.K);
        return QARL_ERR_UNSUPPORTED;
    }
    Tile8Params p;
    p.codes = (const unsigned char *)a.codes;
    p.scales = (const float *)a.scales;
    p.x = (const unsigned char *)a.x;
    p.x_scales = a.x_scales;
    p.row_map = a.row_map;
    p.out_row_map = a.out_row_map;
    p.offsets = a.offsets;
    p.out = a.out;
    p.E = a.E;
    p.N = a.N;
    p.K = a.K;
    p.out_f32 = a.out_f32;
    p.n_blocks = (EPI == QARL_EPI_SILU_MUL) ? (a.N / 2 + kFTN / 2 - 1) / (kFTN / 2) : (a.N + kFTN - 1) / kFTN;
    const int64_t slots = (a.M + kFTM - 1) / kFTM + a.E;
    // a workgroup computes bpw neighbouring column blocks of its token tile one after the other: the expert
    // lookup and the row gather are paid once, and a block's stores hide the first copies of the next
    p.bpw = p.n_blocks >= 6 ? 3 : (p.n_blocks >= 2 ? 2 : 1);
    p.n_bgroups = (p.n_blocks + p.bpw - 1) / p.bpw;
    const int64_t total = ((slots * p.n_bgroups + 7) / 8) * 8;
    if (total > 0x7fffffffLL) {
        set_error("qgemm (prefill path): grid too large");
        return QARL_ERR_UNSUPPORTED;
    }
    p.m_slots = (int)slots;
    p.total = (int)total;
    static LdsLimitOnce once;
    auto kern = qgemm_tile_fp8_kernel<EPI, W4>;
    if (int rc = raise_lds_limit((const void *)kern, once, "hipFuncSetAttribute(tile fp8)")) return rc;
    kern<<<dim3((unsigned)total), dim3(kFThreads), kFStages * stage_bytes(W4), s>>>(p);
    return check_hip(hipGetLastError(), "qgemm_tile_fp8_kernel");
}

int launch_qgemm_tile_fp8(const GemmArgs &a, hipStream_t s)
{
    if (a.fmt == QARL_FP4_E2M1_CH)
        return a.epilogue == QARL_EPI_SILU_MUL ? launch_fp8_cfg<QARL_EPI_SILU_MUL, true>(a, s) : launch_fp8_cfg<QARL_EPI_NONE, true>(a, s);
    return a.epilogue == QARL_EPI_SILU_MUL ? launch_fp8_cfg<QARL_EPI_SILU_MUL, false>(a, s) : launch_fp8_cfg<QARL_EPI_NONE, false>(a, s);
}

}  // namespace qarl
