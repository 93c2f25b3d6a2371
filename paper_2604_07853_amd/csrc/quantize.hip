// Weight / activation quantizers: the Quant equations of section 2.2.
//   int4: integer Quant with z = 0, one bf16 scale per 128 consecutive k of a row; codes are
//         written in 1 KiB blocks of 16 rows x 128 k, the unit the GEMM kernels load;
//   fp8 : FP Quant with alpha = 448 (e4m3), one fp32 scale per row.
// Both are HBM-bound streams: 16-byte coalesced loads, the absmax reduced with wavefront shuffles.  Codes
// and scales are DEFINED as the results of IEEE fp32 divides (absmax / 7 or / 448, w / scale), so any IEEE
// implementation of the equations reproduces them bit for bit; the kernels reach those same bits without a
// divide per element: a reciprocal multiply with an exact FMA tie test (int4), a reciprocal with one
// correction step that yields the correctly rounded quotient (fp8).
#include "common.hpp"

namespace qarl {

// ------------------------------------------------------------------ int4 --
// A wavefront produces one 1 KiB block of the packed layout: 16 rows x 128 k (one scale group of
// each row).  Lane (c = lane & 15, q = lane >> 4) owns row c, k in [32 q, 32 q + 32): it reads 64
// contiguous bytes of bf16, the four lanes of a row reduce the absmax with two shuffles, and the
// lane writes its four code words as one 16-byte store at byte 16 * lane of the block.  The loads
// are plain (temporal) ones: a lane's four 16-byte loads fall into the same 64 bytes, so every
// load instruction touches a quarter of each cache line it needs, and a nontemporal load would
// fetch the line again for each of them (measured: 4.5 TB/s against 5.8 TB/s for this pattern).
// Next to HBM the kernel is bound by VALU issue (about a dozen operations per weight), so the
// rounding of a weight is arranged to take as few of them as possible.
constexpr int kQThreads = 256;

__global__ __launch_bounds__(kQThreads) void quantize_int4_kernel(const uint16_t *__restrict__ w, int64_t n_blocks,
                                                                  int K, uint32_t *__restrict__ codes,
                                                                  uint16_t *__restrict__ scales)
{
    const int lane = threadIdx.x & 63;
    const int c = lane & 15, q = lane >> 4;
    const int G = K / kGroup;
    const int64_t blk = (int64_t)blockIdx.x * (kQThreads / 64) + (threadIdx.x >> 6);
    if (blk >= n_blocks) return;  // whole wavefront
    const int64_t tile = blk / G;
    const int g = (int)(blk % G);
    const int64_t row = tile * 16 + c;
    const u32x4 *src = (const u32x4 *)(w + row * K + g * kGroup + q * 32);
    u32x4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] = src[u];
    float f[32];
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[u * 8 + 2 * i] = __uint_as_float(v[u][i] << 16);
            f[u * 8 + 2 * i + 1] = __uint_as_float(v[u][i] & 0xffff0000u);
        }
    float am = 0.f;
#pragma unroll
    for (int i = 0; i < 32; ++i) am = fmaxf(am, fabsf(f[i]));
    am = fmaxf(am, __shfl_xor(am, 16, 64));
    am = fmaxf(am, __shfl_xor(am, 32, 64));
    const uint32_t sb = f32_to_bf16_bits(am / 7.0f);
    const float s = bf16_bits_to_f32(sb);
    u32x4 out = {0x44444444u, 0x44444444u, 0x44444444u, 0x44444444u};  // code 0 (u = 8) in every element
    if (s >= 0x1p-100f && s < 0x1p100f) {
        // rne(w / s) without the IEEE divide.  w and s carry 8 significant bits each and |w / s| < 8.5, so the
        // quotient either IS a half-integer or stays at least 2^-11 away from every half-integer: away from a
        // tie the approximate quotient w * rcp(s) (a few ulp off) rounds like the exact one, and a tie is
        // found exactly: with h the half-integer next to the quotient, w - h s is computed without error by
        // one FMA (h s has at most 13 bits) and is zero if and only if w / s == h; then rne(h) is the answer.
        // The rounding itself is the fp32 addition of 1.5 * 2^23 (+ 8 for the stored offset): it rounds to
        // nearest even and leaves q + 8 in the low bits of the sum, which a shift-and-add drops into its
        // nibble; the constant high bits of the eight sums of a word are subtracted once at the end.
        const float rs = __builtin_amdgcn_rcpf(s);
        constexpr float kMagic = 12582912.f + 8.f;          // bit pattern 0x4B400008
        uint32_t bias = 0;                                   // sum over the eight elements of 0x4B400000 rotated into place
#pragma unroll
        for (int i = 0; i < 8; ++i)
            bias += i < 7 ? 0x4B400000u << int4_bit_pos(i) : __builtin_rotateleft32(0x4B400000u, int4_bit_pos(i));
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            uint32_t word = 0;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const float wv = f[u * 8 + i];
                const float r0 = wv * rs;
                const float h = floorf(r0) + 0.5f;
                const float sel = fmaf(-h, s, wv) == 0.f ? h : r0;
                // clamp first (it only bites on non-finite input; NaN -> -8), then round by the magic addition
                const float y = __builtin_amdgcn_fmed3f(sel, -8.f, 7.f) + kMagic;
                // element i -> its bit position: one shift-and-add; element 7 wraps around the word (a rotation)
                word += i < 7 ? __float_as_uint(y) << int4_bit_pos(i) : __builtin_rotateleft32(__float_as_uint(y), int4_bit_pos(i));
            }
            out[u] = word - bias;
        }
    } else if (s != 0.f) {
        // scales outside the range where rcp is safe (never reached by finite weights of sane magnitude)
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            uint32_t word = 0;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                float r = rintf(f[u * 8 + i] / s);
                r = fminf(fmaxf(r, -8.f), 7.f);
                word |= __builtin_rotateleft32((uint32_t)((int)r + 8), int4_bit_pos(i));
            }
            out[u] = word;
        }
    }
    __builtin_nontemporal_store(out, (u32x4 *)(codes + blk * 256 + lane * 4));
    if (q == 0) scales[row * G + g] = (uint16_t)sb;
}

int launch_quantize_int4(const void *w, int64_t rows, int K, void *codes, void *scales, hipStream_t s)
{
    const int64_t n_blocks = (rows / 16) * (int64_t)(K / kGroup);
    if (n_blocks == 0) return QARL_OK;
    const int per_wg = kQThreads / 64;
    const int64_t wgs = (n_blocks + per_wg - 1) / per_wg;
    if (wgs > 0x7fffffffLL) {
        set_error("quantize: %lld workgroups exceed the grid limit", (long long)wgs);
        return QARL_ERR_UNSUPPORTED;
    }
    quantize_int4_kernel<<<dim3((unsigned)wgs), dim3(kQThreads), 0, s>>>((const uint16_t *)w, n_blocks, K,
                                                                         (uint32_t *)codes, (uint16_t *)scales);
    return check_hip(hipGetLastError(), "quantize_int4_kernel");
}

// ------------------------------------------------------------- fp8 / fp4 --
// FP4 = true: the same FP Quant with alpha = 6 into e2m1 codes, eight per 32-bit word (byte b of the word: element
// b in the low nibble, element 4 + b in the high nibble).
// One wavefront per row; rows of up to 4096 elements are read once and wait in registers between the absmax
// pass and the conversion pass, longer rows are read a second time (a cache hit).
constexpr int kF8Threads = 256;

// Chunk c (8 elements, 16 bytes of bf16) of a row -> its codes: 8 bytes of e4m3, or 4 bytes of e2m1.
template <bool FP4>
__device__ __forceinline__ void store_codes_bf16x8(uint8_t *codes, int64_t row, int K, int c, const RowScale &rs, float s, const u32x4 v)
{
    if (FP4) {
        uint32_t w = 0;
        if (s != 0.f) {
            // v_cvt_scalef32_pk_fp4_f32 with scale 1 rounds to the nearest e2m1 value, ties to the even code,
            // saturating at 6, and puts its two results into one byte (first source in the low nibble): byte b
            // takes elements b and 4 + b.  Checked against a software encoder (comparisons with the seven rounding
            // boundaries) on every boundary, its two neighbours, zeros of both signs, tiny and huge values and 2^16
            // random ones on gfx950: identical.
            float t[8];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                t[2 * i] = rs.div(__uint_as_float(v[i] << 16));
                t[2 * i + 1] = rs.div(__uint_as_float(v[i] & 0xffff0000u));
            }
            w = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w, t[0], t[4], 1.0f, 0);
            w = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w, t[1], t[5], 1.0f, 1);
            w = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w, t[2], t[6], 1.0f, 2);
            w = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w, t[3], t[7], 1.0f, 3);
        }
        ((uint32_t *)(codes + row * (K / 2)))[c] = w;   // e2m1: 4 bytes per 8 elements
        return;
    }
    ((u32x2 *)(codes + row * K))[c] = e4m3_quantize_bf16x8(rs, v);   // e4m3: 8 bytes per 8 elements
}

// Rows of at most 1024 elements (the intermediate of the MoE layer has 768): a wavefront takes four rows and requests
// all of them before it reduces the first, so that it has 3-8 KB in flight instead of 1.5-2; same arithmetic per row
// as the kernel below (identical bytes).
template <bool FP4>
__global__ __launch_bounds__(kF8Threads) void quantize_fp8_short_rows_kernel(const uint16_t *__restrict__ x, int64_t rows, int K,
                                                                             uint8_t *__restrict__ codes, float *__restrict__ scales)
{
    constexpr int kRowsPerWave = 4;
    const int lane = threadIdx.x & 63;
    const int64_t row0 = ((int64_t)blockIdx.x * (kF8Threads / 64) + (threadIdx.x >> 6)) * kRowsPerWave;
    const int n16 = K / 8;   // <= 128
    u32x4 held[kRowsPerWave][2];
#pragma unroll
    for (int r = 0; r < kRowsPerWave; ++r) {
        const u32x4 *xr = (const u32x4 *)(x + min(row0 + r, rows - 1) * K);
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            held[r][u] = u32x4{0, 0, 0, 0};
            if (lane + 64 * u < n16) held[r][u] = xr[lane + 64 * u];
        }
    }
#pragma unroll
    for (int r = 0; r < kRowsPerWave; ++r) {
        const int64_t row = row0 + r;
        if (row >= rows) break;
        const float am = wave_max(absmax_bf16x8(held[r][1], absmax_bf16x8(held[r][0], 0.f)));
        const float s = am / (FP4 ? 6.0f : 448.0f);
        if (lane == 0) scales[row] = s;
        const RowScale rs(s);
#pragma unroll
        for (int u = 0; u < 2; ++u)
            if (lane + 64 * u < n16) store_codes_bf16x8<FP4>(codes, row, K, lane + 64 * u, rs, s, held[r][u]);
    }
}

template <bool FP4>
__global__ __launch_bounds__(kF8Threads) void quantize_fp8_rows_kernel(const uint16_t *__restrict__ x,
                                                                       int64_t rows, int K,
                                                                       uint8_t *__restrict__ codes,
                                                                       float *__restrict__ scales)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * (kF8Threads / 64) + (threadIdx.x >> 6);
    if (row >= rows) return;
    const u32x4 *xr = (const u32x4 *)(x + row * K);
    const int n16 = K / 8;  // 16-byte chunks in the row
    // rows of up to kKeep * 512 elements stay in registers between the two passes; longer rows are read again
    constexpr int kKeep = 8;
    const bool keep = n16 <= kKeep * 64;
    u32x4 held[kKeep];
    float am = 0.f;
    if (keep) {
#pragma unroll
        for (int u = 0; u < kKeep; ++u) {
            const int c = lane + 64 * u;
            held[u] = u32x4{0, 0, 0, 0};
            if (c < n16) held[u] = xr[c];
        }
#pragma unroll
        for (int u = 0; u < kKeep; ++u) am = absmax_bf16x8(held[u], am);
    } else {
        for (int c = lane; c < n16; c += 64) {
            am = absmax_bf16x8(xr[c], am);
        }
    }
    am = wave_max(am);
    const float s = am / (FP4 ? 6.0f : 448.0f);
    if (lane == 0) scales[row] = s;
    const RowScale rs(s);   // x / s, correctly rounded, from one divide per row
    auto convert = [&](const u32x4 v, int c) { store_codes_bf16x8<FP4>(codes, row, K, c, rs, s, v); };
    if (keep) {
#pragma unroll
        for (int u = 0; u < kKeep; ++u)
            if (lane + 64 * u < n16) convert(held[u], lane + 64 * u);
    } else {
        for (int c = lane; c < n16; c += 64) convert(xr[c], c);
    }
}

int launch_quantize_fp8_rows(const void *x, int64_t rows, int K, void *codes, float *scales, hipStream_t s)
{
    if (rows == 0) return QARL_OK;
    const int per_block = kF8Threads / 64;
    const int64_t blocks = (rows + per_block - 1) / per_block;
    if (blocks > 0x7fffffffLL) {
        set_error("quantize_fp8: %lld blocks exceed the grid limit", (long long)blocks);
        return QARL_ERR_UNSUPPORTED;
    }
    if (K <= 1024) {   // short rows: four per wavefront
        const int64_t b4 = (blocks + 3) / 4;
        quantize_fp8_short_rows_kernel<false><<<dim3((unsigned)b4), dim3(kF8Threads), 0, s>>>((const uint16_t *)x, rows, K,
                                                                                           (uint8_t *)codes, scales);
        return check_hip(hipGetLastError(), "quantize_fp8_short_rows_kernel");
    }
    quantize_fp8_rows_kernel<false><<<dim3((unsigned)blocks), dim3(kF8Threads), 0, s>>>(
        (const uint16_t *)x, rows, K, (uint8_t *)codes, scales);
    return check_hip(hipGetLastError(), "quantize_fp8_rows_kernel");
}

int launch_quantize_fp4_rows(const void *x, int64_t rows, int K, void *codes, float *scales, hipStream_t s)
{
    if (rows == 0) return QARL_OK;
    const int per_block = kF8Threads / 64;
    const int64_t blocks = (rows + per_block - 1) / per_block;
    if (blocks > 0x7fffffffLL) {
        set_error("quantize_fp4: %lld blocks exceed the grid limit", (long long)blocks);
        return QARL_ERR_UNSUPPORTED;
    }
    if (K <= 1024) {   // short rows: four per wavefront
        const int64_t b4 = (blocks + 3) / 4;
        quantize_fp8_short_rows_kernel<true><<<dim3((unsigned)b4), dim3(kF8Threads), 0, s>>>((const uint16_t *)x, rows, K,
                                                                                           (uint8_t *)codes, scales);
        return check_hip(hipGetLastError(), "quantize_fp4_short_rows_kernel");
    }
    quantize_fp8_rows_kernel<true><<<dim3((unsigned)blocks), dim3(kF8Threads), 0, s>>>(
        (const uint16_t *)x, rows, K, (uint8_t *)codes, scales);
    return check_hip(hipGetLastError(), "quantize_fp4_rows_kernel");
}

// ---- canonical view of the packed 4-bit codes, for consumers outside this library (the low-bit tensors of section
// 3.1 are published to the rollout engine after every update): row-major words [rows][K/8], element i of a word
// in bits [4i, 4i+3].  int4: offset-binary q + 8 (the library's own layout is 1 KiB blocks of 16 rows x 128 k with
// the elements of a word at the bit positions int4_bit_pos gives); e2m1: the code itself (the library packs element
// b and 4 + b into byte b).  One thread per output word.
template <bool FP4>
__global__ __launch_bounds__(256) void canonical_codes_kernel(const uint32_t *__restrict__ src, int64_t rows, int K,
                                                              uint32_t *__restrict__ dst)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int wpr = K / 8;
    if (i >= rows * wpr) return;
    const int64_t row = i / wpr;
    const int kw = (int)(i - row * wpr);   // word of the row: k in [8 kw, 8 kw + 8)
    uint32_t w, o = 0;
    if (FP4) {
        w = src[i];
#pragma unroll
        for (int e = 0; e < 8; ++e) o |= ((w >> (4 * ((e & 3) * 2 + (e >> 2)))) & 15u) << (4 * e);
    } else {
        // block (row / 16, g = kw / 16): [4 = (k % 128) / 32][16 = row % 16][4 = (k % 32) / 8] words
        const int G = K / kGroup, g = kw >> 4, q = (kw >> 2) & 3, j = kw & 3;
        w = src[((row >> 4) * G + g) * 256 + q * 64 + (row & 15) * 4 + j];
#pragma unroll
        for (int e = 0; e < 8; ++e) o |= (__builtin_rotateright32(w, int4_bit_pos(e)) & 15u) << (4 * e);
    }
    dst[i] = o;
}

int launch_canonical_codes(int fmt, const void *codes, int64_t rows, int K, void *out, hipStream_t s)
{
    const int64_t n = rows * (K / 8);
    if (n == 0) return QARL_OK;
    const int64_t blocks = (n + 255) / 256;
    if (blocks > 0x7fffffffLL) {
        set_error("canonical codes: grid too large");
        return QARL_ERR_UNSUPPORTED;
    }
    if (fmt == QARL_FP4_E2M1_CH)
        canonical_codes_kernel<true><<<dim3((unsigned)blocks), dim3(256), 0, s>>>((const uint32_t *)codes, rows, K, (uint32_t *)out);
    else
        canonical_codes_kernel<false><<<dim3((unsigned)blocks), dim3(256), 0, s>>>((const uint32_t *)codes, rows, K, (uint32_t *)out);
    return check_hip(hipGetLastError(), "canonical_codes_kernel");
}

// ---- format bridge of the W4A8 scheme.
// e4m3 bytes -> the bf16 values they stand for (exact: four significant bits): lets the W4A16 kernels run on
// e4m3 activations, whose row scale they apply in the epilogue.  One thread per 8 bytes.
__global__ __launch_bounds__(256) void e4m3_to_bf16_kernel(const u32x2 *__restrict__ src, int64_t n8,
                                                           u32x4 *__restrict__ dst)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n8) return;
    const u32x2 v = src[i];
    u32x4 o;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const float f0 = __builtin_amdgcn_cvt_f32_fp8((int)v[h], 0), f1 = __builtin_amdgcn_cvt_f32_fp8((int)v[h], 1);
        const float f2 = __builtin_amdgcn_cvt_f32_fp8((int)v[h], 2), f3 = __builtin_amdgcn_cvt_f32_fp8((int)v[h], 3);
        o[2 * h] = (__float_as_uint(f0) >> 16) | (__float_as_uint(f1) & 0xffff0000u);       // exact: low 16 bits are zero
        o[2 * h + 1] = (__float_as_uint(f2) >> 16) | (__float_as_uint(f3) & 0xffff0000u);
    }
    dst[i] = o;
}

int launch_e4m3_to_bf16(const void *x8, int64_t n, void *x16, hipStream_t s)
{
    const int64_t n8 = n / 8;
    if (n8 == 0) return QARL_OK;
    const int64_t blocks = (n8 + 255) / 256;
    if (blocks > 0x7fffffffLL) {
        set_error("e4m3 -> bf16: grid too large");
        return QARL_ERR_UNSUPPORTED;
    }
    e4m3_to_bf16_kernel<<<dim3((unsigned)blocks), dim3(256), 0, s>>>((const u32x2 *)x8, n8, (u32x4 *)x16);
    return check_hip(hipGetLastError(), "e4m3_to_bf16_kernel");
}

}  // namespace qarl
