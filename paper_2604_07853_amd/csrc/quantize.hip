// Weight / activation quantizers: the Quant equations of section 2.2.
//   int4: integer Quant with z = 0, one bf16 scale per 128 consecutive k of a row;
//   fp8 : FP Quant with alpha = 448 (e4m3), one fp32 scale per row.
// Both are HBM-bound streams: 16-byte coalesced loads, the absmax reduced with
// wavefront shuffles, IEEE fp32 divides so that codes and scales are reproducible
// bit for bit by any IEEE implementation of the same equations.
#include "common.hpp"

namespace qarl {

// ------------------------------------------------------------------ int4 --
// A lane owns 8 consecutive k (one 16-byte load, one packed code word); 16 lanes
// own a scale group; a wavefront covers 512 consecutive k = 1 KiB of the row-major
// stream.  Each thread handles kUnroll such chunks, loads issued before use.
constexpr int kQThreads = 256;
constexpr int kQUnroll = 4;

__global__ __launch_bounds__(kQThreads) void quantize_int4_kernel(const u32x4 *__restrict__ w,
                                                                  int64_t n_chunks,
                                                                  uint32_t *__restrict__ codes,
                                                                  uint16_t *__restrict__ scales)
{
    const int64_t base = ((int64_t)blockIdx.x * kQUnroll) * kQThreads + threadIdx.x;
    u32x4 v[kQUnroll];
#pragma unroll
    for (int u = 0; u < kQUnroll; ++u) {
        int64_t c = base + (int64_t)u * kQThreads;
        v[u] = (c < n_chunks) ? __builtin_nontemporal_load(&w[c]) : u32x4{0, 0, 0, 0};
    }
#pragma unroll
    for (int u = 0; u < kQUnroll; ++u) {
        int64_t c = base + (int64_t)u * kQThreads;
        float f[8];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = __uint_as_float(v[u][i] << 16);
            f[2 * i + 1] = __uint_as_float(v[u][i] & 0xffff0000u);
        }
        float am = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) am = fmaxf(am, fabsf(f[i]));
#pragma unroll
        for (int o = 1; o < 16; o <<= 1) am = fmaxf(am, __shfl_xor(am, o, 64));
        const uint32_t sb = f32_to_bf16_bits(am / 7.0f);
        const float s = bf16_bits_to_f32(sb);
        uint32_t word = 0x88888888u;  // code 0 everywhere
        if (s != 0.f) {
            word = 0;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                float r = rintf(f[i] / s);
                r = fminf(fmaxf(r, -8.f), 7.f);
                word |= (uint32_t)((int)r + 8) << (4 * i);
            }
        }
        if (c < n_chunks) {
            __builtin_nontemporal_store(word, &codes[c]);
            if ((c & 15) == 0) scales[c >> 4] = (uint16_t)sb;
        }
    }
}

int launch_quantize_int4(const void *w, int64_t rows, int K, void *codes, void *scales, hipStream_t s)
{
    const int64_t n_chunks = rows * (int64_t)(K / 8);
    if (n_chunks == 0) return QARL_OK;
    const int64_t per_block = (int64_t)kQThreads * kQUnroll;
    const int64_t blocks = (n_chunks + per_block - 1) / per_block;
    if (blocks > 0x7fffffffLL) {
        set_error("quantize: %lld blocks exceed the grid limit", (long long)blocks);
        return QARL_ERR_UNSUPPORTED;
    }
    quantize_int4_kernel<<<dim3((unsigned)blocks), dim3(kQThreads), 0, s>>>(
        (const u32x4 *)w, n_chunks, (uint32_t *)codes, (uint16_t *)scales);
    return check_hip(hipGetLastError(), "quantize_int4_kernel");
}

// ------------------------------------------------------------------- fp8 --
// e4m3 (OCP fn) nearest-even cast of a finite float, saturating at +-448.
__device__ __forceinline__ uint32_t e4m3_from_f32(float t)
{
    const uint32_t u = __float_as_uint(t);
    const uint32_t sign = (u >> 24) & 0x80u;
    const uint32_t a = u & 0x7fffffffu;
    if (a > 0x7f800000u) return 0x7fu;
    const float af = __uint_as_float(a);
    if (af >= 448.f) return sign | 0x7eu;
    if (af < 0.015625f)  // below the smallest normal 2^-6: fixed quantum 2^-9
        return sign | (uint32_t)(int)rintf(af * 512.f);
    // normal: keep 3 mantissa bits, nearest even, carry may bump the exponent
    const uint32_t r = (a + 0x7ffffu + ((a >> 20) & 1u)) >> 20;
    return sign | (r - ((127u - 7u) << 3));
}

// One wavefront per row; the row is read twice (the second read hits cache).
constexpr int kF8Threads = 256;

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
    float am = 0.f;
    for (int c = lane; c < n16; c += 64) {
        u32x4 v = xr[c];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            am = fmaxf(am, fabsf(__uint_as_float(v[i] << 16)));
            am = fmaxf(am, fabsf(__uint_as_float(v[i] & 0xffff0000u)));
        }
    }
    am = wave_max(am);
    const float s = am / 448.0f;
    if (lane == 0) scales[row] = s;
    u32x2 *cr = (u32x2 *)(codes + row * K);
    for (int c = lane; c < n16; c += 64) {
        u32x4 v = xr[c];
        u32x2 o = {0, 0};
        if (s != 0.f) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                uint32_t lo = e4m3_from_f32(__uint_as_float(v[i] << 16) / s);
                uint32_t hi = e4m3_from_f32(__uint_as_float(v[i] & 0xffff0000u) / s);
                o[i >> 1] |= (lo | (hi << 8)) << (16 * (i & 1));
            }
        }
        cr[c] = o;
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
    quantize_fp8_rows_kernel<<<dim3((unsigned)blocks), dim3(kF8Threads), 0, s>>>(
        (const uint16_t *)x, rows, K, (uint8_t *)codes, scales);
    return check_hip(hipGetLastError(), "quantize_fp8_rows_kernel");
}

}  // namespace qarl
