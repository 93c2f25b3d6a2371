// Shared device helpers of the QaRL hot-path kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "../../include/qarl.h"

namespace qarl {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(8))) int i32x8;
typedef __attribute__((ext_vector_type(4))) int i32x4;

constexpr int kWave = 64;
constexpr int kGroup = 128;  // k per int4 scale group

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t h) { return __uint_as_float(h << 16); }

// Round-to-nearest-even fp32 -> bf16 bit pattern (NaN kept quiet).
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

// The same conversion by the hardware instruction (round-to-nearest-even).
__device__ __forceinline__ uint16_t f32_to_bf16_hw(float f)
{
    return __builtin_bit_cast(uint16_t, (__bf16)f);
}

// silu(g) * u with g / (1 + e^-g) evaluated as g * rcp(1 + exp2(-g log2 e)): hardware exp2 and rcp,
// each within 1 ulp of fp32, far below the bf16 rounding the result goes through.
__device__ __forceinline__ float silu_mul_f32(float g, float u)
{
    const float t = __builtin_amdgcn_exp2f(g * -1.44269504088896340736f);
    return g * __builtin_amdgcn_rcpf(1.f + t) * u;
}

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// ---- FP quantizer of section 2.2 along a row, e4m3 flavour (alpha = 448), shared by the row quantizer and by the
// decode GEMM that quantizes its token rows while it gathers them, so that both produce the same bytes.
// x / s, correctly rounded, without a divide per element: with y = RN(1 / s) (one IEEE divide per row),
// q0 = RN(x y) and the exact remainder r = x - q0 s from one FMA, RN(q0 + r y) is the correctly rounded
// quotient (Markstein's correction step; it needs the correctly rounded reciprocal and no underflow on the
// way, hence the guard on s; below 2^-11 a quotient may differ from the IEEE one, where every value rounds
// to an e4m3 zero; the sign is copied from x, as s > 0).  Checked against the IEEE divide for all 65536 bf16
// values of x and 2^20 scales (the quantizer's own absmax / alpha and random ones): no difference at |x / s| >= 2^-11.
struct RowScale {
    float s, y;
    bool fast;
    __device__ __forceinline__ explicit RowScale(float s_) : s(s_), y(1.0f / s_)
    {
        fast = s_ >= 0x1p-100f && s_ < 0x1p100f && (__float_as_uint(s_) & 0x7fffffu) != 0x7fffffu;
    }
    __device__ __forceinline__ float div(float x) const
    {
        if (!fast) return x / s;
        const float q0 = x * y;
        return copysignf(fmaf(fmaf(-q0, s, x), y, q0), x);   // the sign of x also where the steps end in +0 (x = -0)
    }
};

// absmax of eight bf16 values held in four dwords, folded into am
__device__ __forceinline__ float absmax_bf16x8(u32x4 v, float am)
{
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        am = fmaxf(am, fabsf(__uint_as_float(v[i] << 16)));
        am = fmaxf(am, fabsf(__uint_as_float(v[i] & 0xffff0000u)));
    }
    return am;
}

// Eight bf16 values -> eight e4m3 bytes of x / s (zeros for a zero row).  v_cvt_pk_fp8_f32 rounds to nearest even
// into OCP e4m3 (subnormals included) for every finite |t| <= 448 (checked over all 2^32 bit patterns on gfx950
// against a software encoder); the clamp keeps the quotient of the row's absmax, which may exceed 448 by an ulp,
// in that range (and sends a NaN to -448).
__device__ __forceinline__ u32x2 e4m3_quantize_bf16x8(const RowScale &rs, u32x4 v)
{
    u32x2 o = {0, 0};
    if (rs.s != 0.f) {
        float t[8];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            t[2 * i] = __builtin_amdgcn_fmed3f(rs.div(__uint_as_float(v[i] << 16)), -448.f, 448.f);
            t[2 * i + 1] = __builtin_amdgcn_fmed3f(rs.div(__uint_as_float(v[i] & 0xffff0000u)), -448.f, 448.f);
        }
        int w0 = __builtin_amdgcn_cvt_pk_fp8_f32(t[0], t[1], 0, false);
        w0 = __builtin_amdgcn_cvt_pk_fp8_f32(t[2], t[3], w0, true);
        int w1 = __builtin_amdgcn_cvt_pk_fp8_f32(t[4], t[5], 0, false);
        w1 = __builtin_amdgcn_cvt_pk_fp8_f32(t[6], t[7], w1, true);
        o[0] = (uint32_t)w0;
        o[1] = (uint32_t)w1;
    }
    return o;
}

// A constant the optimiser cannot see through, held in a scalar (vector) register.  (a & mask) | c with such operands
// is selected as one v_and_or_b32; with literal operands the compiler emits v_and + v_or (a VOP3 encoding takes no
// literal on this target).  The operation itself must stay an instruction the compiler knows: a matrix instruction
// that reads a register needs wait states after the VALU instruction that wrote it, which the compiler inserts for
// its own instructions and cannot insert for the contents of an inline asm (with v_and_or_b32 written as inline
// asm, a matrix instruction scheduled directly behind it read the register's previous contents now and then).
__device__ __forceinline__ uint32_t opaque_sgpr(uint32_t v)
{
    asm("" : "+s"(v));
    return v;
}
__device__ __forceinline__ uint32_t opaque_vgpr(uint32_t v)
{
    asm("" : "+v"(v));
    return v;
}

// Bit position of the low bit of element e (0..7) of a packed word of int4 codes (stored as u = q+8).
// Elements 2i and 2i+1 (i < 3) sit 16 bits apart at bits 3+4i and 19+4i, i.e. already in the top four
// mantissa bits of the two bf16 halves of a dword after a right shift by 4i; element 6 sits at bits
// 15..18 and element 7 wraps around the word (its low bit at bit 31, the other three at bits 0..2), so
// that a rotation by 12 brings both into place.
__host__ __device__ constexpr int int4_bit_pos(int e) { return e < 6 ? 3 + 4 * (e >> 1) + 16 * (e & 1) : (e == 6 ? 15 : 31); }

// One packed word of eight int4 codes -> eight exact bf16 values (q+24)/16 in element order 0..7: the
// code lands in the top four mantissa bits of bf16 1.0.  Seven VALU operations per word: one and-or for
// the first pair, a shift (or the rotation) and an and-or for each of the other three.
__device__ __forceinline__ bf16x8 unpack_int4_word(uint32_t w)
{
    const uint32_t mask = opaque_sgpr(0x00780078u), one = opaque_vgpr(0x3f803f80u);
    u32x4 d;
    d[0] = (w & mask) | one;
    d[1] = ((w >> 4) & mask) | one;
    d[2] = ((w >> 8) & mask) | one;
    d[3] = (__builtin_rotateright32(w, 12) & mask) | one;
    return __builtin_bit_cast(bf16x8, d);
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also drains every outstanding
// global load of the wavefront (the workgroup-scope fence waits on vmcnt), which would stall the
// weight prefetch rings; kernels whose cross-wavefront traffic goes through LDS alone use this.
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Asynchronous global -> LDS copy of one wavefront: active lane L's 16 bytes land at lds_dst + 16 L.
// lds_dst must be the same in all lanes.  Completion is counted by vmcnt, in order with the
// wavefront's other vector loads.
__device__ __forceinline__ void copy16_to_lds(const void *gsrc, void *lds_dst)
{
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)gsrc,
                                     (__attribute__((address_space(3))) void *)lds_dst, 16, 0, 0);
}

// Barrier for LDS buffers filled by copy16_to_lds: every wavefront first waits for its own copies
// (and LDS operations), then for the others.
__device__ __forceinline__ void copy_barrier()
{
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Host-side error plumbing (api.hip).
void set_error(const char *fmt, ...);
int check_hip(hipError_t e, const char *what);

// Kernels that take more than the default 64 KiB of dynamic LDS need their limit raised once per device.
// Every caller raises it to the same value (the 160 KiB of a gfx950 CU less the kernel's static LDS), so concurrent host threads cannot
// undo each other; `done` (one object per kernel instantiation, zero-initialised) remembers the devices served.
constexpr int kMaxLdsBytes = 160 * 1024;
struct LdsLimitOnce {
    std::atomic<unsigned> devices_done[2];   // bit d of word d / 32: device d (devices >= 64 are set every call)
};
int raise_lds_limit(const void *kernel, LdsLimitOnce &done, const char *what);

// Kernel launchers (one per .hip file); all validate nothing: api.hip does.
int launch_quantize_int4(const void *w, int64_t rows, int K, void *codes, void *scales, hipStream_t s);
int launch_quantize_fp8_rows(const void *x, int64_t rows, int K, void *codes, float *scales, hipStream_t s);
int launch_quantize_fp4_rows(const void *x, int64_t rows, int K, void *codes, float *scales, hipStream_t s);
int launch_canonical_codes(int fmt, const void *codes, int64_t rows, int K, void *out, hipStream_t s);
int launch_e4m3_to_bf16(const void *x8, int64_t n, void *x16, hipStream_t s);               // e4m3 bytes -> bf16 (exact)
int launch_route_only(const void *logits, int T, int E, int topk, int renorm, int32_t *ids, float *w, hipStream_t s);
int launch_route(const void *logits, int T, int E, int topk, int renorm, int32_t *ids, float *w,
                 int32_t *counts, int32_t *offsets, int32_t *pairs, int32_t *tokens, hipStream_t s);

struct GemmArgs {
    int fmt;
    int E, N, K;
    const void *codes;
    const void *scales;
    const void *x;
    const float *x_scales;       // FP8 / FP4: scale of each activation row; W4A8: the same, applied in the epilogue
    const float *x_group_sums;   // W4A16 prefill path: -1.5 * sum of x over each 128-k group, [x_rows][K/128]
    const int32_t *row_map;      // gather of activation rows, or null
    const int32_t *out_row_map;  // scatter of output rows, or null
    const int32_t *offsets;
    int64_t M;
    int64_t x_rows;     // rows of x (bound of row_map values)
    int epilogue;       // NONE or SILU_MUL here; COMBINE is NONE into ws + combine kernel
    void *out;          // [M][N] or [M][N/2]
    int out_f32;
    // routed mode of the decode kernels (ids != null; offsets and row maps unused): row = pair id
    // t * topk + slot of expert ids[row], activation row t (x_per_token) or the pair id, output row = pair id;
    // x is bf16 for every format (the e4m3-activation formats quantize the rows they gather)
    const int32_t *ids = nullptr;
    int topk = 0;
    int x_per_token = 0;
};
int launch_qgemm_stream(const GemmArgs &a, hipStream_t s);
bool qgemm_stream_supported(int fmt, int N, int K);
bool qgemm_stream_routed_supported(int fmt, int N, int K, int T, int topk);
int launch_qgemm_stream_w4(const GemmArgs &a, hipStream_t s);
bool qgemm_stream_w4_supported(int N, int K);
bool qgemm_stream_w4_routed_supported(int N, int K, int T, int topk);
int launch_qgemm_tile(const GemmArgs &a, hipStream_t s);
int launch_qgemm_tile_fp8(const GemmArgs &a, hipStream_t s);
// Straight-through backward of the W4A16 grouped GEMM: a.x = dY bf16 [M][N], a.out = dX [M][K]
int launch_qgemm_dx(const GemmArgs &a, hipStream_t s);
int launch_grouped_dw(const void *dy, const void *x, const int32_t *row_map, const int32_t *offsets, int E, int N, int K,
                      void *out, int out_f32, hipStream_t s);
int launch_group_sums(const void *x_bf16, int64_t rows, int K, float *sums, hipStream_t s);
int launch_combine(const float *y_pair_order, const float *w, int T, int topk, int N, void *out, int out_f32,
                   hipStream_t s);
int launch_logprob(const void *h, const void *wlm, const int32_t *target, int T, int H, int V,
                   float inv_temp, float *logprob, void *ws, hipStream_t s);
size_t logprob_ws_bytes(int T, int H, int V);
// Device address, on the current device, of the library's own file-scope scratch array (kLogprobScratchBytes).
constexpr size_t kLogprobScratchBytes = (size_t)4 << 20;
int logprob_static_scratch(void **ptr);
int launch_fill_f32(float *p, int n, float v, hipStream_t s);
int launch_tbpo(const float *lp_cur, const float *lp_old, const float *lp_smp, const int32_t *seq_offsets, int S,
                const float *adv, float eps_low, float eps_high, float delta_low, float delta_high, float c,
                float *r_seq, float *w_clip, float *r_clip, int32_t *in_band, float *obj_seq, float *objective,
                float *grad, hipStream_t s);
int launch_mismatch(const float *lp_a, const float *lp_b, int T, const int32_t *seq_offsets, int S, float c,
                    float *delta, float *token_w, float *seq_w, float *seq_wc, hipStream_t s);

}  // namespace qarl
