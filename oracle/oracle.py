"""numpy/ctypes front end of oracle/qarl_oracle.c (TEST INFRASTRUCTURE ONLY).

Every function takes and returns numpy arrays: bf16 tensors travel as uint16 bit
patterns, e4m3 tensors as uint8.  The arithmetic lives in the C file; this module only
marshals arguments.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(_build.build())
        _lib.oracle_e4m3_decode.restype = C.c_double
        _lib.oracle_e4m3_decode.argtypes = [C.c_uint8]
        _lib.oracle_e4m3_encode.restype = C.c_uint8
        _lib.oracle_e4m3_encode.argtypes = [C.c_double]
        _lib.oracle_e4m3_encode_fast.restype = C.c_uint8
        _lib.oracle_e4m3_encode_fast.argtypes = [C.c_double]
        _lib.oracle_e2m1_decode.restype = C.c_double
        _lib.oracle_e2m1_decode.argtypes = [C.c_uint8]
        _lib.oracle_e2m1_encode.restype = C.c_uint8
        _lib.oracle_e2m1_encode.argtypes = [C.c_double]
        _lib.oracle_bf16_from_double.restype = C.c_uint16
        _lib.oracle_bf16_from_double.argtypes = [C.c_double]
        _lib.oracle_bf16_to_double.restype = C.c_double
        _lib.oracle_bf16_to_double.argtypes = [C.c_uint16]
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _c(a, dt):
    a = np.ascontiguousarray(a, dtype=dt)
    return a


def cores():
    """Threads the OpenMP loops of the oracle use."""
    n = os.environ.get("OMP_NUM_THREADS")
    return int(n) if n else (os.cpu_count() or 1)


def bf16_to_f64(bits):
    bits = _c(bits, np.uint16)
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def bf16_from_f64(x):
    x = np.asarray(x, dtype=np.float64)
    f = lib().oracle_bf16_from_double
    return np.array([f(float(v)) for v in x.ravel()], dtype=np.uint16).reshape(x.shape)


def e4m3_decode(codes):
    codes = _c(codes, np.uint8)
    f = lib().oracle_e4m3_decode
    tab = np.array([f(c) for c in range(256)], dtype=np.float64)
    return tab[codes]


def e4m3_encode(x, fast=False):
    x = np.asarray(x, dtype=np.float64)
    f = lib().oracle_e4m3_encode_fast if fast else lib().oracle_e4m3_encode
    return np.array([f(float(v)) for v in x.ravel()], dtype=np.uint8).reshape(x.shape)


def e2m1_decode(codes):
    codes = _c(codes, np.uint8)
    f = lib().oracle_e2m1_decode
    tab = np.array([f(c) for c in range(16)], dtype=np.float64)
    return tab[codes & 15]


def e2m1_encode(x):
    x = np.asarray(x, dtype=np.float64)
    f = lib().oracle_e2m1_encode
    return np.array([f(float(v)) for v in x.ravel()], dtype=np.uint8).reshape(x.shape)


def quantize_fp4_rows(x_bits):
    """x_bits uint16 [..., K] -> e2m1 codes uint8 [..., K] (one per byte, 0..15), scales float32 [...]."""
    x = _c(x_bits, np.uint16)
    K = x.shape[-1]
    rows = x.size // K
    codes = np.empty(x.shape, dtype=np.uint8)
    scales = np.empty(x.shape[:-1], dtype=np.float32)
    lib().oracle_quantize_fp4_rows(_p(x), C.c_int64(rows), C.c_int(K), _p(codes), _p(scales))
    return codes, scales


def quantize_int4(w_bits, group=128):
    """w_bits uint16 [..., K] -> codes uint32 [..., K/8], scales uint16 (bf16) [..., K/group]."""
    w = _c(w_bits, np.uint16)
    K = w.shape[-1]
    rows = w.size // K
    codes = np.empty(w.shape[:-1] + (K // 8,), dtype=np.uint32)
    scales = np.empty(w.shape[:-1] + (K // group,), dtype=np.uint16)
    lib().oracle_quantize_int4(_p(w), C.c_int64(rows), C.c_int(K), C.c_int(group), _p(codes), _p(scales))
    return codes, scales


def unpack_int4(codes):
    """uint32 [..., K/8] -> int8 [..., K] logical codes q in [-8, 7] (documented packing)."""
    codes = _c(codes, np.uint32)
    sh = np.arange(8, dtype=np.uint32) * 4
    u = (codes[..., None] >> sh) & 15
    return (u.astype(np.int8) - 8).reshape(codes.shape[:-1] + (codes.shape[-1] * 8,))


def dequant_int4(codes, scales, group=128):
    codes = _c(codes, np.uint32)
    scales = _c(scales, np.uint16)
    K = codes.shape[-1] * 8
    rows = codes.size // (K // 8)
    out = np.empty(codes.shape[:-1] + (K,), dtype=np.float32)
    lib().oracle_dequant_int4(_p(codes), _p(scales), C.c_int64(rows), C.c_int(K), C.c_int(group), _p(out))
    return out


def quantize_fp8_rows(x_bits):
    """x_bits uint16 [..., K] -> codes uint8 [..., K], scales float32 [...] (one per row)."""
    x = _c(x_bits, np.uint16)
    K = x.shape[-1]
    rows = x.size // K
    codes = np.empty(x.shape, dtype=np.uint8)
    scales = np.empty(x.shape[:-1], dtype=np.float32)
    lib().oracle_quantize_fp8_rows(_p(x), C.c_int64(rows), C.c_int(K), _p(codes), _p(scales))
    return codes, scales


def route(logit_bits, topk=8, renorm=True):
    """logits uint16 [T, E] -> ids int32 [T, topk], weights float64 [T, topk]."""
    lg = _c(logit_bits, np.uint16)
    T, E = lg.shape
    ids = np.empty((T, topk), dtype=np.int32)
    w = np.empty((T, topk), dtype=np.float64)
    lib().oracle_route(_p(lg), C.c_int(T), C.c_int(E), C.c_int(topk), C.c_int(int(renorm)), _p(ids), _p(w))
    return ids, w


def group(ids, E):
    ids = _c(ids, np.int32)
    T, topk = ids.shape
    counts = np.empty(E, dtype=np.int32)
    offsets = np.empty(E + 1, dtype=np.int32)
    pairs = np.empty(T * topk, dtype=np.int32)
    lib().oracle_group(_p(ids), C.c_int(T), C.c_int(E), C.c_int(topk), _p(counts), _p(offsets), _p(pairs))
    return counts, offsets, pairs


def qgemm_w4a16(x_bits, codes, scales, offsets, row_map=None, group=128, acc32=False):
    """Grouped quantized GEMM.  codes [E, N, K/8], scales [E, N, K/group]; rows i in
    [offsets[e], offsets[e+1]) use expert e and read x[row_map[i]] (identity if None).
    Returns float64 [M, N], M = offsets[-1]."""
    x = _c(x_bits, np.uint16)
    codes = _c(codes, np.uint32)
    scales = _c(scales, np.uint16)
    offsets = _c(offsets, np.int32)
    E, N, K8 = codes.shape
    K = K8 * 8
    M = int(offsets[-1])
    rm = None if row_map is None else _c(row_map, np.int32)
    out = np.zeros((M, N), dtype=np.float64)
    lib().oracle_qgemm_w4a16(_p(x), C.c_int(K), _p(rm), C.c_int64(M), _p(offsets), C.c_int(E),
                             _p(codes), _p(scales), C.c_int(N), C.c_int(group),
                             C.c_int(int(acc32)), _p(out))
    return out


def qgemm_w4a16_dx(dy_bits, codes, scales, offsets, group=128):
    """Input gradient of the grouped W4A16 GEMM under the straight-through estimator: dy bf16 bits [M, N] in the
    forward's output row order -> float64 [M, K]."""
    dy = _c(dy_bits, np.uint16)
    codes = _c(codes, np.uint32)
    scales = _c(scales, np.uint16)
    offsets = _c(offsets, np.int32)
    E, N, K8 = codes.shape
    K = K8 * 8
    M = int(offsets[-1])
    out = np.zeros((M, K), dtype=np.float64)
    lib().oracle_qgemm_w4a16_dx(_p(dy), C.c_int(K), C.c_int64(M), _p(offsets), C.c_int(E), _p(codes), _p(scales),
                                C.c_int(N), C.c_int(group), _p(out))
    return out


def grouped_dw(dy_bits, x_bits, offsets, E, row_map=None):
    """Weight gradient (passed straight to the masters): float64 [E, N, K] = sum over the expert's rows of dy^T x."""
    dy = _c(dy_bits, np.uint16)
    x = _c(x_bits, np.uint16)
    offsets = _c(offsets, np.int32)
    M, N = dy.shape
    K = x.shape[1]
    rm = None if row_map is None else _c(row_map, np.int32)
    out = np.zeros((E, N, K), dtype=np.float64)
    lib().oracle_grouped_dw(_p(dy), _p(x), C.c_int(K), _p(rm), C.c_int64(M), _p(offsets), C.c_int(E), C.c_int(N), _p(out))
    return out


def qgemm_fp8(xq, sx, wq, sw, offsets, row_map=None):
    xq = _c(xq, np.uint8)
    sx = _c(sx, np.float32)
    wq = _c(wq, np.uint8)
    sw = _c(sw, np.float32)
    offsets = _c(offsets, np.int32)
    E, N, K = wq.shape
    M = int(offsets[-1])
    rm = None if row_map is None else _c(row_map, np.int32)
    out = np.zeros((M, N), dtype=np.float64)
    lib().oracle_qgemm_fp8(_p(xq), _p(sx), C.c_int(K), _p(rm), C.c_int64(M), _p(offsets), C.c_int(E),
                           _p(wq), _p(sw), C.c_int(N), _p(out))
    return out


def qgemm_fp4w(xq, sx, wq, sw, offsets, row_map=None):
    """e4m3 activations x e2m1 weights (codes one per byte); returns float64 [M, N]."""
    xq = _c(xq, np.uint8)
    sx = _c(sx, np.float32)
    wq = _c(wq, np.uint8)
    sw = _c(sw, np.float32)
    offsets = _c(offsets, np.int32)
    E, N, K = wq.shape
    M = int(offsets[-1])
    rm = None if row_map is None else _c(row_map, np.int32)
    out = np.zeros((M, N), dtype=np.float64)
    lib().oracle_qgemm_fp4w(_p(xq), _p(sx), C.c_int(K), _p(rm), C.c_int64(M), _p(offsets), C.c_int(E),
                            _p(wq), _p(sw), C.c_int(N), _p(out))
    return out


def qgemm_w4a8(xq, sx, codes, scales, offsets, row_map=None, group=128):
    """e4m3 activations x int4 g128 weights; returns float64 [M, N]."""
    xq = _c(xq, np.uint8)
    sx = _c(sx, np.float32)
    codes = _c(codes, np.uint32)
    scales = _c(scales, np.uint16)
    offsets = _c(offsets, np.int32)
    E, N, K8 = codes.shape
    K = K8 * 8
    M = int(offsets[-1])
    rm = None if row_map is None else _c(row_map, np.int32)
    out = np.zeros((M, N), dtype=np.float64)
    lib().oracle_qgemm_w4a8(_p(xq), _p(sx), C.c_int(K), _p(rm), C.c_int64(M), _p(offsets), C.c_int(E),
                            _p(codes), _p(scales), C.c_int(N), C.c_int(group), _p(out))
    return out


def silu_mul(gu):
    """gu float64 [M, 2I] (gate columns first) -> (a bf16 bits [M, I], a exact float64)."""
    gu = _c(gu, np.float64)
    M, I2 = gu.shape
    I = I2 // 2
    a = np.empty((M, I), dtype=np.uint16)
    ex = np.empty((M, I), dtype=np.float64)
    lib().oracle_silu_mul(_p(gu), C.c_int64(M), C.c_int(I), _p(a), _p(ex))
    return a, ex


def combine(y, sorted_pairs, wts, T, topk):
    y = _c(y, np.float64)
    sp = _c(sorted_pairs, np.int32)
    wts = _c(wts, np.float64)
    N = y.shape[1]
    out = np.empty((T, N), dtype=np.float64)
    ob = np.empty((T, N), dtype=np.uint16)
    lib().oracle_combine(_p(y), _p(sp), _p(wts), C.c_int(T), C.c_int(topk), C.c_int(N), _p(out), _p(ob))
    return out, ob


def token_logprob(h_bits, wlm_bits, target, inv_temp=1.0):
    h = _c(h_bits, np.uint16)
    w = _c(wlm_bits, np.uint16)
    tg = _c(target, np.int32)
    T, H = h.shape
    V = w.shape[0]
    lp = np.empty(T, dtype=np.float64)
    lib().oracle_token_logprob(_p(h), _p(w), _p(tg), C.c_int(T), C.c_int(H), C.c_int(V),
                               C.c_double(inv_temp), _p(lp))
    return lp


def mismatch(lp_learner, lp_sampler, seq_offsets, c=2.0):
    a = _c(lp_learner, np.float64)
    b = _c(lp_sampler, np.float64)
    so = _c(seq_offsets, np.int32)
    S = so.size - 1
    T = a.size
    delta = np.zeros(T)
    w = np.ones(T)
    ws = np.empty(S)
    wc = np.empty(S)
    lib().oracle_mismatch(_p(a), _p(b), _p(so), C.c_int(S), C.c_double(c), _p(delta), _p(w), _p(ws), _p(wc))
    return delta, w, ws, wc


def tbpo(lp_cur, lp_old, lp_smp, seq_offsets, adv, eps_low, eps_high, delta_low, delta_high, c=2.0):
    """Sequence-level surrogate (section 3.2); returns dict(r, w_clip, r_clip, in_band, obj_seq, objective, grad)."""
    a = _c(lp_cur, np.float64)
    b = _c(lp_old, np.float64)
    d = _c(lp_smp, np.float64)
    so = _c(seq_offsets, np.int32)
    av = _c(adv, np.float64)
    S = so.size - 1
    r = np.empty(S)
    wc = np.empty(S)
    rc = np.empty(S)
    ib = np.empty(S, dtype=np.int32)
    ob = np.empty(S)
    J = np.zeros(1)
    g = np.zeros(a.size)
    lib().oracle_tbpo(_p(a), _p(b), _p(d), _p(so), C.c_int(S), _p(av), C.c_double(eps_low), C.c_double(eps_high),
                      C.c_double(delta_low), C.c_double(delta_high), C.c_double(c), _p(r), _p(wc), _p(rc), _p(ib),
                      _p(ob), _p(J), _p(g))
    return dict(r=r, w_clip=wc, r_clip=rc, in_band=ib, obj_seq=ob, objective=float(J[0]), grad=g)


def moe_ffn_w4a16(x_bits, logit_bits, gu_codes, gu_scales, dn_codes, dn_scales, topk=8, acc32=False):
    """Whole MoE layer (route -> gate_up -> SiLU*mul -> down -> combine), W4A16.
    Returns a dict with every intermediate."""
    E = gu_codes.shape[0]
    T = x_bits.shape[0]
    ids, w = route(logit_bits, topk)
    counts, offsets, pairs = group(ids, E)
    row_map = (pairs // topk).astype(np.int32)
    gu = qgemm_w4a16(x_bits, gu_codes, gu_scales, offsets, row_map, acc32=acc32)
    a, _ = silu_mul(gu)
    y = qgemm_w4a16(a, dn_codes, dn_scales, offsets, None, acc32=acc32)
    out, out_bf16 = combine(y, pairs, w, T, topk)
    return dict(ids=ids, w=w, counts=counts, offsets=offsets, pairs=pairs, row_map=row_map,
                gu=gu, a=a, y=y, out=out, out_bf16=out_bf16)


def moe_ffn_fp8(x_bits, logit_bits, gu_q, gu_s, dn_q, dn_s, topk=8):
    """Whole MoE layer, FP8 W8A8: per-token e4m3 activations, per-channel e4m3 weights."""
    E = gu_q.shape[0]
    T = x_bits.shape[0]
    ids, w = route(logit_bits, topk)
    counts, offsets, pairs = group(ids, E)
    row_map = (pairs // topk).astype(np.int32)
    xq, sx = quantize_fp8_rows(x_bits)
    gu = qgemm_fp8(xq, sx, gu_q, gu_s, offsets, row_map)
    a, _ = silu_mul(gu)
    aq, sa = quantize_fp8_rows(a)
    y = qgemm_fp8(aq, sa, dn_q, dn_s, offsets, None)
    out, out_bf16 = combine(y, pairs, w, T, topk)
    return dict(ids=ids, w=w, counts=counts, offsets=offsets, pairs=pairs, row_map=row_map,
                xq=xq, sx=sx, gu=gu, a=a, aq=aq, sa=sa, y=y, out=out, out_bf16=out_bf16)
