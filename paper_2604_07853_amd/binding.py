"""Thin ctypes binding of include/qarl.h: argument marshalling only.

Every function has the name of the C entry point it calls.  Tensors are torch CUDA tensors
(device memory and streams are all PyTorch is used for); each call enqueues on torch's
current stream.  There is no CPU fallback: if libqarl.so is missing the import of `lib()`
fails loudly.
"""
import ctypes as C
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libqarl.so")

QARL_OK = 0
QARL_ERR_INVALID_ARG, QARL_ERR_UNSUPPORTED, QARL_ERR_ALIGNMENT, QARL_ERR_WORKSPACE, QARL_ERR_HIP = -1, -2, -3, -4, -5
QARL_W4A16_G128, QARL_FP8_E4M3_CH, QARL_FP4_E2M1_CH, QARL_W4A8_G128 = 1, 2, 3, 4
INT4_FORMATS = (QARL_W4A16_G128, QARL_W4A8_G128)          # int4 g128 codes + bf16 group scales
ROUTED_FORMATS = (QARL_W4A16_G128, QARL_FP8_E4M3_CH, QARL_FP4_E2M1_CH, QARL_W4A8_G128)
E4M3_ACT_FORMATS = (QARL_FP8_E4M3_CH, QARL_FP4_E2M1_CH, QARL_W4A8_G128)   # e4m3 activations + row scales
QARL_PATH_AUTO, QARL_PATH_DECODE, QARL_PATH_PREFILL = 0, 1, 2
QARL_EPI_NONE, QARL_EPI_SILU_MUL, QARL_EPI_COMBINE = 0, 1, 2
QARL_OUT_BF16, QARL_OUT_F32 = 0, 1

# the first six return a string or a size, the rest a qarl_status
EXPORTS = ["qarl_last_error", "qarl_qgemm_workspace_bytes", "qarl_logprob_workspace_bytes",
           "qarl_token_logprob_static_limit", "qarl_codes_bytes", "qarl_scales_bytes", "qarl_quantize_weights", "qarl_quantize_rows_fp8", "qarl_moe_route", "qarl_qgemm_grouped",
           "qarl_qgemm_routed", "qarl_token_logprob", "qarl_logprob_mismatch", "qarl_tbpo_objective",
           "qarl_token_logprob_static", "qarl_codes_to_canonical", "qarl_qgemm_grouped_dx",
           "qarl_grouped_dw"]


class QarlError(RuntimeError):
    def __init__(self, status, text):
        super().__init__("qarl status %d: %s" % (status, text))
        self.status = status


class qarl_qweight(C.Structure):
    _fields_ = [("fmt", C.c_int32), ("E", C.c_int32), ("N", C.c_int32), ("K", C.c_int32),
                ("group", C.c_int32), ("codes", C.c_void_p), ("scales", C.c_void_p)]


_lib = None


def lib():
    """Load libqarl.so (built by paper_2604_07853_amd/build.py); raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("HIP library %s is missing: run `python -m paper_2604_07853_amd.build` "
                              "(or __graft_entry__.build()) first; there is no fallback path" % LIB_PATH)
        L = C.CDLL(LIB_PATH)
        L.qarl_last_error.restype = C.c_char_p
        L.qarl_qgemm_workspace_bytes.restype = C.c_size_t
        L.qarl_qgemm_workspace_bytes.argtypes = [C.POINTER(qarl_qweight), C.c_int64, C.c_int64, C.c_int]
        L.qarl_logprob_workspace_bytes.restype = C.c_size_t
        L.qarl_logprob_workspace_bytes.argtypes = [C.c_int, C.c_int, C.c_int]
        L.qarl_quantize_weights.argtypes = [C.c_void_p, C.POINTER(qarl_qweight), C.c_void_p]
        L.qarl_quantize_rows_fp8.argtypes = [C.c_void_p, C.c_int64, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p]
        L.qarl_moe_route.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int] + [C.c_void_p] * 7
        L.qarl_qgemm_grouped.argtypes = [C.POINTER(qarl_qweight), C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p,
                                         C.c_void_p, C.c_int64, C.c_int, C.c_void_p, C.c_void_p, C.c_int, C.c_int,
                                         C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_size_t, C.c_void_p]
        L.qarl_qgemm_routed.argtypes = [C.POINTER(qarl_qweight), C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_int,
                                        C.c_int, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_size_t, C.c_void_p]
        L.qarl_token_logprob.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_float,
                                         C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_float, C.c_void_p,
                                         C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.qarl_logprob_mismatch.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_float,
                                            C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.qarl_tbpo_objective.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_void_p,
                                          C.c_float, C.c_float, C.c_float, C.c_float, C.c_float] + [C.c_void_p] * 8
        for fn in (L.qarl_codes_bytes, L.qarl_scales_bytes):
            fn.restype = C.c_size_t
            fn.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int]
        L.qarl_codes_to_canonical.argtypes = [C.POINTER(qarl_qweight), C.c_void_p, C.c_void_p]
        L.qarl_qgemm_grouped_dx.argtypes = [C.POINTER(qarl_qweight), C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p,
                                            C.c_void_p, C.c_int, C.c_void_p]
        L.qarl_grouped_dw.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int, C.c_int, C.c_int,
                                      C.c_void_p, C.c_int, C.c_void_p]
        L.qarl_token_logprob_static.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_float,
                                                C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_float, C.c_void_p,
                                                C.c_void_p, C.c_void_p, C.c_void_p]
        L.qarl_token_logprob_static_limit.restype = C.c_size_t
        L.qarl_token_logprob_static_limit.argtypes = []
        for name in EXPORTS[6:]:
            getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def _check(rc):
    if rc != QARL_OK:
        raise QarlError(rc, lib().qarl_last_error().decode())


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


class QWeight:
    """Quantized weights of E matrices [N, K]: the tensors plus the C descriptor."""

    def __init__(self, fmt, E, N, K, codes, scales):
        self.fmt, self.E, self.N, self.K = fmt, E, N, K
        self.codes, self.scales = codes, scales
        self.desc = qarl_qweight(fmt, E, N, K, 128 if fmt in INT4_FORMATS else 0,
                                 codes.data_ptr(), scales.data_ptr())

    @staticmethod
    def empty(fmt, E, N, K, device="cuda"):
        if fmt in INT4_FORMATS:
            codes = torch.empty((E, N, K // 8), dtype=torch.int32, device=device)
            scales = torch.empty((E, N, K // 128), dtype=torch.bfloat16, device=device)
        elif fmt == QARL_FP4_E2M1_CH:
            codes = torch.empty((E, N, K // 8), dtype=torch.int32, device=device)
            scales = torch.empty((E, N), dtype=torch.float32, device=device)
        else:
            codes = torch.empty((E, N, K), dtype=torch.uint8, device=device)
            scales = torch.empty((E, N), dtype=torch.float32, device=device)
        return QWeight(fmt, E, N, K, codes, scales)


def qarl_quantize_weights(w, fmt=QARL_W4A16_G128, out=None):
    """w bf16 [E, N, K] -> QWeight (codes + scales written by the quantize kernel)."""
    assert w.dtype == torch.bfloat16 and w.is_cuda and w.is_contiguous() and w.dim() == 3
    E, N, K = w.shape
    if out is None:
        out = QWeight.empty(fmt, E, N, K, w.device)
    _check(lib().qarl_quantize_weights(_ptr(w), C.byref(out.desc), _stream()))
    return out


def qarl_codes_to_canonical(W, out=None):
    """Codes of W in the layout-free packing of include/qarl.h: int32 words [E, N, K/8] (4-bit formats) or uint8 [E, N, K]."""
    if out is None:
        if W.fmt == QARL_FP8_E4M3_CH:
            out = torch.empty((W.E, W.N, W.K), dtype=torch.uint8, device=W.codes.device)
        else:
            out = torch.empty((W.E, W.N, W.K // 8), dtype=torch.int32, device=W.codes.device)
    assert out.numel() * out.element_size() == lib().qarl_codes_bytes(W.fmt, W.E, W.N, W.K)
    _check(lib().qarl_codes_to_canonical(C.byref(W.desc), _ptr(out), _stream()))
    return out


def qarl_quantize_rows_fp8(x, codes=None, scales=None):
    """x bf16 [rows, K] -> (e4m3 codes uint8 [rows, K], fp32 scales [rows])."""
    assert x.dtype == torch.bfloat16 and x.is_cuda and x.is_contiguous() and x.dim() == 2
    rows, K = x.shape
    if codes is None:
        codes = torch.empty((rows, K), dtype=torch.uint8, device=x.device)
    if scales is None:
        scales = torch.empty((rows,), dtype=torch.float32, device=x.device)
    _check(lib().qarl_quantize_rows_fp8(_ptr(x), rows, K, _ptr(codes), _ptr(scales), _stream()))
    return codes, scales


class Routing:
    """Outputs of qarl_moe_route."""

    def __init__(self, T, E, topk, device):
        i32 = dict(dtype=torch.int32, device=device)
        self.T, self.E, self.topk = T, E, topk
        self.ids = torch.empty((T, topk), **i32)
        self.w = torch.empty((T, topk), dtype=torch.float32, device=device)
        self.counts = torch.empty((E,), **i32)
        self.offsets = torch.empty((E + 1,), **i32)
        self.pairs = torch.empty((T * topk,), **i32)
        self.tokens = torch.empty((T * topk,), **i32)


def qarl_moe_route(logits, topk=8, renorm=True, out=None, group=True):
    """group=False: ids and weights only (the grouping outputs of `out` keep their old contents)."""
    assert logits.dtype == torch.bfloat16 and logits.is_cuda and logits.is_contiguous() and logits.dim() == 2
    T, E = logits.shape
    r = out if out is not None else Routing(T, E, topk, logits.device)
    if group:
        _check(lib().qarl_moe_route(_ptr(logits), T, E, topk, int(renorm), _ptr(r.ids), _ptr(r.w), _ptr(r.counts),
                                    _ptr(r.offsets), _ptr(r.pairs), _ptr(r.tokens), _stream()))
    else:
        _check(lib().qarl_moe_route(_ptr(logits), T, E, topk, int(renorm), _ptr(r.ids), _ptr(r.w), None, None, None,
                                    None, _stream()))
    return r


def qarl_qgemm_workspace_bytes(W, x_rows, M, epilogue):
    return lib().qarl_qgemm_workspace_bytes(C.byref(W.desc), x_rows, M, epilogue)


def qarl_qgemm_grouped(W, x, expert_offsets, M, row_map=None, x_scales=None, epilogue=QARL_EPI_NONE,
                       combine_w=None, sorted_pairs=None, T=0, topk=0, out=None, out_dtype=QARL_OUT_BF16,
                       path=QARL_PATH_AUTO, ws=None):
    """Grouped quantized GEMM; see include/qarl.h.  Allocates `out` / `ws` when not given."""
    dev = x.device
    N = W.N
    if out is None:
        dt = torch.float32 if out_dtype == QARL_OUT_F32 else torch.bfloat16
        if epilogue == QARL_EPI_COMBINE:
            out = torch.empty((T, N), dtype=dt, device=dev)
        elif epilogue == QARL_EPI_SILU_MUL:
            out = torch.empty((M, N // 2), dtype=dt, device=dev)
        else:
            out = torch.empty((M, N), dtype=dt, device=dev)
    need = qarl_qgemm_workspace_bytes(W, x.shape[0], M, epilogue)
    if ws is None and need:
        ws = torch.empty((need,), dtype=torch.uint8, device=dev)
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    _check(lib().qarl_qgemm_grouped(C.byref(W.desc), _ptr(x), _ptr(x_scales), x.shape[0], _ptr(row_map),
                                    _ptr(expert_offsets), M, epilogue, _ptr(combine_w), _ptr(sorted_pairs), T, topk,
                                    _ptr(out), out_dtype, path, _ptr(ws), ws_bytes, _stream()))
    return out


def qarl_qgemm_routed(W, x, topk_ids, T, topk, x_per_token, epilogue=QARL_EPI_NONE, combine_w=None, out=None,
                      out_dtype=QARL_OUT_BF16, ws=None):
    """Grouped quantized GEMM driven by the router's ids; see include/qarl.h.  Allocates `out` / `ws` when not given."""
    dev = x.device
    N, M = W.N, T * topk
    if out is None:
        dt = torch.float32 if out_dtype == QARL_OUT_F32 else torch.bfloat16
        if epilogue == QARL_EPI_COMBINE:
            out = torch.empty((T, N), dtype=dt, device=dev)
        elif epilogue == QARL_EPI_SILU_MUL:
            out = torch.empty((M, N // 2), dtype=dt, device=dev)
        else:
            out = torch.empty((M, N), dtype=dt, device=dev)
    need = qarl_qgemm_workspace_bytes(W, x.shape[0], M, epilogue)
    if ws is None and need:
        ws = torch.empty((need,), dtype=torch.uint8, device=dev)
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    _check(lib().qarl_qgemm_routed(C.byref(W.desc), _ptr(x), int(bool(x_per_token)), _ptr(topk_ids), T, topk, epilogue,
                                   _ptr(combine_w), _ptr(out), out_dtype, _ptr(ws), ws_bytes, _stream()))
    return out


def qarl_qgemm_grouped_dx(W, dy, expert_offsets, M, out_row_map=None, out=None, out_dtype=QARL_OUT_BF16):
    """Input gradient of the grouped W4A16 GEMM (straight-through backward); see include/qarl.h."""
    if out is None:
        out = torch.empty((M, W.K), dtype=torch.float32 if out_dtype == QARL_OUT_F32 else torch.bfloat16, device=dy.device)
    _check(lib().qarl_qgemm_grouped_dx(C.byref(W.desc), _ptr(dy), _ptr(expert_offsets), M, _ptr(out_row_map), _ptr(out),
                                       out_dtype, _stream()))
    return out


def qarl_grouped_dw(dy, x, expert_offsets, E, row_map=None, out=None, out_dtype=QARL_OUT_BF16):
    """Weight gradient dy^T x per expert (passed straight to the masters); see include/qarl.h."""
    M, N = dy.shape
    K = x.shape[1]
    if out is None:
        out = torch.empty((E, N, K), dtype=torch.float32 if out_dtype == QARL_OUT_F32 else torch.bfloat16, device=dy.device)
    _check(lib().qarl_grouped_dw(_ptr(dy), _ptr(x), _ptr(row_map), _ptr(expert_offsets), M, E, N, K, _ptr(out), out_dtype,
                                 _stream()))
    return out


def qarl_logprob_workspace_bytes(T, H, V):
    return lib().qarl_logprob_workspace_bytes(T, H, V)


def qarl_token_logprob(h, w_lm, target, inv_temperature=1.0, ref_logprob=None, seq_offsets=None, tis_cap_c=2.0,
                       ws=None, want_delta=False):
    """Returns dict(logprob[, delta, seq_w, seq_w_clipped])."""
    T, H = h.shape
    V = w_lm.shape[0]
    dev = h.device
    lp = torch.empty((T,), dtype=torch.float32, device=dev)
    need = lib().qarl_logprob_workspace_bytes(T, H, V)
    if ws is None:
        ws = torch.empty((max(need, 16),), dtype=torch.uint8, device=dev)
    S = 0 if seq_offsets is None else seq_offsets.numel() - 1
    delta = torch.empty((T,), dtype=torch.float32, device=dev) if (ref_logprob is not None and want_delta) else None
    seq_w = torch.empty((S,), dtype=torch.float32, device=dev) if (ref_logprob is not None and S > 0) else None
    seq_wc = torch.empty((S,), dtype=torch.float32, device=dev) if (ref_logprob is not None and S > 0) else None
    _check(lib().qarl_token_logprob(_ptr(h), _ptr(w_lm), _ptr(target), T, H, V, inv_temperature, _ptr(lp),
                                    _ptr(ref_logprob), _ptr(seq_offsets), S, tis_cap_c, _ptr(delta), _ptr(seq_w),
                                    _ptr(seq_wc), _ptr(ws), ws.numel(), _stream()))
    return dict(logprob=lp, delta=delta, seq_w=seq_w, seq_w_clipped=seq_wc)


def qarl_token_logprob_static_limit():
    return lib().qarl_token_logprob_static_limit()


def qarl_token_logprob_static(h, w_lm, target, logprob, inv_temperature=1.0):
    """qarl_token_logprob on the library's built-in scratch; writes the caller's `logprob` [T] and allocates nothing."""
    T, H = h.shape
    V = w_lm.shape[0]
    _check(lib().qarl_token_logprob_static(_ptr(h), _ptr(w_lm), _ptr(target), T, H, V, inv_temperature, _ptr(logprob),
                                           None, None, 0, 2.0, None, None, None, _stream()))
    return logprob


def qarl_logprob_mismatch(lp_learner, lp_sampler, seq_offsets=None, tis_cap_c=2.0):
    T = lp_learner.numel()
    dev = lp_learner.device
    S = 0 if seq_offsets is None else seq_offsets.numel() - 1
    delta = torch.empty((T,), dtype=torch.float32, device=dev)
    tw = torch.empty((T,), dtype=torch.float32, device=dev)
    seq_w = torch.empty((S,), dtype=torch.float32, device=dev) if S > 0 else None
    seq_wc = torch.empty((S,), dtype=torch.float32, device=dev) if S > 0 else None
    _check(lib().qarl_logprob_mismatch(_ptr(lp_learner), _ptr(lp_sampler), T, _ptr(seq_offsets), S, tis_cap_c,
                                       _ptr(delta), _ptr(tw), _ptr(seq_w), _ptr(seq_wc), _stream()))
    return dict(delta=delta, token_w=tw, seq_w=seq_w, seq_w_clipped=seq_wc)


class MoELayer:
    """One quantized MoE FFN layer driven through the C ABI: route -> gate_up (SiLU*mul) -> down (combine).
    Holds the preallocated intermediates so a step launches kernels only."""

    def __init__(self, gate_up: QWeight, down: QWeight, T, topk=8, path=QARL_PATH_AUTO, device="cuda", routed=None):
        self.gu, self.dn, self.T, self.topk, self.path = gate_up, down, T, topk, path
        self.fp8 = gate_up.fmt in E4M3_ACT_FORMATS        # e4m3 activations with per-row scales
        # decode-sized batches skip the grouping pass: the GEMMs read the router's ids themselves (and, for the
        # e4m3-activation formats, quantize the 16-bit token rows they gather)
        self.routed = (routed if routed is not None else
                       (gate_up.fmt in ROUTED_FORMATS and path == QARL_PATH_DECODE and 0 < T <= 512 and T * topk <= 4096))
        E, I, H = gate_up.E, gate_up.N // 2, gate_up.K
        self.E, self.I, self.H = E, I, H
        M = T * topk
        self.M = M
        self.routing = Routing(T, E, topk, device)
        self.a = torch.empty((M, I), dtype=torch.bfloat16, device=device)
        self.out = torch.empty((T, H), dtype=torch.bfloat16, device=device)
        need = max(qarl_qgemm_workspace_bytes(gate_up, T, M, QARL_EPI_SILU_MUL),
                   qarl_qgemm_workspace_bytes(down, M, M, QARL_EPI_COMBINE), 16)
        self.ws = torch.empty((need,), dtype=torch.uint8, device=device)
        if self.fp8 and not self.routed:
            self.xq = torch.empty((T, H), dtype=torch.uint8, device=device)
            self.sx = torch.empty((T,), dtype=torch.float32, device=device)
            self.aq = torch.empty((M, I), dtype=torch.uint8, device=device)
            self.sa = torch.empty((M,), dtype=torch.float32, device=device)

    def forward(self, x, logits):
        if self.routed:
            r = qarl_moe_route(logits, self.topk, True, out=self.routing, group=False)
            qarl_qgemm_routed(self.gu, x, r.ids, self.T, self.topk, True, epilogue=QARL_EPI_SILU_MUL, out=self.a,
                              ws=self.ws)
            qarl_qgemm_routed(self.dn, self.a, r.ids, self.T, self.topk, False, epilogue=QARL_EPI_COMBINE,
                              combine_w=r.w, out=self.out, ws=self.ws)
            return self.out
        r = qarl_moe_route(logits, self.topk, True, out=self.routing)
        if self.fp8:
            qarl_quantize_rows_fp8(x, self.xq, self.sx)
            qarl_qgemm_grouped(self.gu, self.xq, r.offsets, self.M, row_map=r.tokens, x_scales=self.sx,
                               epilogue=QARL_EPI_SILU_MUL, out=self.a, path=self.path, ws=self.ws)
            qarl_quantize_rows_fp8(self.a, self.aq, self.sa)
            qarl_qgemm_grouped(self.dn, self.aq, r.offsets, self.M, x_scales=self.sa, epilogue=QARL_EPI_COMBINE,
                               combine_w=r.w, sorted_pairs=r.pairs, T=self.T, topk=self.topk, out=self.out,
                               path=self.path, ws=self.ws)
        else:
            qarl_qgemm_grouped(self.gu, x, r.offsets, self.M, row_map=r.tokens, epilogue=QARL_EPI_SILU_MUL,
                               out=self.a, path=self.path, ws=self.ws)
            qarl_qgemm_grouped(self.dn, self.a, r.offsets, self.M, epilogue=QARL_EPI_COMBINE, combine_w=r.w,
                               sorted_pairs=r.pairs, T=self.T, topk=self.topk, out=self.out, path=self.path,
                               ws=self.ws)
        return self.out


def qarl_tbpo_objective(lp_current, lp_old, lp_sampler, seq_offsets, advantage, eps_low, eps_high, delta_low,
                        delta_high, tis_cap_c=2.0, want_grad=True, out=None):
    """Sequence-level surrogate of section 3.2; see include/qarl.h.
    Returns dict(r, w_clip, r_clip, in_band, obj_seq, objective[, grad]); `out` = a dict from an earlier call of
    the same sizes, whose buffers are written again."""
    T = lp_current.numel()
    S = seq_offsets.numel() - 1
    dev = lp_current.device
    f32 = dict(dtype=torch.float32, device=dev)
    if out is not None:
        r, wc, rc, ib, ob, J = out["r"], out["w_clip"], out["r_clip"], out["in_band"], out["obj_seq"], out["objective"]
        g = out.get("grad") if want_grad else None
    else:
        r = torch.empty((S,), **f32)
        wc = torch.empty((S,), **f32)
        rc = torch.empty((S,), **f32)
        ib = torch.empty((S,), dtype=torch.int32, device=dev)
        ob = torch.empty((S,), **f32)
        J = torch.empty((1,), **f32)
        g = torch.zeros((T,), **f32) if want_grad else None
    _check(lib().qarl_tbpo_objective(_ptr(lp_current), _ptr(lp_old), _ptr(lp_sampler), T, _ptr(seq_offsets), S,
                                     _ptr(advantage), eps_low, eps_high, delta_low, delta_high, tis_cap_c, _ptr(r),
                                     _ptr(wc), _ptr(rc), _ptr(ib), _ptr(ob), _ptr(J), _ptr(g), _stream()))
    out = dict(r=r, w_clip=wc, r_clip=rc, in_band=ib, obj_seq=ob, objective=J)
    if want_grad:
        out["grad"] = g
    return out
