"""Seeded random shapes through every grouped-GEMM entry point, format and kernel path against the oracle: expert
counts, ragged and empty experts, one heavy expert, row maps over a larger activation buffer, output widths that are
not multiples of a column block, and the routed mode with the router's own ids up to 512 tokens.  Every call is made
twice and must return the same bits (the kernels have no atomics and no order that depends on timing)."""
import numpy as np
import pytest
import torch

from paper_2604_07853_amd import synth
from gpu_util import np_bits, norm_err, norm_err_bf16, flip_fraction

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-3
TOL = {"w4a16": 2e-5, "w4a8": 2e-5, "fp8": 1e-3, "fp4": 1e-3}   # the bars of test_gpu_qgemm / test_gpu_lowbit_formats
MAX_FLIPS = 0.06
FORMATS = ["w4a16", "fp8", "fp4", "w4a8"]


@pytest.fixture(scope="module")
def q():
    from paper_2604_07853_amd import binding
    binding.lib()
    return binding


def _i32(a):
    return torch.tensor(np.asarray(a), dtype=torch.int32, device="cuda")


def _fmt_id(q, fmt):
    return {"w4a16": q.QARL_W4A16_G128, "w4a8": q.QARL_W4A8_G128, "fp8": q.QARL_FP8_E4M3_CH, "fp4": q.QARL_FP4_E2M1_CH}[fmt]


def _quantize(q, oracle, fmt, w):
    wb = np_bits(w)
    if fmt in ("w4a16", "w4a8"):
        c, s = oracle.quantize_int4(wb)
    elif fmt == "fp8":
        c, s = oracle.quantize_fp8_rows(wb)
    else:
        c, s = oracle.quantize_fp4_rows(wb)
    return c, s, q.qarl_quantize_weights(w.cuda(), _fmt_id(q, fmt))


def _ref(oracle, fmt, xb, c, s, off, rm):
    if fmt == "w4a16":
        return oracle.qgemm_w4a16(xb, c, s, off, rm)
    xq, sx = oracle.quantize_fp8_rows(xb)
    gemm = {"w4a8": oracle.qgemm_w4a8, "fp8": oracle.qgemm_fp8, "fp4": oracle.qgemm_fp4w}[fmt]
    return gemm(xq, sx, c, s, off, rm)


def _k_choices(fmt):
    return [256, 512, 768, 1024, 2048] if fmt in ("w4a16", "w4a8") else [128, 256, 384, 768, 1024, 2048]


@pytest.mark.parametrize("case", range(32))
def test_grouped_random_shape(q, oracle, case):
    rng = np.random.default_rng(41000 + case)
    fmt = FORMATS[case % 4]
    E, N = int(rng.integers(1, 10)), 32 * int(rng.integers(1, 21))
    K = int(rng.choice(_k_choices(fmt)))
    kind = (case // 4) % 3
    if kind == 0:
        rows = rng.integers(0, 40, size=E)                                   # decode-like loads
    elif kind == 1:
        rows = rng.integers(0, 150, size=E) * (rng.random(E) < 0.6)          # several tiles, empty experts
    else:
        rows = rng.integers(0, 8, size=E)
        rows[rng.integers(0, E)] = int(rng.integers(100, 400))               # one heavy expert
    rows = rows.astype(np.int64)
    if rows.sum() == 0:
        rows[0] = 3
    M = int(rows.sum())
    x_rows = M + int(rng.integers(0, 5))
    w = synth.normal_bf16((E, N, K), 0.02, seed=42000 + case)
    x = synth.normal_bf16((x_rows, K), 1.0, seed=43000 + case)
    off = np.concatenate([[0], np.cumsum(rows)]).astype(np.int32)
    rm = rng.permutation(x_rows)[:M].astype(np.int32)
    c, s, qw = _quantize(q, oracle, fmt, w)
    ref = _ref(oracle, fmt, np_bits(x), c, s, off, rm)
    a_bits, a_ref = oracle.silu_mul(ref)
    xin, sx = (x.cuda(), None) if fmt == "w4a16" else q.qarl_quantize_rows_fp8(x.cuda())
    for path in (q.QARL_PATH_DECODE, q.QARL_PATH_PREFILL):
        what = (fmt, E, N, K, rows.tolist(), path)
        call = lambda **kw: q.qarl_qgemm_grouped(qw, xin, _i32(off), M, row_map=_i32(rm), x_scales=sx, path=path, **kw)
        y = call(out_dtype=q.QARL_OUT_F32)
        assert norm_err(y.cpu().numpy(), ref) <= TOL[fmt], what
        assert torch.equal(y, call(out_dtype=q.QARL_OUT_F32)), what
        a = call(epilogue=q.QARL_EPI_SILU_MUL)
        assert norm_err_bf16(a.float().cpu().numpy(), a_ref) <= TOL_BF16, what
        assert flip_fraction(np_bits(a), a_bits) <= MAX_FLIPS, what


@pytest.mark.parametrize("case", range(24))
def test_routed_random_shape(q, oracle, case):
    rng = np.random.default_rng(44000 + case)
    fmt = FORMATS[case % 4]
    T = int(rng.integers(1, 513))
    E = int(rng.choice([64, 128, 192, 256]))
    topk = int(rng.choice([1, 2, 4, 8]))
    N = 32 * int(rng.choice([1, 2, 3, 4, 6, 8, 16, 24, 48]))
    K = int(rng.choice(_k_choices(fmt)))
    w = synth.normal_bf16((E, N, K), 0.02, seed=45000 + case)
    x = synth.normal_bf16((T, K), 1.0, seed=46000 + case)
    lg = synth.router_logits(T, E, seed=47000 + case, zipf_s=float(rng.choice([0.0, 1.1])))
    c, s, qw = _quantize(q, oracle, fmt, w)
    r = q.qarl_moe_route(lg.cuda(), topk)
    ids, _ = oracle.route(np_bits(lg), topk)
    assert np.array_equal(r.ids.cpu().numpy().reshape(T, topk), ids)
    _, offsets, pairs = oracle.group(ids, E)
    ref = _ref(oracle, fmt, np_bits(x), c, s, offsets, (pairs // topk).astype(np.int32))   # rows in (expert, token, slot) order
    what = (fmt, T, E, topk, N, K)

    def call(**kw):
        out = q.qarl_qgemm_routed(qw, x.cuda(), r.ids, T, topk, True, **kw)
        return out
    y = call(out_dtype=q.QARL_OUT_F32)                     # output row = pair id t * topk + slot
    assert norm_err(y.cpu().numpy()[pairs], ref) <= TOL[fmt], what
    assert torch.equal(y, call(out_dtype=q.QARL_OUT_F32)), what
    a = call(epilogue=q.QARL_EPI_SILU_MUL)
    a_bits, a_ref = oracle.silu_mul(ref)
    assert norm_err_bf16(a.float().cpu().numpy()[pairs], a_ref) <= TOL_BF16, what
    assert flip_fraction(np_bits(a)[pairs], a_bits) <= MAX_FLIPS, what
