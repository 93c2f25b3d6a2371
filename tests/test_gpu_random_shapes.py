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


@pytest.mark.parametrize("case", range(16))
def test_quantizers_router_logprob_backward_random_shape(q, oracle, case):
    """The other entry points on random sizes: the three weight quantizers and the row quantizer (bit-exact, weight
    magnitudes from 1e-3 to 300), router + grouping (bit-exact, weights 1e-6), the fused log-prob (1e-4) and both
    gradients of the straight-through backward (the bars of test_gpu_backward)."""
    from gpu_util import unblock_int4
    rng = np.random.default_rng(48000 + case)
    E, N, K = int(rng.integers(1, 5)), 32 * int(rng.integers(1, 9)), 128 * int(rng.integers(1, 33))
    std = float(rng.choice([1e-3, 0.02, 1.0, 300.0]))
    w = synth.normal_bf16((E, N, K), std, seed=48100 + case)
    c, s = oracle.quantize_int4(np_bits(w))
    qw = q.qarl_quantize_weights(w.cuda(), q.QARL_W4A16_G128)
    assert np.array_equal(qw.scales.cpu().view(torch.int16).numpy().view(np.uint16), s), (E, N, K, std)
    assert np.array_equal(unblock_int4(qw.codes, E, N, K), c), (E, N, K, std)
    c, s = oracle.quantize_fp8_rows(np_bits(w))
    qw = q.qarl_quantize_weights(w.cuda(), q.QARL_FP8_E4M3_CH)
    assert np.array_equal(qw.scales.cpu().numpy(), s) and np.array_equal(qw.codes.cpu().numpy(), c), (E, N, K, std)
    c, s = oracle.quantize_fp4_rows(np_bits(w))
    qw = q.qarl_quantize_weights(w.cuda(), q.QARL_FP4_E2M1_CH)
    assert np.array_equal(qw.scales.cpu().numpy(), s), (E, N, K, std)
    want = np.zeros((E, N, K // 8), dtype=np.uint32)           # the oracle's one code per byte -> nibble i of a word
    for i in range(8):
        want |= c.reshape(E, N, K // 8, 8)[..., i].astype(np.uint32) << np.uint32(4 * i)
    assert np.array_equal(q.qarl_codes_to_canonical(qw).cpu().numpy().view(np.uint32).reshape(want.shape), want), (E, N, K, std)
    rows = int(rng.integers(1, 300))
    x = synth.normal_bf16((rows, K), std, seed=48200 + case)
    c, s = oracle.quantize_fp8_rows(np_bits(x))
    gc, gs = q.qarl_quantize_rows_fp8(x.cuda())
    assert np.array_equal(gs.cpu().numpy(), s) and np.array_equal(gc.cpu().numpy(), c), (rows, K, std)

    T, Er, topk = int(rng.integers(1, 3000)), int(rng.choice([64, 128, 192, 256])), int(rng.integers(1, 17))
    lg = synth.router_logits(T, Er, seed=48300 + case, zipf_s=float(rng.choice([0.0, 1.1, 1.5])))
    ids, wts = oracle.route(np_bits(lg), topk)
    counts, offsets, pairs = oracle.group(ids, Er)
    r = q.qarl_moe_route(lg.cuda(), topk)
    what = (T, Er, topk)
    assert np.array_equal(r.ids.cpu().numpy(), ids) and np.array_equal(r.counts.cpu().numpy(), counts), what
    assert np.array_equal(r.offsets.cpu().numpy(), offsets) and np.array_equal(r.pairs.cpu().numpy(), pairs), what
    assert np.array_equal(r.tokens.cpu().numpy(), pairs // topk), what
    assert np.allclose(r.w.cpu().numpy().astype(np.float64), wts, rtol=1e-6, atol=0), what

    Tl, H, V = int(rng.integers(1, 400)), 64 * int(rng.integers(1, 9)), int(rng.integers(1, 3000))
    inv_t = float(rng.choice([1.0, 0.5, 3.0]))
    h = synth.normal_bf16((Tl, H), 1.0, seed=48400 + case)
    wl = synth.normal_bf16((V, H), 0.3, seed=48500 + case)
    tg = synth.targets(Tl, V, seed=48600 + case)
    ref = oracle.token_logprob(np_bits(h), np_bits(wl), tg.numpy(), inv_t)
    got = q.qarl_token_logprob(h.cuda(), wl.cuda(), tg.cuda(), inv_t)["logprob"]
    assert np.abs(got.cpu().numpy().astype(np.float64) - ref).max() <= 1e-4 * max(1.0, np.abs(ref).max() / 10), (Tl, H, V, inv_t)
    assert torch.equal(got, q.qarl_token_logprob(h.cuda(), wl.cuda(), tg.cuda(), inv_t)["logprob"]), (Tl, H, V, inv_t)

    Eb, Nb, Kb = int(rng.integers(1, 5)), 128 * int(rng.integers(1, 5)), 128 * int(rng.integers(1, 9))
    rws = (rng.integers(0, 200, size=Eb) * (rng.random(Eb) < 0.75)).astype(np.int64)
    if rws.sum() == 0:
        rws[0] = 5
    M = int(rws.sum())
    wq = synth.normal_bf16((Eb, Nb, Kb), 0.02, seed=48700 + case)
    dy = synth.normal_bf16((M, Nb), 1.0, seed=48800 + case)
    xb = synth.normal_bf16((M + 3, Kb), 1.0, seed=48900 + case)
    off = np.concatenate([[0], np.cumsum(rws)]).astype(np.int32)
    rm = rng.permutation(M + 3)[:M].astype(np.int32)
    codes, scales = oracle.quantize_int4(np_bits(wq))
    qwb = q.qarl_quantize_weights(wq.cuda())
    what = (Eb, Nb, Kb, rws.tolist())
    dx = q.qarl_qgemm_grouped_dx(qwb, dy.cuda(), _i32(off), M, out_dtype=q.QARL_OUT_F32)
    dw = q.qarl_grouped_dw(dy.cuda(), xb.cuda(), _i32(off), Eb, row_map=_i32(rm), out_dtype=q.QARL_OUT_F32)
    assert norm_err(dx.cpu().numpy(), oracle.qgemm_w4a16_dx(np_bits(dy), codes, scales, off)) <= 1e-2, what
    assert norm_err(dw.cpu().numpy(), oracle.grouped_dw(np_bits(dy), np_bits(xb), off, Eb, rm)) <= TOL["w4a16"], what
    assert torch.equal(dx, q.qarl_qgemm_grouped_dx(qwb, dy.cuda(), _i32(off), M, out_dtype=q.QARL_OUT_F32)), what
    assert torch.equal(dw, q.qarl_grouped_dw(dy.cuda(), xb.cuda(), _i32(off), Eb, row_map=_i32(rm), out_dtype=q.QARL_OUT_F32)), what
