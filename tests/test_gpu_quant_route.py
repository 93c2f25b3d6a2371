"""GPU parity: quantizers and router must match the oracle bit for bit (codes, scales, ids,
counts, offsets, sorted pairs); router weights within 1e-6 relative."""
import numpy as np
import pytest
import torch

from paper_2604_07853_amd import synth
from gpu_util import np_bits, unblock_int4

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def q():
    from paper_2604_07853_amd import binding
    binding.lib()
    return binding


def _planted(w):
    """Add exact ties, a zero group, a constant group and extreme magnitudes to a weight tensor."""
    wb = np_bits(w).copy()
    one = np_bits(torch.tensor([2.0 ** -6]).to(torch.bfloat16))[0]
    flat = wb.reshape(-1, wb.shape[-1])
    vals = torch.tensor([7.0, 2.5, 3.5, -2.5, -3.5, 0.5, 1.5, -0.5, 6.5, -6.5, 4.5, 5.5]) * 2.0 ** -6
    flat[0, :128] = 0
    flat[0, :12] = np_bits(vals.to(torch.bfloat16))
    flat[1, 128:256] = 0                                   # zero group
    flat[2, :128] = one                                    # constant group
    flat[3, :128] = np_bits((torch.randn(128) * 1e30).to(torch.bfloat16))
    flat[4, :128] = np_bits((torch.randn(128) * 1e-30).to(torch.bfloat16))
    return synth.from_bits(wb)


@pytest.mark.parametrize("shape,seed", [((1, 768, 2048), 0), ((3, 64, 768), 1), ((2, 32, 128), 2)])
def test_quantize_int4_bit_exact(q, oracle, shape, seed):
    w = _planted(synth.normal_bf16(shape, 0.02, seed))
    codes, scales = oracle.quantize_int4(np_bits(w))
    qw = q.qarl_quantize_weights(w.cuda(), q.QARL_W4A16_G128)
    torch.cuda.synchronize()
    assert np.array_equal(qw.scales.cpu().view(torch.int16).numpy().view(np.uint16), scales)
    assert np.array_equal(unblock_int4(qw.codes, *shape), codes)


@pytest.mark.parametrize("shape,seed", [((2, 64, 2048), 3), ((1, 32, 768), 4), ((1, 32, 128), 5),
                                        ((1, 32, 4096), 6),      # the longest row the kernel keeps in registers
                                        ((1, 32, 4224), 7), ((1, 32, 8192), 8)])   # longer rows: read twice
def test_quantize_fp8_bit_exact(q, oracle, shape, seed):
    w = _planted(synth.normal_bf16(shape, 0.02, seed))
    wb = np_bits(w).copy()
    wb.reshape(-1, shape[-1])[5, :] = 0                    # zero row
    w = synth.from_bits(wb)
    codes, scales = oracle.quantize_fp8_rows(wb)
    qw = q.qarl_quantize_weights(w.cuda(), q.QARL_FP8_E4M3_CH)
    torch.cuda.synchronize()
    assert np.array_equal(qw.scales.cpu().numpy(), scales)
    assert np.array_equal(qw.codes.cpu().numpy(), codes)
    # activation entry point: same arithmetic on [rows, K]
    x = synth.normal_bf16((37, 768), 1.0, seed + 10)
    c2, s2 = oracle.quantize_fp8_rows(np_bits(x))
    gc, gs = q.qarl_quantize_rows_fp8(x.cuda())
    assert np.array_equal(gs.cpu().numpy(), s2) and np.array_equal(gc.cpu().numpy(), c2)


def test_fp8_cast_all_magnitudes(q, oracle):
    """Sweep the cast over every binade e4m3 covers, including subnormals and saturation."""
    g = torch.Generator().manual_seed(6)
    x = torch.randn(64, 1024, generator=g) * torch.logspace(-5, 0, 1024)
    x[:, 0] = 1.0                                          # row absmax ~ O(1): quotient spans 448 * 1e-5 .. 448
    xb = x.to(torch.bfloat16)
    c2, s2 = oracle.quantize_fp8_rows(np_bits(xb))
    gc, gs = q.qarl_quantize_rows_fp8(xb.cuda())
    assert np.array_equal(gs.cpu().numpy(), s2) and np.array_equal(gc.cpu().numpy(), c2)
    assert (c2 & 0x78 == 0).sum() > 100                    # subnormal codes were exercised


def test_fp8_rows_signed_zero_ties_and_random_patterns(q, oracle):
    """The row quantizer divides by a reciprocal with an exact correction and converts with the hardware
    instruction: rows of arbitrary bf16 bit patterns (every exponent the row's scale lets through, +-0,
    subnormal bf16 inputs), exact ties between neighbouring e4m3 values and both signs of zero must give
    the oracle's bytes (IEEE divide, then round to nearest even)."""
    rng = np.random.default_rng(11)
    K = 1024
    rows = []
    for r in range(96):
        top = rng.integers(100, 150)                                  # exponent field of the row's absmax
        ex = rng.integers(max(1, top - 40), top + 1, size=K)          # spread over 40 binades below it
        bits = (rng.integers(0, 2, size=K) << 15) | (ex << 7) | rng.integers(0, 128, size=K)
        bits[rng.integers(0, K, size=8)] = 0x0000                     # +0
        bits[rng.integers(0, K, size=8)] = 0x8000                     # -0
        bits[rng.integers(0, K, size=4)] = rng.integers(1, 128, size=4)            # subnormal bf16 inputs
        bits[0] = (top << 7) | rng.integers(0, 128)                   # the row's absmax
        rows.append(bits.astype(np.uint16))
    # rows whose scale is a power of two: every bf16 input with <= 5 significant bits lands on an e4m3 value or
    # exactly between two of them
    for r in range(32):
        m = rng.integers(0, 32, size=K) << 2                          # mantissa with 5 significant bits (incl. hidden one)
        ex = rng.integers(110, 128, size=K)
        bits = (rng.integers(0, 2, size=K) << 15) | (ex << 7) | m
        bits[0] = (127 << 7) | 0x60                                   # absmax 1.75 * 2^0 = 448 * 2^-8
        rows.append(bits.astype(np.uint16))
    xb = np.stack(rows)
    c_ref, s_ref = oracle.quantize_fp8_rows(xb)
    gc, gs = q.qarl_quantize_rows_fp8(synth.from_bits(xb).cuda())
    assert np.array_equal(gs.cpu().numpy(), s_ref)
    assert np.array_equal(gc.cpu().numpy(), c_ref)
    assert ((c_ref == 0x80).sum() > 100) and ((c_ref == 0x00).sum() > 100)     # both zeros occurred


@pytest.mark.parametrize("T,E,topk,zipf", [(300, 128, 8, 0.0), (1000, 128, 8, 1.1), (64, 64, 2, 0.0),
                                           (33, 256, 8, 0.0), (1, 128, 8, 0.0), (257, 128, 1, 0.0)])
def test_route_exact(q, oracle, T, E, topk, zipf):
    lg = synth.router_logits(T, E, seed=T + E, zipf_s=zipf)
    lb = np_bits(lg).copy()
    if T >= 64:
        lb[5, :] = lb[5, 0]                                # a token whose logits all tie
        lb[6, :] = 0x8000                                  # all -0
        lb[6, ::2] = 0x0000                                # mixed +0 / -0 compare equal
    lg = synth.from_bits(lb)
    ids, w = oracle.route(lb, topk)
    counts, offsets, pairs = oracle.group(ids, E)
    r = q.qarl_moe_route(lg.cuda(), topk)
    torch.cuda.synchronize()
    assert np.array_equal(r.ids.cpu().numpy(), ids)
    assert np.array_equal(r.counts.cpu().numpy(), counts)
    assert np.array_equal(r.offsets.cpu().numpy(), offsets)
    assert np.array_equal(r.pairs.cpu().numpy(), pairs)
    assert np.array_equal(r.tokens.cpu().numpy(), pairs // topk)
    gw = r.w.cpu().numpy().astype(np.float64)
    assert np.allclose(gw, w, rtol=1e-6, atol=0)
    assert np.allclose(gw.sum(axis=1), 1.0, atol=1e-6)


@pytest.mark.parametrize("T,E,topk", [(701, 64, 3), (5000, 128, 8), (4099, 256, 5)])
def test_grouping_large_batches_any_alignment(q, oracle, T, E, topk):
    """The large-batch grouping (one workgroup per expert, a contiguous range of pairs per wavefront): pair counts
    that leave ragged tails in the last wavefront's range and in the last 4-pair load, experts without tokens
    (Zipf), and an ids buffer that is not 16-byte aligned (the scalar-load path)."""
    lg = synth.router_logits(T, E, seed=3 * T + E, zipf_s=1.3)
    ids, w = oracle.route(np_bits(lg), topk)
    counts, offsets, pairs = oracle.group(ids, E)
    for shift in (0, 1):
        r = q.Routing(T, E, topk, "cuda")
        store = torch.empty((T * topk + 4,), dtype=torch.int32, device="cuda")
        r.ids = store[shift:shift + T * topk].view(T, topk)           # shift = 1: 4 bytes off a 16-byte boundary
        assert (r.ids.data_ptr() % 16 == 0) == (shift == 0)
        q.qarl_moe_route(lg.cuda(), topk, out=r)
        torch.cuda.synchronize()
        assert np.array_equal(r.ids.cpu().numpy(), ids)
        assert np.array_equal(r.counts.cpu().numpy(), counts)
        assert np.array_equal(r.offsets.cpu().numpy(), offsets)
        assert np.array_equal(r.pairs.cpu().numpy(), pairs)
        assert np.array_equal(r.tokens.cpu().numpy(), pairs // topk)


def test_route_empty_and_errors(q):
    lg = torch.empty((0, 128), dtype=torch.bfloat16, device="cuda")
    r = q.qarl_moe_route(lg, 8)
    torch.cuda.synchronize()
    assert int(r.counts.sum()) == 0 and int(r.offsets.abs().sum()) == 0
    with pytest.raises(q.QarlError) as ei:
        q.qarl_moe_route(torch.zeros((4, 100), dtype=torch.bfloat16, device="cuda"), 8)
    assert ei.value.status == q.QARL_ERR_UNSUPPORTED
    with pytest.raises(q.QarlError):
        q.qarl_quantize_weights(torch.zeros((1, 32, 100), dtype=torch.bfloat16, device="cuda"))
