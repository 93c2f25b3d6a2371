"""GPU parity of the 4-bit-weight x 8-bit-activation formats against the oracle: FP4 (e2m1, alpha = 6) weights and
int4 g128 weights (W4A8), both under per-token e4m3 activations; quantizer bit-exact, GEMM in both kernel paths."""
import numpy as np
import pytest
import torch

from paper_2604_07853_amd import synth
from gpu_util import np_bits, norm_err, norm_err_bf16, flip_fraction, unblock_int4

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-3
TOL_F32 = 2e-5        # int4 weights: every product exact in fp32, accumulation-order noise only
TOL_F32_FP8 = 1e-3    # e4m3 x e4m3 products inside the matrix core (see test_gpu_qgemm)
MAX_FLIPS = 0.02
MAX_FLIPS_FP8 = 0.06


@pytest.fixture(scope="module")
def q():
    from paper_2604_07853_amd import binding
    binding.lib()
    return binding


def _i32(a):
    return torch.tensor(np.asarray(a), dtype=torch.int32, device="cuda")


def unpack_e2m1(words):
    """Packed FP4 codes as the library stores them (byte b of a word: element b in the low nibble, element 4 + b in
    the high nibble) -> one code per byte in element order.  Pure index permutation."""
    w = np.ascontiguousarray(words.detach().cpu().numpy()).view(np.uint32)
    out = np.empty(w.shape + (8,), dtype=np.uint8)
    for e in range(8):
        out[..., e] = (w >> np.uint32(4 * ((e & 3) * 2 + (e >> 2)))) & np.uint32(15)
    return out.reshape(w.shape[:-1] + (w.shape[-1] * 8,))


def test_fp4_quantizer_bit_exact(q, oracle):
    E, N, K = 3, 64, 768
    w = synth.normal_bf16((E, N, K), 0.02, seed=51)
    wb = np_bits(w).copy()
    wb[0, 3, :] = 0                                                      # a zero row
    wb[1, 5, :7] = 0x8000                                                # negative zeros
    # a row whose scale is exactly 2^-6 (absmax 6 * 2^-6) with elements on every rounding boundary, both signs
    mids = np.array([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0, 6.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 0.125, 0.3125])
    row = np.concatenate([mids, -mids, np.zeros(K - 32)]) * 2.0 ** -6
    wb[2, 7, :] = np_bits(torch.tensor(row, dtype=torch.float32).to(torch.bfloat16))
    w = torch.from_numpy(wb.view(np.int16)).view(torch.bfloat16)
    codes_ref, s_ref = oracle.quantize_fp4_rows(wb)
    qw = q.qarl_quantize_weights(w.cuda(), q.QARL_FP4_E2M1_CH)
    assert np.array_equal(qw.scales.cpu().numpy(), s_ref)
    got = unpack_e2m1(qw.codes)
    assert np.array_equal(got, codes_ref)
    assert s_ref[2, 7] == 2.0 ** -6 and list(codes_ref[2, 7, :8]) == [0, 2, 2, 4, 4, 6, 6, 7]   # ties went to even


_GEMM_SHAPES = [(3, 96, 256, (37, 0, 5)), (2, 288, 512, (300, 129)), (1, 32, 256, (1,)),
                (2, 96, 128, (40, 3)),          # a single 128-k stage
                (2, 544, 384, (130, 260))]      # three stages, three column blocks, ragged token tiles


# (the int4 decode kernel takes K % 256 == 0: W4A8 runs the shapes that both paths accept)
@pytest.mark.parametrize("fmt,E,N,K,rows", [(f,) + sh for f in ("fp4", "w4a8") for sh in _GEMM_SHAPES
                                            if f == "fp4" or sh[2] % 256 == 0])
def test_gemm_both_paths(q, oracle, fmt, E, N, K, rows):
    seed = 2100 + N + K
    w = synth.normal_bf16((E, N, K), 0.02, seed=seed)
    M = int(sum(rows))
    x = synth.normal_bf16((M, K), 1.0, seed=seed + 1)
    off = np.concatenate([[0], np.cumsum(rows)]).astype(np.int32)
    rm = np.random.default_rng(seed).permutation(M).astype(np.int32)
    xq_ref, sx_ref = oracle.quantize_fp8_rows(np_bits(x))
    xq, sx = q.qarl_quantize_rows_fp8(x.cuda())
    if fmt == "fp4":
        wq, sw = oracle.quantize_fp4_rows(np_bits(w))
        ref = oracle.qgemm_fp4w(xq_ref, sx_ref, wq, sw, off, rm)
        qw, tol = q.qarl_quantize_weights(w.cuda(), q.QARL_FP4_E2M1_CH), TOL_F32_FP8
    else:
        c4, s4 = oracle.quantize_int4(np_bits(w))
        ref = oracle.qgemm_w4a8(xq_ref, sx_ref, c4, s4, off, rm)
        qw, tol = q.qarl_quantize_weights(w.cuda(), q.QARL_W4A8_G128), TOL_F32
        assert np.array_equal(unblock_int4(qw.codes, E, N, K), c4)       # the W4A16 quantizer's codes
    for path in (q.QARL_PATH_DECODE, q.QARL_PATH_PREFILL):
        y = q.qarl_qgemm_grouped(qw, xq, _i32(off), M, row_map=_i32(rm), x_scales=sx, out_dtype=q.QARL_OUT_F32, path=path)
        e = norm_err(y.cpu().numpy(), ref)
        assert e <= tol, (fmt, path, e)


# Experts with several token tiles each on the tiled path: ragged last tiles, empty experts, one / three (odd) / eight
# 128-k stages, a last column block that is not full, and all three epilogues on the same product.
_TALL_SHAPES = [(2, 544, 384, (517, 390)), (1, 96, 128, (400,)), (3, 288, 1024, (0, 1300, 0)), (2, 64, 256, (256, 512))]


def _quantized(q, oracle, fmt, w):
    if fmt == "fp4":
        wq, sw = oracle.quantize_fp4_rows(np_bits(w))
        return wq, sw, oracle.qgemm_fp4w, q.qarl_quantize_weights(w.cuda(), q.QARL_FP4_E2M1_CH)
    wq, sw = oracle.quantize_fp8_rows(np_bits(w))
    return wq, sw, oracle.qgemm_fp8, q.qarl_quantize_weights(w.cuda(), q.QARL_FP8_E4M3_CH)


@pytest.mark.parametrize("fmt,E,N,K,rows", [(f,) + sh for f in ("fp8", "fp4") for sh in _TALL_SHAPES])
def test_tiled_path_several_tiles_per_expert(q, oracle, fmt, E, N, K, rows):
    seed = 2500 + N + K
    w = synth.normal_bf16((E, N, K), 0.02, seed=seed)
    M = int(sum(rows))
    x = synth.normal_bf16((M, K), 1.0, seed=seed + 1)
    off = np.concatenate([[0], np.cumsum(rows)]).astype(np.int32)
    rm = np.random.default_rng(seed).permutation(M).astype(np.int32)
    xq_ref, sx_ref = oracle.quantize_fp8_rows(np_bits(x))
    xq, sx = q.qarl_quantize_rows_fp8(x.cuda())
    wq, sw, gemm, qw = _quantized(q, oracle, fmt, w)
    ref = gemm(xq_ref, sx_ref, wq, sw, off, rm)
    y = q.qarl_qgemm_grouped(qw, xq, _i32(off), M, row_map=_i32(rm), x_scales=sx, out_dtype=q.QARL_OUT_F32,
                             path=q.QARL_PATH_PREFILL)
    assert norm_err(y.cpu().numpy(), ref) <= TOL_F32_FP8
    yb = q.qarl_qgemm_grouped(qw, xq, _i32(off), M, row_map=_i32(rm), x_scales=sx, path=q.QARL_PATH_PREFILL)
    assert np.array_equal(np_bits(yb), np_bits(y.to(torch.bfloat16)))        # the 16-bit output is the rounded fp32 one
    # gate rows then up rows: the SiLU-gated epilogue on the same product
    a = q.qarl_qgemm_grouped(qw, xq, _i32(off), M, row_map=_i32(rm), x_scales=sx, epilogue=q.QARL_EPI_SILU_MUL,
                             path=q.QARL_PATH_PREFILL)
    a_bits, a_ref = oracle.silu_mul(ref)
    assert norm_err_bf16(a.float().cpu().numpy(), a_ref) <= TOL_BF16
    assert flip_fraction(np_bits(a), a_bits) <= MAX_FLIPS_FP8


@pytest.mark.parametrize("fmt", ["fp8", "fp4"])
def test_one_hot_probe_four_token_tiles(q, oracle, fmt):
    """512 one-hot rows (448 e_k, scale 1) of one expert, 320 weight rows: the tiled kernel returns 448 times the
    dequantized weight bit for bit, i.e. every k of every stage meets its own weight element in every wavefront's tiles
    of every token tile and column block."""
    K, N = 512, 320
    w = synth.normal_bf16((1, N, K), 0.02, seed=63)
    x = (torch.eye(K) * 448).to(torch.bfloat16).cuda()
    xq, sx = q.qarl_quantize_rows_fp8(x)
    wq, sw, _, qw = _quantized(q, oracle, fmt, w)
    dec = oracle.e2m1_decode(wq[0]) if fmt == "fp4" else oracle.e4m3_decode(wq[0])
    want = (dec * 448.0 * sw[0][:, None].astype(np.float64)).T
    y = q.qarl_qgemm_grouped(qw, xq, _i32([0, K]), K, x_scales=sx, out_dtype=q.QARL_OUT_F32, path=q.QARL_PATH_PREFILL)
    assert np.array_equal(y.cpu().numpy().astype(np.float64), want.astype(np.float32).astype(np.float64))


@pytest.mark.parametrize("fmt", ["fp4", "w4a8"])
def test_one_hot_probe_bit_exact(q, oracle, fmt):
    """x rows = 448 e_k with scale 1: the output is 448 times the dequantized weight, no accumulation, both paths."""
    K, N = 256, 64
    w = synth.normal_bf16((1, N, K), 0.02, seed=61)
    x = (torch.eye(K) * 448).to(torch.bfloat16).cuda()
    xq, sx = q.qarl_quantize_rows_fp8(x)
    assert bool((sx == 1.0).all())
    if fmt == "fp4":
        wq, sw = oracle.quantize_fp4_rows(np_bits(w))
        want = (oracle.e2m1_decode(wq[0]) * 448.0 * sw[0][:, None].astype(np.float64)).T
        qw = q.qarl_quantize_weights(w.cuda(), q.QARL_FP4_E2M1_CH)
    else:
        c4, s4 = oracle.quantize_int4(np_bits(w))
        want = 448.0 * oracle.dequant_int4(c4, s4)[0].astype(np.float64).T
        qw = q.qarl_quantize_weights(w.cuda(), q.QARL_W4A8_G128)
    for path in (q.QARL_PATH_DECODE, q.QARL_PATH_PREFILL):
        y = q.qarl_qgemm_grouped(qw, xq, _i32([0, K]), K, x_scales=sx, out_dtype=q.QARL_OUT_F32, path=path)
        assert np.array_equal(y.cpu().numpy().astype(np.float64), want.astype(np.float32).astype(np.float64)), (fmt, path)


@pytest.mark.parametrize("path", [1, 2])
@pytest.mark.parametrize("fmt", ["fp4", "w4a8"])
def test_moe_layer_stage_wise(q, oracle, fmt, path):
    """Scaled-down MoE layer (E = 64, H = 512, I = 256, 301 tokens, Zipf router): every stage against the oracle on
    the GPU's own input to that stage, as for the FP8 format."""
    E, H, I, T, topk = 64, 512, 256, 301, 4
    gu, dn = synth.expert_weights(E, H, I, 2300)
    x = synth.normal_bf16((T, H), 1.0, 2302)
    lg = synth.router_logits(T, E, 2303, zipf_s=1.1)
    r = q.qarl_moe_route(lg.cuda(), topk)
    ids, w = oracle.route(np_bits(lg), topk)
    counts, offsets, pairs = oracle.group(ids, E)
    M = T * topk
    tok = (pairs // topk).astype(np.int32)
    if fmt == "fp4":
        (guq, gus), (dnq, dns) = oracle.quantize_fp4_rows(np_bits(gu)), oracle.quantize_fp4_rows(np_bits(dn))
        gid, gemm, tol, flips = q.QARL_FP4_E2M1_CH, oracle.qgemm_fp4w, TOL_F32_FP8, MAX_FLIPS_FP8
    else:
        (guq, gus), (dnq, dns) = oracle.quantize_int4(np_bits(gu)), oracle.quantize_int4(np_bits(dn))
        gid, gemm, tol, flips = q.QARL_W4A8_G128, oracle.qgemm_w4a8, TOL_F32, MAX_FLIPS
    qgu, qdn = q.qarl_quantize_weights(gu.cuda(), gid), q.qarl_quantize_weights(dn.cuda(), gid)
    xq, sx = q.qarl_quantize_rows_fp8(x.cuda())
    xq_ref, sx_ref = oracle.quantize_fp8_rows(np_bits(x))
    a_gpu = q.qarl_qgemm_grouped(qgu, xq, r.offsets, M, row_map=r.tokens, x_scales=sx, epilogue=q.QARL_EPI_SILU_MUL,
                                 path=path)
    a_ref_bits, a_ref = oracle.silu_mul(gemm(xq_ref, sx_ref, guq, gus, offsets, tok))
    assert norm_err_bf16(a_gpu.float().cpu().numpy(), a_ref) <= TOL_BF16
    assert flip_fraction(np_bits(a_gpu), a_ref_bits) <= flips
    aq, sa = q.qarl_quantize_rows_fp8(a_gpu)
    aq_ref, sa_ref = oracle.quantize_fp8_rows(np_bits(a_gpu))
    assert np.array_equal(aq.cpu().numpy(), aq_ref) and np.array_equal(sa.cpu().numpy(), sa_ref)
    y_gpu = q.qarl_qgemm_grouped(qdn, aq, r.offsets, M, x_scales=sa, out_dtype=q.QARL_OUT_F32, path=path)
    y_ref = gemm(aq_ref, sa_ref, dnq, dns, offsets)
    assert norm_err(y_gpu.cpu().numpy(), y_ref) <= tol
    out_gpu = q.qarl_qgemm_grouped(qdn, aq, r.offsets, M, x_scales=sa, epilogue=q.QARL_EPI_COMBINE, combine_w=r.w,
                                   sorted_pairs=r.pairs, T=T, topk=topk, path=path)
    out_ref, _ = oracle.combine(y_ref, pairs, w, T, topk)
    assert norm_err_bf16(out_gpu.float().cpu().numpy(), out_ref) <= TOL_BF16
    layer = q.MoELayer(qgu, qdn, T, topk, path)
    out2 = layer.forward(x.cuda(), lg.cuda())
    assert np.array_equal(np_bits(out2), np_bits(out_gpu))


def test_codes_to_canonical_equals_the_oracles_packing(q, oracle):
    """qarl_codes_to_canonical undoes the library's blocked / bit-permuted packings on the device: its output is the
    oracle's own row-major words (int4: q + 8 in nibble i; e2m1: the code in nibble i; e4m3: the bytes)."""
    E, N, K = 3, 96, 512
    w = synth.normal_bf16((E, N, K), 0.02, seed=71)
    c4, _ = oracle.quantize_int4(np_bits(w))
    for fmt in (q.QARL_W4A16_G128, q.QARL_W4A8_G128):
        qw = q.qarl_quantize_weights(w.cuda(), fmt)
        got = q.qarl_codes_to_canonical(qw).cpu().numpy().view(np.uint32)
        assert np.array_equal(got, c4)
        assert q.lib().qarl_codes_bytes(fmt, E, N, K) == c4.nbytes and q.lib().qarl_scales_bytes(fmt, E, N, K) == E * N * (K // 128) * 2
    f4, _ = oracle.quantize_fp4_rows(np_bits(w))                          # one code per byte
    want = np.zeros((E, N, K // 8), dtype=np.uint32)
    for i in range(8):
        want |= f4.reshape(E, N, K // 8, 8)[..., i].astype(np.uint32) << np.uint32(4 * i)
    q4 = q.qarl_quantize_weights(w.cuda(), q.QARL_FP4_E2M1_CH)
    assert np.array_equal(q.qarl_codes_to_canonical(q4).cpu().numpy().view(np.uint32), want)
    f8, _ = oracle.quantize_fp8_rows(np_bits(w))
    q8 = q.qarl_quantize_weights(w.cuda(), q.QARL_FP8_E4M3_CH)
    assert np.array_equal(q.qarl_codes_to_canonical(q8).cpu().numpy(), f8)
    assert q.lib().qarl_codes_bytes(q.QARL_FP8_E4M3_CH, E, N, K) == E * N * K
    assert q.lib().qarl_codes_bytes(99, E, N, K) == 0
