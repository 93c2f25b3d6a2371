"""GPU parity of the grouped quantized GEMM against the oracle: bit-exact where the result
does not depend on summation order (one-hot probe, exact-integer regime), within the stated
tolerance on general data; both kernel paths on the same codes and scales."""
import numpy as np
import pytest
import torch

from paper_2604_07853_amd import synth
from gpu_util import np_bits, norm_err, norm_err_bf16, flip_fraction

pytestmark = pytest.mark.gpu

# Tolerance for bf16 outputs (2e-3, the stated bar): max (|d| - half_ulp_bf16(ref))+ / (|ref| + rms(ref)),
# i.e. the error of the value before it is rounded to the 8-bit-significand output format; a bf16
# rounding alone is up to 2^-8 = 3.9e-3 relative, so it is discounted and checked separately through
# the fraction of outputs whose bits differ from the oracle's own bf16 rounding.
TOL_BF16 = 2e-3
TOL_F32 = 2e-5       # fp32 outputs: accumulation-order noise only
MAX_FLIPS = 0.02     # bf16 outputs that may land on the neighbouring value
# e4m3 x e4m3 MFMA: products are exact, but inside one instruction the matrix core aligns them to the
# largest product's exponent and keeps about 15 bits below it, truncating (measured: next to a
# product of 448*448 = 2^17.6 a product of 14 arrives as 8, one below 8 as 0).  The result is an error
# of 4e-5..2e-4 of rms whatever K is, identical in both kernel paths, so fp32 outputs of the FP8
# format get a wider bar, still inside the 2e-3 one.
TOL_F32_FP8 = 1e-3
MAX_FLIPS_FP8 = 0.06
# FP8 layer end to end against the oracle's own chain: one moved e4m3 code of the intermediate changes one of I
# products by up to 2^-3 of its size, a moved row scale a few per cent of them; after the down projection and the
# combine that is a few 1e-3 of the output's rms on the rows it hits; a row whose largest element moved gets
# another scale and a few per cent new codes, which is worth up to 1e-1 of the rms on that token.
FP8_E2E_MAX = 5e-2
FP8_E2E_MAX_SCALE = 0.2   # tokens with a pair-row whose scale moved by one bf16 step of its largest element


@pytest.fixture(scope="module")
def q():
    from paper_2604_07853_amd import binding
    binding.lib()
    return binding


def _paths(q):
    return [q.QARL_PATH_DECODE, q.QARL_PATH_PREFILL]


def _i32(a):
    return torch.tensor(np.asarray(a), dtype=torch.int32, device="cuda")


def test_dense_w4a16_config1(q, oracle):
    """Config 1: x [16,2048] N(0,1), W [768,2048] N(0,0.02), W4A16 g128, fp32 out."""
    g = torch.Generator().manual_seed(0)                           # the config's seed 0: x first, then W, one stream
    x = torch.randn((16, 2048), generator=g).to(torch.bfloat16)
    w = (torch.randn((1, 768, 2048), generator=g) * 0.02).to(torch.bfloat16)
    codes, scales = oracle.quantize_int4(np_bits(w))
    off = np.array([0, 16], dtype=np.int32)
    ref = oracle.qgemm_w4a16(np_bits(x), codes, scales, off)
    qw = q.qarl_quantize_weights(w.cuda())
    for path in _paths(q):
        y = q.qarl_qgemm_grouped(qw, x.cuda(), _i32(off), 16, out_dtype=q.QARL_OUT_F32, path=path)
        e = norm_err(y.cpu().numpy(), ref)
        assert e <= TOL_F32, (path, e)
        yb = q.qarl_qgemm_grouped(qw, x.cuda(), _i32(off), 16, out_dtype=q.QARL_OUT_BF16, path=path)
        eb = norm_err_bf16(yb.float().cpu().numpy(), ref)
        assert eb <= TOL_BF16, (path, eb)
        fl = flip_fraction(np_bits(yb), oracle.bf16_from_f64(ref))
        assert fl <= MAX_FLIPS, (path, fl)


@pytest.mark.parametrize("K,N", [(256, 64), (768, 32), (4096, 32)])
def test_one_hot_probe_bit_exact_both_paths(q, oracle, K, N):
    """x = rows of the identity: the output is the dequantized weight s*q itself; both paths
    must reproduce it exactly (identical dequantized numerics)."""
    E = 2
    w = synth.normal_bf16((E, N, K), 0.02, seed=7)
    codes, scales = oracle.quantize_int4(np_bits(w))
    deq = oracle.dequant_int4(codes, scales)                       # [E, N, K] fp32
    eye = torch.eye(K).to(torch.bfloat16)
    x = torch.cat([eye, eye]).cuda()
    off = _i32([0, K, 2 * K])
    qw = q.qarl_quantize_weights(w.cuda())
    for path in _paths(q):
        y = q.qarl_qgemm_grouped(qw, x, off, 2 * K, out_dtype=q.QARL_OUT_F32, path=path).cpu().numpy()
        assert np.array_equal(y[:K], deq[0].T) and np.array_equal(y[K:], deq[1].T), path


def test_exact_integer_regime_bit_exact(q, oracle):
    rng = np.random.default_rng(7)
    E, N, K, M = 3, 64, 512, 75
    qi = rng.integers(-7, 8, size=(E, N, K))
    qi[:, :, ::128] = 7
    ex = rng.integers(-3, 2, size=(E, N, K // 128))
    w = torch.tensor(qi * np.repeat(2.0 ** ex, 128, axis=2), dtype=torch.float32).to(torch.bfloat16)
    x = torch.tensor(rng.integers(-4, 5, size=(M, K)), dtype=torch.float32).to(torch.bfloat16)
    off = np.array([0, 40, 40, 75], dtype=np.int32)                # expert 1 is empty
    rm = rng.permutation(M).astype(np.int32)
    codes, scales = oracle.quantize_int4(np_bits(w))
    ref = oracle.qgemm_w4a16(np_bits(x), codes, scales, off, rm)
    qw = q.qarl_quantize_weights(w.cuda())
    for path in _paths(q):
        y = q.qarl_qgemm_grouped(qw, x.cuda(), _i32(off), M, row_map=_i32(rm), out_dtype=q.QARL_OUT_F32, path=path)
        assert np.array_equal(y.cpu().numpy().astype(np.float64), ref), path


def _moe_case(q, oracle, E, H, I, T, topk, seed, zipf, path, fmt="int4"):
    gu, dn = synth.expert_weights(E, H, I, seed)
    x = synth.normal_bf16((T, H), 1.0, seed + 2)
    lg = synth.router_logits(T, E, seed + 3, zipf_s=zipf)
    r = q.qarl_moe_route(lg.cuda(), topk)
    ids, w = oracle.route(np_bits(lg), topk)
    counts, offsets, pairs = oracle.group(ids, E)
    assert np.array_equal(r.pairs.cpu().numpy(), pairs)
    M = T * topk
    tok = (pairs // topk).astype(np.int32)
    if fmt == "int4":
        guc, gus = oracle.quantize_int4(np_bits(gu))
        dnc, dns = oracle.quantize_int4(np_bits(dn))
        qgu = q.qarl_quantize_weights(gu.cuda())
        qdn = q.qarl_quantize_weights(dn.cuda())
        # stage 1: gate_up + SiLU*mul
        a_gpu = q.qarl_qgemm_grouped(qgu, x.cuda(), r.offsets, M, row_map=r.tokens, epilogue=q.QARL_EPI_SILU_MUL, path=path)
        gu_ref = oracle.qgemm_w4a16(np_bits(x), guc, gus, offsets, tok)
        a_ref_bits, a_ref = oracle.silu_mul(gu_ref)
        a_gpu_bits = np_bits(a_gpu)
        ea = norm_err_bf16(a_gpu.float().cpu().numpy(), a_ref)
        assert ea <= TOL_BF16, ea
        fl = flip_fraction(a_gpu_bits, a_ref_bits)
        assert fl <= MAX_FLIPS, fl
        # stage 2: down on the GPU's own a, Y in fp32 (NONE epilogue)
        y_gpu = q.qarl_qgemm_grouped(qdn, a_gpu, r.offsets, M, out_dtype=q.QARL_OUT_F32, path=path)
        y_ref = oracle.qgemm_w4a16(a_gpu_bits, dnc, dns, offsets)
        ey = norm_err(y_gpu.cpu().numpy(), y_ref)
        assert ey <= TOL_F32, ey
        # stage 3: down + combine, bf16 out, against the oracle on the GPU's a
        out_gpu = q.qarl_qgemm_grouped(qdn, a_gpu, r.offsets, M, epilogue=q.QARL_EPI_COMBINE, combine_w=r.w,
                                       sorted_pairs=r.pairs, T=T, topk=topk, path=path)
        out_ref, out_ref_bits = oracle.combine(y_ref, pairs, w, T, topk)
        eo = norm_err_bf16(out_gpu.float().cpu().numpy(), out_ref)
        assert eo <= TOL_BF16, eo
        fl = flip_fraction(np_bits(out_gpu), out_ref_bits)
        assert fl <= MAX_FLIPS, fl
        # end to end against the oracle's own chain
        full = oracle.moe_ffn_w4a16(np_bits(x), np_bits(lg), guc, gus, dnc, dns, topk)
        layer = q.MoELayer(qgu, qdn, T, topk, path)
        out2 = layer.forward(x.cuda(), lg.cuda())
        e2e = norm_err_bf16(out2.float().cpu().numpy(), full["out"])
        assert e2e <= TOL_BF16, e2e                                # includes the rare one-ulp flips of a
        assert np.array_equal(np_bits(out2), np_bits(out_gpu))     # same kernels, same result
    else:
        guq, gus = oracle.quantize_fp8_rows(np_bits(gu))
        dnq, dns = oracle.quantize_fp8_rows(np_bits(dn))
        qgu = q.qarl_quantize_weights(gu.cuda(), q.QARL_FP8_E4M3_CH)
        qdn = q.qarl_quantize_weights(dn.cuda(), q.QARL_FP8_E4M3_CH)
        xq, sx = q.qarl_quantize_rows_fp8(x.cuda())
        xq_ref, sx_ref = oracle.quantize_fp8_rows(np_bits(x))
        assert np.array_equal(xq.cpu().numpy(), xq_ref) and np.array_equal(sx.cpu().numpy(), sx_ref)
        a_gpu = q.qarl_qgemm_grouped(qgu, xq, r.offsets, M, row_map=r.tokens, x_scales=sx,
                                     epilogue=q.QARL_EPI_SILU_MUL, path=path)
        gu_ref = oracle.qgemm_fp8(xq_ref, sx_ref, guq, gus, offsets, tok)
        a_ref_bits, a_ref = oracle.silu_mul(gu_ref)
        ea = norm_err_bf16(a_gpu.float().cpu().numpy(), a_ref)
        assert ea <= TOL_BF16, ea
        fl = flip_fraction(np_bits(a_gpu), a_ref_bits)
        assert fl <= MAX_FLIPS_FP8, fl
        aq, sa = q.qarl_quantize_rows_fp8(a_gpu)
        aq_ref, sa_ref = oracle.quantize_fp8_rows(np_bits(a_gpu))   # oracle on the GPU's own a
        assert np.array_equal(aq.cpu().numpy(), aq_ref) and np.array_equal(sa.cpu().numpy(), sa_ref)
        y_gpu = q.qarl_qgemm_grouped(qdn, aq, r.offsets, M, x_scales=sa, out_dtype=q.QARL_OUT_F32, path=path)
        y_ref = oracle.qgemm_fp8(aq_ref, sa_ref, dnq, dns, offsets)
        ey = norm_err(y_gpu.cpu().numpy(), y_ref)
        assert ey <= TOL_F32_FP8, ey
        out_gpu = q.qarl_qgemm_grouped(qdn, aq, r.offsets, M, x_scales=sa, epilogue=q.QARL_EPI_COMBINE,
                                       combine_w=r.w, sorted_pairs=r.pairs, T=T, topk=topk, path=path)
        out_ref, _ = oracle.combine(y_ref, pairs, w, T, topk)
        eo = norm_err_bf16(out_gpu.float().cpu().numpy(), out_ref)
        assert eo <= TOL_BF16, eo
        layer = q.MoELayer(qgu, qdn, T, topk, path)
        out2 = layer.forward(x.cuda(), lg.cuda())
        assert np.array_equal(np_bits(out2), np_bits(out_gpu))
        # end to end against the oracle's own chain.  The activation quantizer of eq. (2) is discontinuous: an
        # intermediate that lands on the neighbouring bf16 value can move an e4m3 code by a whole step (2^-4
        # relative), and if it is the row's largest element the row's scale and a few per cent of its codes.  So
        # the stages above carry the parity bar; here the size of that effect is reported and bounded.
        full = oracle.moe_ffn_fp8(np_bits(x), np_bits(lg), guq, gus, dnq, dns, topk)
        a_rows = int((np_bits(a_gpu) != full["a"]).any(axis=1).sum())
        code_rows = int(((aq.cpu().numpy() != full["aq"]).any(axis=1) | (sa.cpu().numpy() != full["sa"])).sum())
        scale_rows = int((sa.cpu().numpy() != full["sa"]).sum())
        ref = full["out"]
        rms = np.sqrt((ref ** 2).mean())
        d = np.abs(out2.float().cpu().numpy().astype(np.float64) - ref) / (np.abs(ref) + rms)
        # tokens one of whose pair-rows got another row scale (their whole row of codes is requantized)
        tok_moved = np.zeros(T, dtype=bool)
        tok_moved[tok[sa.cpu().numpy() != full["sa"]]] = True
        e_same = float(d[~tok_moved].max()) if (~tok_moved).any() else 0.0
        e_moved = float(d[tok_moved].max()) if tok_moved.any() else 0.0
        e_9999, e_med = float(np.quantile(d, 0.9999)), float(np.median(d))
        print("fp8 end to end: T=%d path=%d max %.2e (tokens with a moved row scale: %.2e) p99.99 %.2e median %.2e; "
              "rows of a moved %d / %d, rows with codes or scale moved %d (scale %d)"
              % (T, path, e_same, e_moved, e_9999, e_med, a_rows, M, code_rows, scale_rows))
        assert e_med <= TOL_BF16 and e_same <= FP8_E2E_MAX and e_moved <= FP8_E2E_MAX_SCALE, (e_med, e_same, e_moved)
        assert scale_rows <= max(2, 0.02 * M), scale_rows


@pytest.mark.parametrize("path", [1, 2])
@pytest.mark.parametrize("T,zipf", [(40, 0.0), (301, 1.1)])
def test_moe_layer_small_w4a16(q, oracle, T, zipf, path):
    """Scaled-down layer (E=64, H=512, I=256): ragged expert loads, empty experts, several tiles."""
    _moe_case(q, oracle, 64, 512, 256, T, 4, seed=20 + T, zipf=zipf, path=path)


@pytest.mark.parametrize("path", [1, 2])
@pytest.mark.parametrize("T,zipf", [(40, 0.0), (301, 1.1)])
def test_moe_layer_small_fp8(q, oracle, T, zipf, path):
    _moe_case(q, oracle, 64, 512, 256, T, 4, seed=40 + T, zipf=zipf, path=path, fmt="fp8")


def test_fp8_one_hot_probe(q, oracle):
    """x rows = 448*e_k: s_x = 1 exactly, so the output is s_w * decode(w_q) with no accumulation."""
    K, N = 256, 64
    w = synth.normal_bf16((1, N, K), 0.02, seed=8)
    wq, sw = oracle.quantize_fp8_rows(np_bits(w))
    qw = q.qarl_quantize_weights(w.cuda(), q.QARL_FP8_E4M3_CH)
    x = (torch.eye(K) * 448).to(torch.bfloat16).cuda()
    xq, sx = q.qarl_quantize_rows_fp8(x)
    assert bool((sx == 1.0).all())
    want = (oracle.e4m3_decode(wq[0]) * 448.0 * sw[0][:, None].astype(np.float64)).T
    for path in _paths(q):
        y = q.qarl_qgemm_grouped(qw, xq, _i32([0, K]), K, x_scales=sx, out_dtype=q.QARL_OUT_F32, path=path)
        assert np.array_equal(y.cpu().numpy().astype(np.float64), want.astype(np.float32).astype(np.float64)), path


def _fp8_codes_of(oracle, values):
    return oracle.e4m3_encode(np.asarray(values, dtype=np.float64))


@pytest.mark.parametrize("K", [256, 512])
def test_fp8_matrix_core_truncation_bound(q, oracle, K):
    """One product of 448 * 448 beside many small ones in the same k-block.  Products of two e4m3 values are
    exact, but the matrix core sums the products of one instruction after aligning them to the largest product's
    exponent E and dropping what lies below 2^(E-14).  The oracle sums exactly; the difference must stay below the
    bound that this model gives per output, sum over the 64-k blocks of 63 * 2^(E_block - 14) (+ fp32
    accumulation), in both kernel paths, and must not vanish on this input (else the wider FP8 bar is not needed)."""
    rng = np.random.default_rng(11 + K)
    N, M = 64, 48
    xv = rng.integers(-7, 8, size=(M, K)).astype(np.float64)
    wv = rng.integers(-7, 8, size=(1, N, K)).astype(np.float64)
    xv[:, ::64] = 448.0                                   # first element of every 64-k block of every token row
    wv[0, :, ::64] = 448.0
    xv[M // 2:, 64:] = rng.integers(-7, 8, size=(M - M // 2, K - 64))   # lower half: the big product in block 0 only
    xq, wq = _fp8_codes_of(oracle, xv), _fp8_codes_of(oracle, wv)
    assert np.array_equal(oracle.e4m3_decode(xq), xv) and np.array_equal(oracle.e4m3_decode(wq), wv)
    sx, sw = np.ones(M, dtype=np.float32), np.ones((1, N), dtype=np.float32)
    off = np.array([0, M], dtype=np.int32)
    ref = oracle.qgemm_fp8(xq, sx, wq, sw, off)
    prod = np.abs(xv[:, None, :] * wv[0][None, :, :]).reshape(M, N, K // 64, 64)
    top = prod.max(axis=3)
    Eb = np.floor(np.log2(np.maximum(top, 1.0)))
    bound = (63.0 * 2.0 ** (Eb - 14)).sum(axis=2) + K * 2.0 ** -24 * prod.sum(axis=(2, 3))
    qw = q.QWeight(q.QARL_FP8_E4M3_CH, 1, N, K, torch.tensor(wq, device="cuda"), torch.tensor(sw, device="cuda"))
    for path in _paths(q):
        y = q.qarl_qgemm_grouped(qw, torch.tensor(xq, device="cuda"), _i32(off), M,
                                 x_scales=torch.tensor(sx, device="cuda"), out_dtype=q.QARL_OUT_F32, path=path)
        d = np.abs(y.cpu().numpy().astype(np.float64) - ref)
        print("fp8 truncation K=%d path=%d: max |d| %.1f (bound there %.1f), mean |d| %.2f, rel. to rms %.2e"
              % (K, path, d.max(), bound.flat[d.argmax()], d.mean(), d.max() / np.sqrt((ref ** 2).mean())))
        assert np.all(d <= bound), (path, float((d - bound).max()))
        assert d.max() > 0, path


def test_moe_decode_config2_full_size(q, oracle):
    """Config 2 at full size: 256 tokens, 128 experts, H 2048, I 768, top-8, W4A16, decode path."""
    _moe_case(q, oracle, synth.E, synth.H, synth.I, 256, synth.TOPK, seed=1, zipf=0.0, path=1)


def test_empty_and_error_paths(q):
    w = synth.normal_bf16((2, 32, 128), 0.02, seed=1).cuda()
    qw = q.qarl_quantize_weights(w)
    x = torch.zeros((4, 128), dtype=torch.bfloat16, device="cuda")
    off = _i32([0, 0, 0])
    y = q.qarl_qgemm_grouped(qw, x, off, 0, out_dtype=q.QARL_OUT_F32)          # M = 0: no-op
    assert y.shape == (0, 32)
    with pytest.raises(q.QarlError) as ei:                                      # COMBINE without workspace
        q.lib().qarl_qgemm_grouped
        q._check(q.lib().qarl_qgemm_grouped(q.C.byref(qw.desc), q._ptr(x), None, 4, None, q._ptr(off), 4,
                                            q.QARL_EPI_COMBINE, q._ptr(x), q._ptr(off), 1, 4, q._ptr(x), 0, 0,
                                            None, 0, None))
    assert ei.value.status == q.QARL_ERR_WORKSPACE
    with pytest.raises(q.QarlError) as ei:
        q.qarl_qgemm_grouped(qw, x, off, 4, epilogue=q.QARL_EPI_SILU_MUL, out_dtype=q.QARL_OUT_F32)
    assert ei.value.status == q.QARL_ERR_UNSUPPORTED


@pytest.mark.parametrize("fmt", ["int4", "fp8"])
@pytest.mark.parametrize("E,N,K,rows", [(3, 96, 128, (37, 0, 5)), (2, 288, 384, (300, 129)), (1, 32, 128, (1,)),
                                        (2, 544, 768, (64, 257))])
def test_ragged_shapes_both_paths(q, oracle, fmt, E, N, K, rows):
    """Shapes that leave partial column tiles (N not a multiple of the tile width), a single 128-k stage,
    empty experts, one-row experts and experts spanning several token tiles; plain epilogue, fp32 out."""
    seed = 700 + N + K
    w = synth.normal_bf16((E, N, K), 0.02, seed=seed)
    M = int(sum(rows))
    x = synth.normal_bf16((M, K), 1.0, seed=seed + 1)
    off = np.concatenate([[0], np.cumsum(rows)]).astype(np.int32)
    if fmt == "int4":
        codes, scales = oracle.quantize_int4(np_bits(w))
        ref = oracle.qgemm_w4a16(np_bits(x), codes, scales, off)
        qw = q.qarl_quantize_weights(w.cuda())
        xin, xs, tol = x.cuda(), None, TOL_F32
    else:
        wq, sw = oracle.quantize_fp8_rows(np_bits(w))
        xq_ref, sx_ref = oracle.quantize_fp8_rows(np_bits(x))
        ref = oracle.qgemm_fp8(xq_ref, sx_ref, wq, sw, off)
        qw = q.qarl_quantize_weights(w.cuda(), q.QARL_FP8_E4M3_CH)
        xin, xs = q.qarl_quantize_rows_fp8(x.cuda())
        tol = TOL_F32_FP8
    for path in _paths(q):
        try:
            y = q.qarl_qgemm_grouped(qw, xin, _i32(off), M, x_scales=xs, out_dtype=q.QARL_OUT_F32, path=path)
        except q.QarlError as err:      # the streaming path takes W4A16 only with K a multiple of 256
            assert path == q.QARL_PATH_DECODE and err.status == q.QARL_ERR_UNSUPPORTED and fmt == "int4" and K % 256
            continue
        e = norm_err(y.cpu().numpy(), ref)
        assert e <= tol, (path, e)


@pytest.mark.parametrize("E,N,K,T,topk", [(8, 64, 2048, 600, 3),     # row maps too large to sit beside the LDS tile
                                          (3, 96, 4096, 50, 2),      # K beyond 2048: 16-row LDS tile, several row blocks
                                          (4, 512, 2048, 60, 3),     # 64-row blocks over a K-chunked tile, one pair per wavefront
                                          (4, 1024, 2048, 200, 3),   # the same with two pairs and several row blocks
                                          (4, 64, 512, 37, 3),       # M = 111: last quad of the map is partial
                                          (16, 32, 256, 1500, 3),    # M = 4500: maps stay in global memory
                                          (6, 96, 768, 171, 5)])     # 64-row blocks (K fits), M = 855
def test_decode_row_map_paths(q, oracle, E, N, K, T, topk):
    """Decode path with the gather map (routed tokens) and the scatter map (pair order of the combine):
    every way the kernel fetches its row ids (copied to LDS next to the tile, into the tile region, or read
    from global memory), experts that need several row blocks and several passes, M not a multiple of 4."""
    seed = 900 + K + T
    w = synth.normal_bf16((E, N, K), 0.02, seed=seed)
    x = synth.normal_bf16((T, K), 1.0, seed=seed + 1)
    lg = synth.router_logits(T, E, seed + 2, zipf_s=1.1)
    ids, wts = oracle.route(np_bits(lg), topk)                     # the router kernel takes E % 64 == 0 only:
    counts, offsets, pairs = oracle.group(ids, E)                  # the oracle's routing is this test's input
    M = T * topk
    tok = (pairs // topk).astype(np.int32)
    d_off, d_tok, d_pairs = _i32(offsets), _i32(tok), _i32(pairs)
    d_w = torch.tensor(np.asarray(wts, dtype=np.float32), device="cuda")
    codes, scales = oracle.quantize_int4(np_bits(w))
    qw = q.qarl_quantize_weights(w.cuda())
    # gather only: rows of x picked through row_map, fp32 out in sorted order
    y_ref = oracle.qgemm_w4a16(np_bits(x), codes, scales, offsets, tok)
    y = q.qarl_qgemm_grouped(qw, x.cuda(), d_off, M, row_map=d_tok, out_dtype=q.QARL_OUT_F32,
                             path=q.QARL_PATH_DECODE)
    assert norm_err(y.cpu().numpy(), y_ref) <= TOL_F32
    # gather + scatter: the same product through the combine epilogue (out_row_map = sorted pairs)
    xg = x[torch.tensor(tok, dtype=torch.long)].contiguous()       # rows already in sorted order
    y2_ref = oracle.qgemm_w4a16(np_bits(xg), codes, scales, offsets)
    out_ref, out_ref_bits = oracle.combine(y2_ref, pairs, wts, T, topk)
    out = q.qarl_qgemm_grouped(qw, xg.cuda(), d_off, M, epilogue=q.QARL_EPI_COMBINE, combine_w=d_w,
                               sorted_pairs=d_pairs, T=T, topk=topk, path=q.QARL_PATH_DECODE)
    assert norm_err_bf16(out.float().cpu().numpy(), out_ref) <= TOL_BF16
    assert flip_fraction(np_bits(out), out_ref_bits) <= MAX_FLIPS


@pytest.mark.parametrize("E,N,K,T,topk", [(8, 64, 2048, 500, 3),      # several row blocks per expert, partial last quad of ids
                                          (4, 512, 2048, 60, 3),      # 64-row blocks over a K-chunked tile
                                          (4, 1024, 2048, 200, 3),    # ... two pairs per wavefront, several row blocks
                                          (4, 64, 512, 37, 3),        # 111 pairs
                                          (6, 96, 768, 171, 5),       # 64-row blocks
                                          (128, 64, 256, 512, 8)])    # the largest routed batch: 512 tokens, 4096 pairs
def test_routed_mode_equals_grouped_decode(q, oracle, E, N, K, T, topk):
    """qarl_qgemm_routed (every workgroup lists its expert's pairs from the router's ids) against the oracle and,
    bit for bit, against the grouped decode path fed with the grouping of the same ids: plain epilogue with x per
    token, SiLU*mul, and the combine on rows in pair order."""
    seed = 1300 + K + T
    w = synth.normal_bf16((E, N, K), 0.02, seed=seed)
    x = synth.normal_bf16((T, K), 1.0, seed=seed + 1)
    lg = synth.router_logits(T, E, seed + 2, zipf_s=1.1)
    ids, wts = oracle.route(np_bits(lg), topk)
    counts, offsets, pairs = oracle.group(ids, E)
    M = T * topk
    tok = (pairs // topk).astype(np.int32)
    d_ids = _i32(np.asarray(ids).reshape(-1))
    d_off, d_tok, d_pairs = _i32(offsets), _i32(tok), _i32(pairs)
    d_w = torch.tensor(np.asarray(wts, dtype=np.float32), device="cuda")
    codes, scales = oracle.quantize_int4(np_bits(w))
    qw = q.qarl_quantize_weights(w.cuda())
    inv = torch.tensor(pairs, dtype=torch.long, device="cuda")     # sorted position i holds pair pairs[i]
    # plain epilogue, activation row = token: row pr of the routed result is row i of the grouped one, pairs[i] = pr
    y_ref = oracle.qgemm_w4a16(np_bits(x), codes, scales, offsets, tok)
    y_grp = q.qarl_qgemm_grouped(qw, x.cuda(), d_off, M, row_map=d_tok, out_dtype=q.QARL_OUT_F32,
                                 path=q.QARL_PATH_DECODE)
    y_rt = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    q.qarl_qgemm_routed(qw, x.cuda(), d_ids, T, topk, True, out=y_rt, out_dtype=q.QARL_OUT_F32)
    assert norm_err(y_rt[inv].cpu().numpy(), y_ref) <= TOL_F32
    assert torch.equal(y_rt[inv], y_grp)
    # SiLU*mul
    a_grp = q.qarl_qgemm_grouped(qw, x.cuda(), d_off, M, row_map=d_tok, epilogue=q.QARL_EPI_SILU_MUL,
                                 path=q.QARL_PATH_DECODE)
    a_rt = q.qarl_qgemm_routed(qw, x.cuda(), d_ids, T, topk, True, epilogue=q.QARL_EPI_SILU_MUL)
    assert np.array_equal(np_bits(a_rt[inv]), np_bits(a_grp))
    # combine: activation row = pair id
    xp = x[torch.tensor(np.arange(M) // topk, dtype=torch.long)].contiguous()   # one row per pair, pair order
    xg = xp[torch.tensor(pairs, dtype=torch.long)].contiguous()                 # the same rows in sorted order
    out_grp = q.qarl_qgemm_grouped(qw, xg.cuda(), d_off, M, epilogue=q.QARL_EPI_COMBINE, combine_w=d_w,
                                   sorted_pairs=d_pairs, T=T, topk=topk, path=q.QARL_PATH_DECODE)
    out_rt = q.qarl_qgemm_routed(qw, xp.cuda(), d_ids, T, topk, False, epilogue=q.QARL_EPI_COMBINE, combine_w=d_w)
    y2_ref = oracle.qgemm_w4a16(np_bits(xg), codes, scales, offsets)
    out_ref, _ = oracle.combine(y2_ref, pairs, wts, T, topk)
    assert norm_err_bf16(out_rt.float().cpu().numpy(), out_ref) <= TOL_BF16
    assert np.array_equal(np_bits(out_rt), np_bits(out_grp))


_ROUTED_QX_SHAPES = [(8, 64, 2048, 500, 3),      # several row blocks per expert, partial last quad of ids
                     (4, 512, 2048, 60, 3),      # two token tiles per block
                     (4, 64, 512, 37, 3),        # 111 pairs
                     (6, 96, 768, 171, 5),       # ring depth 3; rows with 1.5 chunks per lane
                     (3, 64, 4096, 50, 2),       # eight chunks per lane and row
                     (128, 64, 256, 512, 8)]     # the largest routed batch: 512 tokens, 4096 pairs


# (the int4 decode kernel's routed mode takes K % 256 == 0 up to 2048: W4A8 runs the shapes it accepts)
@pytest.mark.parametrize("fmt_name,E,N,K,T,topk", [(f,) + sh for f in ("fp8", "fp4", "w4a8") for sh in _ROUTED_QX_SHAPES
                                                   if f != "w4a8" or (sh[2] % 256 == 0 and sh[2] <= 2048)])
def test_routed_mode_quantizes_its_rows_like_the_row_quantizer(q, oracle, fmt_name, E, N, K, T, topk):
    """qarl_qgemm_routed on the e4m3-activation formats takes 16-bit rows and quantizes what it gathers: bit for bit
    the row quantizer followed by the grouped decode path on the grouping of the same ids, and within tolerance of
    the oracle's quantizer + GEMM.  Plain epilogue with x per token, SiLU*mul, and the combine on rows in pair
    order."""
    fmt = {"fp8": q.QARL_FP8_E4M3_CH, "fp4": q.QARL_FP4_E2M1_CH, "w4a8": q.QARL_W4A8_G128}[fmt_name]
    seed = 1700 + K + T
    w = synth.normal_bf16((E, N, K), 0.02, seed=seed)
    x = synth.normal_bf16((T, K), 1.0, seed=seed + 1)
    x[T // 2] = 0                                                  # a zero row: scale 0, codes 0, output 0
    lg = synth.router_logits(T, E, seed + 2, zipf_s=1.1)
    ids, wts = oracle.route(np_bits(lg), topk)
    counts, offsets, pairs = oracle.group(ids, E)
    M = T * topk
    tok = (pairs // topk).astype(np.int32)
    d_ids = _i32(np.asarray(ids).reshape(-1))
    d_off, d_tok, d_pairs = _i32(offsets), _i32(tok), _i32(pairs)
    d_w = torch.tensor(np.asarray(wts, dtype=np.float32), device="cuda")
    qw = q.qarl_quantize_weights(w.cuda(), fmt)
    inv = torch.tensor(pairs, dtype=torch.long, device="cuda")     # sorted position i holds pair pairs[i]
    xq, sx = q.qarl_quantize_rows_fp8(x.cuda())
    y_grp = q.qarl_qgemm_grouped(qw, xq, d_off, M, row_map=d_tok, x_scales=sx, out_dtype=q.QARL_OUT_F32,
                                 path=q.QARL_PATH_DECODE)
    y_rt = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    q.qarl_qgemm_routed(qw, x.cuda(), d_ids, T, topk, True, out=y_rt, out_dtype=q.QARL_OUT_F32)
    assert torch.equal(y_rt[inv], y_grp)
    xq_ref, sx_ref = oracle.quantize_fp8_rows(np_bits(x))
    if fmt_name == "fp8":
        wc, wsc = oracle.quantize_fp8_rows(np_bits(w).reshape(E * N, K))
        y_ref = oracle.qgemm_fp8(xq_ref, sx_ref, wc.reshape(E, N, K), wsc.reshape(E, N), offsets, tok)
    elif fmt_name == "fp4":
        wc, wsc = oracle.quantize_fp4_rows(np_bits(w).reshape(E * N, K))
        y_ref = oracle.qgemm_fp4w(xq_ref, sx_ref, wc.reshape(E, N, K), wsc.reshape(E, N), offsets, tok)
    else:
        c4, s4 = oracle.quantize_int4(np_bits(w))
        y_ref = oracle.qgemm_w4a8(xq_ref, sx_ref, c4, s4, offsets, tok)
    assert norm_err(y_rt[inv].cpu().numpy(), y_ref) <= (TOL_F32 if fmt_name == "w4a8" else TOL_F32_FP8)
    # SiLU*mul
    a_grp = q.qarl_qgemm_grouped(qw, xq, d_off, M, row_map=d_tok, x_scales=sx, epilogue=q.QARL_EPI_SILU_MUL,
                                 path=q.QARL_PATH_DECODE)
    a_rt = q.qarl_qgemm_routed(qw, x.cuda(), d_ids, T, topk, True, epilogue=q.QARL_EPI_SILU_MUL)
    assert np.array_equal(np_bits(a_rt[inv]), np_bits(a_grp))
    # combine: activation row = pair id
    xp = x[torch.tensor(np.arange(M) // topk, dtype=torch.long)].contiguous()   # one row per pair, pair order
    xg = xp[torch.tensor(pairs, dtype=torch.long)].contiguous()                 # the same rows in sorted order
    xgq, sxg = q.qarl_quantize_rows_fp8(xg.cuda())
    out_grp = q.qarl_qgemm_grouped(qw, xgq, d_off, M, x_scales=sxg, epilogue=q.QARL_EPI_COMBINE, combine_w=d_w,
                                   sorted_pairs=d_pairs, T=T, topk=topk, path=q.QARL_PATH_DECODE)
    out_rt = q.qarl_qgemm_routed(qw, xp.cuda(), d_ids, T, topk, False, epilogue=q.QARL_EPI_COMBINE, combine_w=d_w)
    assert np.array_equal(np_bits(out_rt), np_bits(out_grp))


@pytest.mark.parametrize("fmt_name", ["fp8", "w4a8"])
def test_routed_mode_rows_outside_the_fast_division_range(q, oracle, fmt_name):
    """Rows whose scale leaves the range of the corrected-reciprocal division (absmax near 2^-100 and near 2^100),
    a zero row, negative zeros and a row of one repeated value: the kernel that quantizes its own rows must fall back
    to the IEEE division exactly where the row quantizer does, so routed and grouped results stay bit-identical, and
    the codes the grouped path consumed are the oracle's."""
    fmt = q.QARL_FP8_E4M3_CH if fmt_name == "fp8" else q.QARL_W4A8_G128
    E, N, K, T, topk = 4, 64, 512, 40, 2
    w = synth.normal_bf16((E, N, K), 0.02, seed=1901)
    x = synth.normal_bf16((T, K), 1.0, seed=1902).float()
    x[0] *= 2.0 ** -110
    x[1] *= 2.0 ** 115
    x[2] = 0
    x[3] = 0.375
    x[4, :9] = -0.0
    x[5] *= 2.0 ** -126            # bf16 subnormals
    x = x.to(torch.bfloat16)
    lg = synth.router_logits(T, E, 1903)
    ids, _ = oracle.route(np_bits(lg), topk)
    counts, offsets, pairs = oracle.group(ids, E)
    M = T * topk
    tok = (pairs // topk).astype(np.int32)
    qw = q.qarl_quantize_weights(w.cuda(), fmt)
    xq, sx = q.qarl_quantize_rows_fp8(x.cuda())
    xq_ref, sx_ref = oracle.quantize_fp8_rows(np_bits(x))
    assert np.array_equal(xq.cpu().numpy(), xq_ref) and np.array_equal(sx.cpu().numpy(), sx_ref)
    y_grp = q.qarl_qgemm_grouped(qw, xq, _i32(offsets), M, row_map=_i32(tok), x_scales=sx, out_dtype=q.QARL_OUT_F32,
                                 path=q.QARL_PATH_DECODE)
    y_rt = q.qarl_qgemm_routed(qw, x.cuda(), _i32(np.asarray(ids).reshape(-1)), T, topk, True, out_dtype=q.QARL_OUT_F32)
    inv = torch.tensor(pairs, dtype=torch.long, device="cuda")
    assert torch.equal(y_rt[inv].view(torch.int32), y_grp.view(torch.int32))


def test_routed_mode_errors_and_route_only(q):
    w = synth.normal_bf16((64, 32, 256), 0.02, seed=3).cuda()
    qw = q.qarl_quantize_weights(w)
    x = synth.normal_bf16((600, 256), 1.0, seed=4).cuda()
    ids = torch.zeros((600 * 8,), dtype=torch.int32, device="cuda")
    with pytest.raises(q.QarlError) as ei:                       # more than 512 tokens
        q.qarl_qgemm_routed(qw, x, ids, 600, 8, True)
    assert ei.value.status == q.QARL_ERR_UNSUPPORTED
    with pytest.raises(q.QarlError) as ei:                       # more than 4096 pairs
        q.qarl_qgemm_routed(qw, x, ids, 500, 9, True)
    assert ei.value.status == q.QARL_ERR_UNSUPPORTED
    q8 = q.qarl_quantize_weights(synth.normal_bf16((4, 32, 4096), 0.02, seed=5).cuda(), q.QARL_W4A8_G128)
    with pytest.raises(q.QarlError) as ei:                       # the int4 kernels' routed mode stops at K = 2048
        q.qarl_qgemm_routed(q8, synth.normal_bf16((16, 4096), 1.0, seed=6).cuda(), ids, 16, 8, True)
    assert ei.value.status == q.QARL_ERR_UNSUPPORTED
    out = q.qarl_qgemm_routed(qw, x, ids, 0, 8, True)            # T = 0: nothing to do
    assert out.shape[0] == 0
    # the router without its grouping pass writes the same ids and weights
    lg = synth.router_logits(300, 64, 9).cuda()
    r1 = q.qarl_moe_route(lg, 4)
    r2 = q.qarl_moe_route(lg, 4, group=False)
    assert torch.equal(r1.ids, r2.ids) and torch.equal(r1.w, r2.w)


@pytest.mark.parametrize("path", [1, 2])
def test_layer_is_reproducible_run_to_run(q, path):
    """Wavefronts draw their weight tiles dynamically and workgroups finish in any order; no result may depend on
    it: repeated runs of one layer give the same bits, interleaved with a different batch in between."""
    E, H, I, T, topk = 64, 512, 256, 301, 4
    gu, dn = synth.expert_weights(E, H, I, seed=77)
    layer = q.MoELayer(q.qarl_quantize_weights(gu.cuda()), q.qarl_quantize_weights(dn.cuda()), T, topk, path)
    x = synth.normal_bf16((T, H), 1.0, 78).cuda()
    lg = synth.router_logits(T, E, 79, zipf_s=1.1).cuda()
    x2 = synth.normal_bf16((T, H), 1.0, 80).cuda()
    lg2 = synth.router_logits(T, E, 81).cuda()
    first = layer.forward(x, lg).clone()
    for _ in range(5):
        layer.forward(x2, lg2)
        again = layer.forward(x, lg)
        assert torch.equal(first.view(torch.int16), again.view(torch.int16))


def test_routed_mode_ids_outside_the_expert_range_leave_their_rows_alone(q, oracle):
    """Pairs whose id is not an expert (negative, >= E) select no weight matrix: their output rows keep what the
    buffer held, every other row is unaffected."""
    E, N, K, T, topk = 4, 64, 256, 20, 2
    w = synth.normal_bf16((E, N, K), 0.02, seed=31)
    x = synth.normal_bf16((T, K), 1.0, seed=32)
    rng = np.random.default_rng(33)
    ids = rng.integers(0, E, size=(T, topk)).astype(np.int32)
    ids[:, 1] = (ids[:, 0] + 1) % E                               # a token lists an expert at most once
    good = ids.copy()
    ids[2, 0], ids[7, 1], ids[19, 1] = -1, E, 1000
    qw = q.qarl_quantize_weights(w.cuda())
    M = T * topk
    y = torch.full((M, N), -777.0, dtype=torch.float32, device="cuda")
    q.qarl_qgemm_routed(qw, x.cuda(), _i32(ids.reshape(-1)), T, topk, True, out=y, out_dtype=q.QARL_OUT_F32)
    y2 = torch.full((M, N), -777.0, dtype=torch.float32, device="cuda")
    q.qarl_qgemm_routed(qw, x.cuda(), _i32(good.reshape(-1)), T, topk, True, out=y2, out_dtype=q.QARL_OUT_F32)
    skipped = [2 * topk + 0, 7 * topk + 1, 19 * topk + 1]
    keep = np.ones(M, dtype=bool)
    keep[skipped] = False
    assert bool((y[skipped] == -777.0).all())
    assert torch.equal(y[torch.tensor(keep)], y2[torch.tensor(keep)])
