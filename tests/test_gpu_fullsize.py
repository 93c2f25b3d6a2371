"""GPU parity at the full workload sizes, in the launch configurations the benchmark times.

The oracle cannot finish a 1.2 TFLOP layer in seconds, so at these sizes it evaluates sampled
output rows one by one (every expert's first and last row, the rows around the tile boundaries
of the most loaded experts, a seeded random draw), each stage on the GPU's own input to that
stage; integer work (codes, scales, routing, grouping) is compared in full.  Weights are drawn
on the device and copied to the host, so both sides read the same bits.
"""
import numpy as np
import pytest
import torch

from paper_2604_07853_amd import synth
from gpu_util import np_bits, norm_err, norm_err_bf16, flip_fraction, unblock_int4, unblock_int4_torch

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-3       # bf16 outputs, half-ulp of the output rounding discounted (see test_gpu_qgemm)
TOL_F32 = 2e-5        # fp32 outputs, W4A16
TOL_F32_FP8 = 1e-3    # fp32 outputs, e4m3 x e4m3 matrix-core products
MAX_FLIPS = 0.02
MAX_FLIPS_FP8 = 0.06
TOL_LOGPROB = 1e-4
E, H, I, TOPK, V = synth.E, synth.H, synth.I, synth.TOPK, synth.V


@pytest.fixture(scope="module")
def q():
    from paper_2604_07853_amd import binding
    binding.lib()
    return binding


@pytest.fixture(scope="module")
def layer_int4(q, oracle):
    """One full layer (128 experts) drawn on the device; quantized by the library and by the oracle,
    codes and scales compared bit for bit over the whole layer."""
    gu, dn = synth.expert_weights(E, H, I, seed=300, device="cuda")
    qgu, qdn = q.qarl_quantize_weights(gu), q.qarl_quantize_weights(dn)
    guc, gus = oracle.quantize_int4(np_bits(gu))
    dnc, dns = oracle.quantize_int4(np_bits(dn))
    del gu, dn
    for qw, c, s, N, K in ((qgu, guc, gus, 2 * I, H), (qdn, dnc, dns, H, I)):
        assert np.array_equal(unblock_int4(qw.codes, E, N, K), c)
        assert np.array_equal(np_bits(qw.scales).reshape(s.shape), s)
    return dict(qgu=qgu, qdn=qdn, guc=guc, gus=gus, dnc=dnc, dns=dns)


def _sample_rows(offsets, rng, n_random=96, tile=64):
    """Sorted-row indices to check: first and last row of every expert, the rows next to the token
    tile boundaries of the three most loaded experts, and a seeded random draw."""
    counts = np.diff(offsets)
    rows = set()
    for e in np.nonzero(counts)[0]:
        rows.add(int(offsets[e]))
        rows.add(int(offsets[e + 1] - 1))
    for e in np.argsort(-counts)[:3]:
        for b in range(tile, int(counts[e]), max(tile, (int(counts[e]) // (4 * tile)) * tile)):
            for d in (-1, 0, 1):
                if 0 <= b + d < counts[e]:
                    rows.add(int(offsets[e] + b + d))
    rows.update(int(r) for r in rng.integers(0, int(offsets[-1]), n_random))
    return np.array(sorted(rows), dtype=np.int64)


def _sub_offsets(rows, offsets):
    """Expert offsets of the sub-problem made of the sampled sorted rows."""
    e_of = np.searchsorted(offsets, rows, side="right") - 1
    sub = np.zeros(offsets.size, dtype=np.int32)
    np.add.at(sub, e_of + 1, 1)
    return np.cumsum(sub).astype(np.int32)


def _token_rows(tokens, pairs, topk):
    """Sorted-row position of every (token, slot) pair of the given tokens, ascending."""
    inv = np.empty(pairs.size, dtype=np.int64)
    inv[pairs] = np.arange(pairs.size)
    pos = inv[(tokens[:, None] * topk + np.arange(topk)[None, :]).reshape(-1)]
    return np.sort(pos)


def _check_route(q, oracle, lg, T):
    r = q.qarl_moe_route(lg, TOPK)
    ids, w = oracle.route(np_bits(lg), TOPK)
    counts, offsets, pairs = oracle.group(ids, E)
    assert np.array_equal(r.ids.cpu().numpy(), ids)
    assert np.array_equal(r.counts.cpu().numpy(), counts)
    assert np.array_equal(r.offsets.cpu().numpy(), offsets)
    assert np.array_equal(r.pairs.cpu().numpy(), pairs)
    assert float(np.abs(r.w.cpu().numpy().astype(np.float64) - w).max()) <= 1e-6
    return r, w, offsets, pairs


def _w4a16_stages(q, oracle, L, x, lg, T, path, seed):
    """gate_up+SiLU, down (fp32) and down+combine (bf16) at full size; sampled rows against the oracle."""
    rng = np.random.default_rng(seed)
    r, w, offsets, pairs = _check_route(q, oracle, lg, T)
    M = T * TOPK
    tok = (pairs // TOPK).astype(np.int32)
    layer = q.MoELayer(L["qgu"], L["qdn"], T, TOPK, path)

    a_gpu = q.qarl_qgemm_grouped(L["qgu"], x, r.offsets, M, row_map=r.tokens, epilogue=q.QARL_EPI_SILU_MUL,
                                 path=path, ws=layer.ws)
    rows = _sample_rows(offsets, rng)
    sub = _sub_offsets(rows, offsets)
    gu_ref = oracle.qgemm_w4a16(np_bits(x), L["guc"], L["gus"], sub, tok[rows])
    a_ref_bits, a_ref = oracle.silu_mul(gu_ref)
    a_rows = a_gpu[torch.from_numpy(rows).cuda()]
    ea = norm_err_bf16(a_rows.float().cpu().numpy(), a_ref)
    assert ea <= TOL_BF16, ea
    fl = flip_fraction(np_bits(a_rows), a_ref_bits)
    assert fl <= MAX_FLIPS, fl

    y_gpu = q.qarl_qgemm_grouped(L["qdn"], a_gpu, r.offsets, M, out_dtype=q.QARL_OUT_F32, path=path, ws=layer.ws)
    y_ref = oracle.qgemm_w4a16(np_bits(a_rows), L["dnc"], L["dns"], sub)
    ey = norm_err(y_gpu[torch.from_numpy(rows).cuda()].cpu().numpy(), y_ref)
    assert ey <= TOL_F32, ey
    del y_gpu

    out_gpu = q.qarl_qgemm_grouped(L["qdn"], a_gpu, r.offsets, M, epilogue=q.QARL_EPI_COMBINE, combine_w=r.w,
                                   sorted_pairs=r.pairs, T=T, topk=TOPK, path=path, ws=layer.ws)
    toks = np.unique(np.concatenate([[0, T - 1], rng.integers(0, T, 46)])).astype(np.int64)
    trows = _token_rows(toks, pairs, TOPK)
    tsub = _sub_offsets(trows, offsets)
    yt_ref = oracle.qgemm_w4a16(np_bits(a_gpu[torch.from_numpy(trows).cuda()]), L["dnc"], L["dns"], tsub)
    renum = np.searchsorted(toks, pairs[trows] // TOPK) * TOPK + pairs[trows] % TOPK
    out_ref, out_ref_bits = oracle.combine(yt_ref, renum.astype(np.int32), w[toks], toks.size, TOPK)
    out_rows = out_gpu[torch.from_numpy(toks).cuda()]
    eo = norm_err_bf16(out_rows.float().cpu().numpy(), out_ref)
    assert eo <= TOL_BF16, eo
    fl = flip_fraction(np_bits(out_rows), out_ref_bits)
    assert fl <= MAX_FLIPS, fl

    out2 = layer.forward(x, lg)                                   # the call sequence the benchmark times
    assert torch.equal(out2.view(torch.int16), out_gpu.view(torch.int16))
    assert bool(torch.isfinite(out2.float()).all())
    return out_gpu


def test_prefill_config3_w4a16_zipf(q, oracle, layer_int4):
    """Config 3: 8 x 2048 tokens, Zipf(1.1)-skewed router, W4A16, prefill path."""
    T = 16384
    x = synth.normal_bf16((T, H), 1.0, seed=310, device="cuda")
    lg = synth.router_logits(T, E, seed=311, device="cuda", zipf_s=1.1)
    _w4a16_stages(q, oracle, layer_int4, x, lg, T, q.QARL_PATH_PREFILL, seed=312)


def test_decode_config5_requantize_then_512_tokens(q, oracle, layer_int4):
    """Config 5, per layer: masters move by N(0, 1e-4), the layer is re-quantized into the SAME
    buffers, then decoded at 512 tokens.  Codes and scales must follow the new masters bit for bit
    (a stale buffer would keep the old ones) and some of them must actually have changed."""
    T = 512
    for layer_seed in (320, 330):
        gu, dn = synth.expert_weights(E, H, I, seed=layer_seed, device="cuda")
        qgu, qdn = q.qarl_quantize_weights(gu), q.qarl_quantize_weights(dn)
        old_codes = qgu.codes.clone()
        gu2 = synth.perturb(gu, 1e-4, layer_seed + 2)
        dn2 = synth.perturb(dn, 1e-4, layer_seed + 3)
        del gu, dn
        q.qarl_quantize_weights(gu2, out=qgu)
        q.qarl_quantize_weights(dn2, out=qdn)
        guc, gus = oracle.quantize_int4(np_bits(gu2))
        dnc, dns = oracle.quantize_int4(np_bits(dn2))
        del gu2, dn2
        for qw, c, s, N, K in ((qgu, guc, gus, 2 * I, H), (qdn, dnc, dns, H, I)):
            assert np.array_equal(unblock_int4(qw.codes, E, N, K), c)
            assert np.array_equal(np_bits(qw.scales).reshape(s.shape), s)
        changed = float((old_codes != qgu.codes).float().mean())
        assert 0.01 < changed < 0.5, changed      # fraction of 8-code words that moved
        L = dict(qgu=qgu, qdn=qdn, guc=guc, gus=gus, dnc=dnc, dns=dns)
        x = synth.normal_bf16((T, H), 1.0, seed=layer_seed + 4, device="cuda")
        lg = synth.router_logits(T, E, seed=layer_seed + 5, device="cuda")
        _w4a16_stages(q, oracle, L, x, lg, T, q.QARL_PATH_DECODE, seed=layer_seed + 6)


def test_config5_all_48_layers_codes_and_scales(q, oracle):
    """Config 5, the weight pass over the whole stack: every one of the 48 layers is drawn, moved by N(0, 1e-4),
    re-quantized into the buffers that held the previous layer's codes, and compared with the oracle's codes and
    scales bit for bit (the GEMM stages run on two layers in the test above)."""
    qgu = q.QWeight.empty(q.QARL_W4A16_G128, E, 2 * I, H)
    qdn = q.QWeight.empty(q.QARL_W4A16_G128, E, H, I)
    for layer in range(48):
        gu, dn = synth.expert_weights(E, H, I, seed=5000 + 2 * layer, device="cuda")
        gu2 = synth.perturb(gu, 1e-4, 6000 + 2 * layer)
        dn2 = synth.perturb(dn, 1e-4, 6001 + 2 * layer)
        del gu, dn
        q.qarl_quantize_weights(gu2, out=qgu)
        q.qarl_quantize_weights(dn2, out=qdn)
        for qw, m, N, K in ((qgu, gu2, 2 * I, H), (qdn, dn2, H, I)):
            c, s = oracle.quantize_int4(np_bits(m))
            got = unblock_int4_torch(qw.codes, E, N, K)
            assert torch.equal(got, torch.from_numpy(c.view(np.int32)).cuda()), layer
            assert torch.equal(qw.scales.view(torch.int16).reshape(s.shape),
                               torch.from_numpy(s.view(np.int16)).cuda()), layer
        del gu2, dn2
        if layer % 8 == 7:
            print("config 5: layers 0..%d identical" % layer, flush=True)


@pytest.mark.parametrize("T,path", [(256, 1), (8192, 2)])
def test_fp8_config4(q, oracle, T, path):
    """Config 4: e4m3 weights with per-channel scales, per-token e4m3 activations; 256 tokens on the
    decode path and 8192 tokens on the prefill path."""
    rng = np.random.default_rng(400 + T)
    gu, dn = synth.expert_weights(E, H, I, seed=400, device="cuda")
    qgu = q.qarl_quantize_weights(gu, q.QARL_FP8_E4M3_CH)
    qdn = q.qarl_quantize_weights(dn, q.QARL_FP8_E4M3_CH)
    guq, gus = oracle.quantize_fp8_rows(np_bits(gu))
    dnq, dns = oracle.quantize_fp8_rows(np_bits(dn))
    del gu, dn
    for qw, c, s in ((qgu, guq, gus), (qdn, dnq, dns)):
        assert np.array_equal(qw.codes.cpu().numpy().reshape(c.shape), c)
        assert np.array_equal(qw.scales.cpu().numpy().reshape(s.shape), s)
    x = synth.normal_bf16((T, H), 1.0, seed=401 + T, device="cuda")
    lg = synth.router_logits(T, E, seed=402 + T, device="cuda")
    r, w, offsets, pairs = _check_route(q, oracle, lg, T)
    M = T * TOPK
    tok = (pairs // TOPK).astype(np.int32)
    layer = q.MoELayer(qgu, qdn, T, TOPK, path)

    xq, sx = q.qarl_quantize_rows_fp8(x)
    xq_ref, sx_ref = oracle.quantize_fp8_rows(np_bits(x))
    assert np.array_equal(xq.cpu().numpy(), xq_ref) and np.array_equal(sx.cpu().numpy(), sx_ref)
    a_gpu = q.qarl_qgemm_grouped(qgu, xq, r.offsets, M, row_map=r.tokens, x_scales=sx,
                                 epilogue=q.QARL_EPI_SILU_MUL, path=path, ws=layer.ws)
    rows = _sample_rows(offsets, rng)
    sub = _sub_offsets(rows, offsets)
    gu_ref = oracle.qgemm_fp8(xq_ref, sx_ref, guq, gus, sub, tok[rows])
    a_ref_bits, a_ref = oracle.silu_mul(gu_ref)
    a_rows = a_gpu[torch.from_numpy(rows).cuda()]
    ea = norm_err_bf16(a_rows.float().cpu().numpy(), a_ref)
    assert ea <= TOL_BF16, ea
    fl = flip_fraction(np_bits(a_rows), a_ref_bits)
    assert fl <= MAX_FLIPS_FP8, fl

    aq, sa = q.qarl_quantize_rows_fp8(a_gpu)
    aq_ref, sa_ref = oracle.quantize_fp8_rows(np_bits(a_gpu))       # the oracle on the GPU's own a
    assert np.array_equal(aq.cpu().numpy(), aq_ref) and np.array_equal(sa.cpu().numpy(), sa_ref)
    y_gpu = q.qarl_qgemm_grouped(qdn, aq, r.offsets, M, x_scales=sa, out_dtype=q.QARL_OUT_F32, path=path,
                                 ws=layer.ws)
    y_ref = oracle.qgemm_fp8(aq_ref[rows], sa_ref[rows], dnq, dns, sub)
    ey = norm_err(y_gpu[torch.from_numpy(rows).cuda()].cpu().numpy(), y_ref)
    assert ey <= TOL_F32_FP8, ey
    del y_gpu

    out_gpu = q.qarl_qgemm_grouped(qdn, aq, r.offsets, M, x_scales=sa, epilogue=q.QARL_EPI_COMBINE,
                                   combine_w=r.w, sorted_pairs=r.pairs, T=T, topk=TOPK, path=path, ws=layer.ws)
    toks = np.unique(np.concatenate([[0, T - 1], rng.integers(0, T, 46)])).astype(np.int64)
    trows = _token_rows(toks, pairs, TOPK)
    tsub = _sub_offsets(trows, offsets)
    yt_ref = oracle.qgemm_fp8(aq_ref[trows], sa_ref[trows], dnq, dns, tsub)
    renum = np.searchsorted(toks, pairs[trows] // TOPK) * TOPK + pairs[trows] % TOPK
    out_ref, _ = oracle.combine(yt_ref, renum.astype(np.int32), w[toks], toks.size, TOPK)
    eo = norm_err_bf16(out_gpu[torch.from_numpy(toks).cuda()].float().cpu().numpy(), out_ref)
    assert eo <= TOL_BF16, eo
    out2 = layer.forward(x, lg)
    assert torch.equal(out2.view(torch.int16), out_gpu.view(torch.int16))


@pytest.mark.parametrize("T,path", [(256, 1), (8192, 2)])
def test_fp4_full_size(q, oracle, T, path):
    """The FP4 (e2m1 weights, e4m3 activations) layer at the sizes the benchmark times: codes of the whole gate_up
    tensor through the canonical export against the oracle's quantizer, then sampled rows of gate_up (SiLU*mul) and of
    down on the GPU's own intermediate: 256 tokens on the decode path (also driven by the router's ids), 8192 tokens
    on the tiled path, where the matrix instruction reads the e2m1 codes natively."""
    rng = np.random.default_rng(600 + T)
    gu, dn = synth.expert_weights(E, H, I, seed=600, device="cuda")
    qgu = q.qarl_quantize_weights(gu, q.QARL_FP4_E2M1_CH)
    qdn = q.qarl_quantize_weights(dn, q.QARL_FP4_E2M1_CH)
    guq, gus = oracle.quantize_fp4_rows(np_bits(gu))      # one code per byte
    dnq, dns = oracle.quantize_fp4_rows(np_bits(dn))
    del gu, dn
    for qw, c, s in ((qgu, guq, gus), (qdn, dnq, dns)):
        canon = q.qarl_codes_to_canonical(qw).cpu().numpy().view(np.uint8).reshape(c.shape[:-1] + (c.shape[-1] // 2,))
        assert np.array_equal(canon & 15, c[..., 0::2]) and np.array_equal(canon >> 4, c[..., 1::2])
        assert np.array_equal(qw.scales.cpu().numpy().reshape(s.shape), s)
        del canon
    x = synth.normal_bf16((T, H), 1.0, seed=601 + T, device="cuda")
    lg = synth.router_logits(T, E, seed=602 + T, device="cuda")
    r, w, offsets, pairs = _check_route(q, oracle, lg, T)
    M = T * TOPK
    tok = (pairs // TOPK).astype(np.int32)
    layer = q.MoELayer(qgu, qdn, T, TOPK, path)
    xq, sx = q.qarl_quantize_rows_fp8(x)
    xq_ref, sx_ref = oracle.quantize_fp8_rows(np_bits(x))
    a_gpu = q.qarl_qgemm_grouped(qgu, xq, r.offsets, M, row_map=r.tokens, x_scales=sx,
                                 epilogue=q.QARL_EPI_SILU_MUL, path=path, ws=layer.ws)
    rows = _sample_rows(offsets, rng, tile=128)
    sub = _sub_offsets(rows, offsets)
    a_ref_bits, a_ref = oracle.silu_mul(oracle.qgemm_fp4w(xq_ref, sx_ref, guq, gus, sub, tok[rows]))
    a_rows = a_gpu[torch.from_numpy(rows).cuda()]
    ea = norm_err_bf16(a_rows.float().cpu().numpy(), a_ref)
    assert ea <= TOL_BF16, ea
    assert flip_fraction(np_bits(a_rows), a_ref_bits) <= MAX_FLIPS_FP8
    aq, sa = q.qarl_quantize_rows_fp8(a_gpu)
    aq_h, sa_h = aq.cpu().numpy(), sa.cpu().numpy()
    y_gpu = q.qarl_qgemm_grouped(qdn, aq, r.offsets, M, x_scales=sa, out_dtype=q.QARL_OUT_F32, path=path, ws=layer.ws)
    y_ref = oracle.qgemm_fp4w(aq_h[rows], sa_h[rows], dnq, dns, sub)
    ey = norm_err(y_gpu[torch.from_numpy(rows).cuda()].cpu().numpy(), y_ref)
    assert ey <= TOL_F32_FP8, ey
    del y_gpu
    out_gpu = q.qarl_qgemm_grouped(qdn, aq, r.offsets, M, x_scales=sa, epilogue=q.QARL_EPI_COMBINE,
                                   combine_w=r.w, sorted_pairs=r.pairs, T=T, topk=TOPK, path=path, ws=layer.ws)
    out2 = layer.forward(x, lg)            # at 256 tokens the layer runs the routed kernels on 16-bit rows
    assert torch.equal(out2.view(torch.int16), out_gpu.view(torch.int16))


def test_logprob_config3_and_path_mismatch(q, oracle, layer_int4):
    """Config 3's second half: the LM head [151936, 2048] over 16384 hidden states with the fused
    per-token log-prob, sampled rows against the oracle; then the comparison the method exists for:
    the same 8 sequences pushed through the decode path (256 tokens at a time, as a sampler would)
    and through the prefill path (all at once, as the learner does) must give per-token log-probs
    whose sequence-level ratio stays far inside the paper's 3e-4 band (training-dynamics section)."""
    T, S = 16384, 8
    rng = np.random.default_rng(500)
    L = layer_int4
    x = synth.normal_bf16((T, H), 1.0, seed=510, device="cuda")
    lg = synth.router_logits(T, E, seed=511, device="cuda", zipf_s=1.1)
    h_pre = q.MoELayer(L["qgu"], L["qdn"], T, TOPK, q.QARL_PATH_PREFILL).forward(x, lg).clone()
    dec = q.MoELayer(L["qgu"], L["qdn"], 256, TOPK, q.QARL_PATH_DECODE)
    h_dec = torch.empty_like(h_pre)
    for b in range(T // 256):
        h_dec[b * 256:(b + 1) * 256] = dec.forward(x[b * 256:(b + 1) * 256].contiguous(),
                                                   lg[b * 256:(b + 1) * 256].contiguous())
    # same codes, same scales, same dequantization rule: the two paths differ by summation order only
    d = (h_pre.float() - h_dec.float()).abs()
    rms = float(h_pre.float().pow(2).mean().sqrt())
    assert float(d.max()) <= 2.0 ** -7 * (float(h_pre.float().abs().max()) + rms)   # at most one bf16 step
    assert float((d > 0).float().mean()) <= MAX_FLIPS

    wlm = synth.normal_bf16((V, H), 0.02, seed=512, device="cuda")
    # logits peaked enough that sampled tokens carry probabilities of a few percent to ~0.8
    z_std = rms * (H ** 0.5) * 0.02
    inv_t = float(np.float32(4.0 / z_std))
    # targets are an input: half uniform over the vocabulary (low-probability tokens), half drawn from
    # the softmax by Gumbel-max on fp32 logits formed here, outside the library
    tg = synth.targets(T, V, seed=513, device="cuda")
    g = torch.Generator(device="cuda")
    g.manual_seed(514)
    for t0 in range(0, T, 4096):
        sl = slice(t0 + 2048, t0 + 4096)
        z = (h_pre[sl].float() @ wlm.float().T) * inv_t
        z += -torch.log(-torch.log(torch.rand(z.shape, generator=g, device="cuda").clamp_min(1e-20)))
        tg[sl] = z.argmax(dim=1).to(torch.int32)
        del z
    ws = torch.empty((q.qarl_logprob_workspace_bytes(T, H, V),), dtype=torch.uint8, device="cuda")
    lp_pre = q.qarl_token_logprob(h_pre, wlm, tg, inv_temperature=inv_t, ws=ws)["logprob"].clone()
    lp_dec = q.qarl_token_logprob(h_dec, wlm, tg, inv_temperature=inv_t, ws=ws)["logprob"].clone()
    assert bool(torch.isfinite(lp_pre).all()) and float(lp_pre.max()) <= 0.0

    rows = np.unique(np.concatenate([[0, 127, 128, T - 1], rng.integers(0, T, 20)])).astype(np.int64)
    idx = torch.from_numpy(rows).cuda()
    lp_ref = oracle.token_logprob(np_bits(h_pre[idx]), np_bits(wlm), tg[idx].cpu().numpy(), inv_t)
    e = float(np.abs(lp_pre[idx].cpu().numpy().astype(np.float64) - lp_ref).max())
    assert e <= TOL_LOGPROB, e
    p = np.exp(lp_ref)
    assert p.max() > 0.02, p.max()         # the peaked regime was reached

    so = torch.arange(0, T + 1, T // S, dtype=torch.int32, device="cuda")
    res = q.qarl_logprob_mismatch(lp_pre, lp_dec, so, 2.0)
    dr, wr, wsr, wcr = oracle.mismatch(lp_pre.cpu().numpy(), lp_dec.cpu().numpy(), so.cpu().numpy(), 2.0)
    assert float(np.abs(res["delta"].cpu().numpy() - dr).max()) <= 1e-6
    assert float(np.abs(res["seq_w"].cpu().numpy() - wsr).max()) <= 1e-6
    assert float(np.abs(res["seq_w_clipped"].cpu().numpy() - wcr).max()) <= 1e-6
    assert float(np.abs(wsr - 1.0).max()) < 3e-4, wsr


def test_dense_mlp_second_model_shape(q, oracle):
    """A dense (non-MoE) SiLU-gated MLP of a second model shape through the same entry points: hidden 4096,
    intermediate 12288 (E = 1), 4096 tokens on the MFMA-tiled path (AUTO), and a 40-token decode batch of the
    gate_up projection on the weight-streaming path, whose K = 4096 takes the 16-row LDS tile (three row blocks).
    K = 12288 (the down projection) is beyond that kernel and must be refused there.  Codes and scales in full,
    GEMM outputs on sampled rows (first and last, rows around the 64-row tile borders, a seeded draw)."""
    H2, I2, T = 4096, 12288, 4096
    gu = synth.normal_bf16((1, 2 * I2, H2), 0.02, seed=700, device="cuda")
    dn = synth.normal_bf16((1, H2, I2), 0.02, seed=701, device="cuda")
    x = synth.normal_bf16((T, H2), 1.0, seed=702, device="cuda")
    qgu, qdn = q.qarl_quantize_weights(gu), q.qarl_quantize_weights(dn)
    guc, gus = oracle.quantize_int4(np_bits(gu))
    dnc, dns = oracle.quantize_int4(np_bits(dn))
    del gu, dn
    for qw, c, s, N, K in ((qgu, guc, gus, 2 * I2, H2), (qdn, dnc, dns, H2, I2)):
        assert np.array_equal(unblock_int4(qw.codes, 1, N, K), c)
        assert np.array_equal(np_bits(qw.scales).reshape(s.shape), s)
    off = torch.tensor([0, T], dtype=torch.int32, device="cuda")
    a = q.qarl_qgemm_grouped(qgu, x, off, T, epilogue=q.QARL_EPI_SILU_MUL, path=q.QARL_PATH_AUTO)
    with pytest.raises(q.QarlError) as ei:
        q.qarl_qgemm_grouped(qdn, a, off, T, out_dtype=q.QARL_OUT_F32, path=q.QARL_PATH_DECODE)
    assert ei.value.status == q.QARL_ERR_UNSUPPORTED
    # decode batch through the streaming kernel: SiLU epilogue in bf16 and the plain one in fp32
    Td = 40
    offd = torch.tensor([0, Td], dtype=torch.int32, device="cuda")
    xd = x[:Td].contiguous()
    subd = np.array([0, Td], dtype=np.int32)
    gud_ref = oracle.qgemm_w4a16(np_bits(xd), guc, gus, subd)
    yd = q.qarl_qgemm_grouped(qgu, xd, offd, Td, out_dtype=q.QARL_OUT_F32, path=q.QARL_PATH_DECODE)
    assert norm_err(yd.cpu().numpy(), gud_ref) <= TOL_F32
    ad = q.qarl_qgemm_grouped(qgu, xd, offd, Td, epilogue=q.QARL_EPI_SILU_MUL, path=q.QARL_PATH_DECODE)
    ad_ref_bits, ad_ref = oracle.silu_mul(gud_ref)
    assert norm_err_bf16(ad.float().cpu().numpy(), ad_ref) <= TOL_BF16
    assert flip_fraction(np_bits(ad), ad_ref_bits) <= MAX_FLIPS
    y = q.qarl_qgemm_grouped(qdn, a, off, T, out_dtype=q.QARL_OUT_F32, path=q.QARL_PATH_AUTO)
    rng = np.random.default_rng(703)
    rows = np.unique(np.concatenate([[0, 1, 63, 64, 65, 127, 128, T - 65, T - 64, T - 1], rng.integers(0, T, 22)]))
    sub = np.array([0, rows.size], dtype=np.int32)
    xr = np_bits(x[torch.tensor(rows, device="cuda")])
    gu_ref = oracle.qgemm_w4a16(xr, guc, gus, sub)
    a_ref_bits, a_ref = oracle.silu_mul(gu_ref)
    a_rows = a[torch.tensor(rows, device="cuda")]
    assert norm_err_bf16(a_rows.float().cpu().numpy(), a_ref) <= TOL_BF16
    assert flip_fraction(np_bits(a_rows), a_ref_bits) <= MAX_FLIPS
    y_ref = oracle.qgemm_w4a16(np_bits(a_rows), dnc, dns, sub)          # on the GPU's own a
    assert norm_err(y[torch.tensor(rows, device="cuda")].cpu().numpy(), y_ref) <= TOL_F32


def test_dense_decode_down_projection_as_k_chunks(q, oracle):
    """The K = 12288 down projection of the dense model at a decode batch, on the weight-streaming path: the
    contraction is cut into six chunks of 2048, chunk c of the weight is expert c (W'[c][n][k'] = W[n][2048 c + k'];
    scale groups of 128 never straddle a chunk, so codes and scales are those of W), the activation matrix
    [T][12288] is read as [6 T][2048] (row 6 t + c = chunk c of token t = the pair id of token t, slot c), every
    token lists all six experts, and the combine epilogue with unit weights adds the six fp32 partial products in
    chunk order.  Against the oracle's dense product of the unchunked tensors."""
    H2, I2, Td, C, KC = 4096, 12288, 40, 6, 2048
    dn = synth.normal_bf16((1, H2, I2), 0.02, seed=701, device="cuda")
    a = synth.normal_bf16((Td, I2), 1.0, seed=705, device="cuda")
    dnc, dns = oracle.quantize_int4(np_bits(dn))
    ref = oracle.qgemm_w4a16(np_bits(a), dnc, dns, np.array([0, Td], dtype=np.int32))
    qc = q.qarl_quantize_weights(dn.view(H2, C, KC).permute(1, 0, 2).contiguous())          # E = 6, N = 4096, K = 2048
    assert np.array_equal(unblock_int4(qc.codes, C, H2, KC), dnc.reshape(H2, C, KC // 8).transpose(1, 0, 2))
    assert np.array_equal(np_bits(qc.scales).reshape(C, H2, KC // 128), dns.reshape(H2, C, KC // 128).transpose(1, 0, 2))
    ids = torch.arange(C, dtype=torch.int32, device="cuda").repeat(Td, 1).contiguous()
    ones = torch.ones((Td, C), dtype=torch.float32, device="cuda")
    out = q.qarl_qgemm_routed(qc, a.view(Td * C, KC), ids, Td, C, False, epilogue=q.QARL_EPI_COMBINE, combine_w=ones)
    assert out.shape == (Td, H2)
    assert norm_err_bf16(out.float().cpu().numpy(), ref) <= TOL_BF16
    ref_bits = np_bits(torch.tensor(ref, dtype=torch.float64).to(torch.bfloat16))
    assert flip_fraction(np_bits(out), ref_bits) <= MAX_FLIPS
