"""GPU parity of the fused LM-head log-prob and the mismatch comparison against the oracle."""
import math

import numpy as np
import pytest
import torch

from paper_2604_07853_amd import synth
from gpu_util import np_bits

pytestmark = pytest.mark.gpu

TOL_LP = 1e-4        # absolute, finer than the paper's 3e-4 sequence clip band


@pytest.fixture(scope="module")
def q():
    from paper_2604_07853_amd import binding
    binding.lib()
    return binding


@pytest.mark.parametrize("T,H,V,inv_t", [(200, 128, 1000, 1.0), (129, 256, 777, 3.0), (5, 64, 256, 1.0)])
def test_logprob_matches_oracle(q, oracle, T, H, V, inv_t):
    h = synth.normal_bf16((T, H), 1.0, seed=T)
    w = synth.normal_bf16((V, H), 0.3, seed=V)
    tg = synth.targets(T, V, seed=3)
    tg[0] = 0
    tg[-1] = V - 1
    ref = oracle.token_logprob(np_bits(h), np_bits(w), tg.numpy(), inv_t)
    res = q.qarl_token_logprob(h.cuda(), w.cuda(), tg.cuda(), inv_t)
    got = res["logprob"].cpu().numpy().astype(np.float64)
    assert np.abs(got - ref).max() <= TOL_LP * max(1.0, np.abs(ref).max() / 10)


def test_logprob_closed_forms(q):
    V, H, T = 151936 // 8, 64, 130
    w = synth.normal_bf16((V, H), 0.02, seed=1).cuda()
    h = torch.zeros((T, H), dtype=torch.bfloat16, device="cuda")
    tg = synth.targets(T, V, seed=2).cuda()
    lp = q.qarl_token_logprob(h, w, tg)["logprob"].cpu().numpy()
    assert np.abs(lp + math.log(V)).max() < 2e-6 * math.log(V) + 1e-5   # h = 0 -> uniform -> -ln V


def test_mismatch_comparison(q, oracle):
    rng = np.random.default_rng(0)
    T = 1000
    a = (-rng.random(T) * 6).astype(np.float32)
    b = (a + rng.normal(size=T).astype(np.float32) * 0.3).astype(np.float32)
    so = np.array([0, 100, 100, 612, 1000], dtype=np.int32)              # one empty sequence
    d, w, ws, wc = oracle.mismatch(a.astype(np.float64), b.astype(np.float64), so, c=2.0)
    res = q.qarl_logprob_mismatch(torch.tensor(a).cuda(), torch.tensor(b).cuda(), torch.tensor(so).cuda(), 2.0)
    assert np.allclose(res["delta"].cpu().numpy(), d, atol=1e-6)
    assert np.allclose(res["token_w"].cpu().numpy(), w, rtol=1e-5)
    assert np.allclose(res["seq_w"].cpu().numpy(), ws, rtol=1e-5)
    assert np.allclose(res["seq_w_clipped"].cpu().numpy(), wc, rtol=1e-5)
    same = q.qarl_logprob_mismatch(torch.tensor(a).cuda(), torch.tensor(a).cuda(), torch.tensor(so).cuda(), 2.0)
    assert bool((same["delta"] == 0).all()) and bool((same["token_w"] == 1).all()) and bool((same["seq_w"] == 1).all())
    # a strongly mismatched sequence is capped at c and 1/c
    big = q.qarl_logprob_mismatch(torch.tensor(a).cuda() + 3.0, torch.tensor(a).cuda(), torch.tensor(so).cuda(), 2.0)
    assert np.allclose(big["seq_w_clipped"].cpu().numpy()[[0, 2, 3]], 2.0, rtol=1e-6)


def test_fused_comparison_outputs(q, oracle):
    T, H, V = 256, 128, 512
    h = synth.normal_bf16((T, H), 1.0, seed=5)
    w = synth.normal_bf16((V, H), 0.3, seed=6)
    tg = synth.targets(T, V, seed=7)
    ref = oracle.token_logprob(np_bits(h), np_bits(w), tg.numpy(), 1.0)
    sampler = torch.tensor(ref + np.random.default_rng(1).normal(size=T) * 1e-3, dtype=torch.float32)
    so = torch.tensor([0, 128, 256], dtype=torch.int32)
    res = q.qarl_token_logprob(h.cuda(), w.cuda(), tg.cuda(), 1.0, ref_logprob=sampler.cuda(),
                               seq_offsets=so.cuda(), want_delta=True)
    d, _, ws, wc = oracle.mismatch(ref, sampler.double().numpy(), so.numpy(), 2.0)
    assert np.abs(res["delta"].cpu().numpy() - d).max() <= 2 * TOL_LP
    assert np.allclose(res["seq_w"].cpu().numpy(), ws, atol=2 * TOL_LP)
    assert np.allclose(res["seq_w_clipped"].cpu().numpy(), wc, atol=2 * TOL_LP)


def test_target_outside_vocabulary_gives_nan_for_that_token_only(q, oracle):
    T, H, V = 70, 128, 600
    h = synth.normal_bf16((T, H), 1.0, seed=21)
    w = synth.normal_bf16((V, H), 0.3, seed=22)
    tg = synth.targets(T, V, seed=23)
    ref = oracle.token_logprob(np_bits(h), np_bits(w), tg.numpy(), 1.0)
    bad = tg.clone()
    bad[3], bad[40], bad[69] = -1, V, 2 ** 31 - 1
    got = q.qarl_token_logprob(h.cuda(), w.cuda(), bad.cuda())["logprob"].cpu().numpy()
    assert np.isnan(got[[3, 40, 69]]).all()
    ok = np.ones(T, dtype=bool)
    ok[[3, 40, 69]] = False
    assert np.abs(got[ok].astype(np.float64) - ref[ok]).max() <= TOL_LP
