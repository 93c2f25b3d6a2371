"""Pins of the oracle's per-token log-prob and mismatch weights (paper eq. (3), the
sequence-level definitions of section 3.2, the appendix figure, and the worked ratio
example of the "Dual Clipping" paragraph)."""
import math
import os

import numpy as np
import scipy.special
import torch

from paper_2604_07853_amd import synth


def test_closed_forms(oracle):
    V, Hh = 1000, 64
    w = synth.bits(synth.normal_bf16((V, Hh), 0.02, seed=1))
    tg = np.array([0, 7, 999], dtype=np.int32)
    lp = oracle.token_logprob(np.zeros((3, Hh), dtype=np.uint16), w, tg)
    assert np.allclose(lp, -math.log(V), rtol=1e-15)               # h = 0 -> uniform
    # one dominant logit -> lp -> 0 for it
    wd = np.zeros((V, Hh), dtype=np.float32)
    wd[5, 0] = 64.0
    h = np.zeros((1, Hh), dtype=np.float32)
    h[0, 0] = 1.0
    lp = oracle.token_logprob(synth.bits(torch.tensor(h).to(torch.bfloat16)),
                              synth.bits(torch.tensor(wd).to(torch.bfloat16)), np.array([5], dtype=np.int32))
    assert -1e-24 < lp[0] <= 0.0


def test_matches_log_softmax_and_normalises(oracle):
    V, Hh, T = 257, 96, 5
    w = synth.normal_bf16((V, Hh), 0.3, seed=2)
    h = synth.normal_bf16((T, Hh), 1.0, seed=3)
    z = h.double().numpy() @ w.double().numpy().T
    for inv_t in (1.0, 2.5):
        ref = scipy.special.log_softmax(z * inv_t, axis=1)
        total = np.zeros(T)
        for v in range(0, V, 17):
            tg = np.full(T, v, dtype=np.int32)
            lp = oracle.token_logprob(synth.bits(h), synth.bits(w), tg, inv_t)
            assert np.allclose(lp, ref[:, v], rtol=1e-12, atol=1e-12)
        allv = np.stack([oracle.token_logprob(synth.bits(h), synth.bits(w), np.full(T, v, dtype=np.int32), inv_t)
                         for v in range(V)], axis=1)
        assert np.allclose(np.exp(allv).sum(axis=1), 1.0, atol=1e-12)


def test_mismatch_weights(oracle):
    rng = np.random.default_rng(0)
    lp = -rng.random(12) * 5
    so = np.array([0, 5, 12], dtype=np.int32)
    d, w, ws, wc = oracle.mismatch(lp, lp, so)
    assert np.all(d == 0) and np.all(w == 1) and np.all(ws == 1) and np.all(wc == 1)
    d, w, ws, wc = oracle.mismatch(lp + 0.25, lp, so)
    assert np.allclose(w, math.exp(0.25)) and np.allclose(ws, math.exp(0.25))
    # sequence weight = geometric mean of the token ratios
    lq = -rng.random(12) * 5
    d, w, ws, wc = oracle.mismatch(lp, lq, so)
    assert np.allclose(ws[0], np.prod(w[:5]) ** (1 / 5)) and np.allclose(ws[1], np.prod(w[5:]) ** (1 / 7))
    # two-sided cap c = 2: weights outside [1/2, 2] are pulled to the bound
    d, w, ws, wc = oracle.mismatch(np.array([1.0, 1.0, -2.0]), np.zeros(3), np.array([0, 2, 3], dtype=np.int32), c=2.0)
    assert np.allclose(ws, [math.e, math.exp(-2.0)]) and np.allclose(wc, [2.0, 0.5])


def test_paper_worked_ratio_example(oracle):
    path = os.path.join(os.path.dirname(__file__), "golden", "ratio_example.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    for p_old, p_new, printed, tol in rows:
        p_old, p_new, printed, tol = map(float, (p_old, p_new, printed, tol))
        d, w, ws, wc = oracle.mismatch(np.array([math.log(p_new)]), np.array([math.log(p_old)]),
                                       np.array([0, 1], dtype=np.int32), c=2.0)
        assert abs(w[0] - printed) <= tol + 1e-12
        assert abs(ws[0] - w[0]) < 1e-15                            # a one-token sequence
    assert abs(wc[0] - 2.0) < 1e-15                                 # 2.5 is capped at c = 2
