"""Pins of the oracle's sequence-level surrogate (paper section 3.2, "Sequence Level Objectives", and the
appendix figure "Sequence ratio and weight definition"): closed forms, the geometric-mean definition computed from
probabilities instead of logs, the two clipping bands, the cap, and a finite-difference check of the gradient."""
import math

import numpy as np

# the paper's experiment table: seq_clip_ratio_high, neg_seq_clip_ratio_low/high, seq_tis_imp_ratio_cap
EPS_H, DELTA_L, DELTA_H, CAP = 0.0004, 0.0003, 0.0007, 2.0


def _case(rng, lens):
    so = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    T = int(so[-1])
    lp_old = -rng.random(T) * 4 - 0.01
    return so, T, lp_old


def test_identical_policies_give_mean_advantage(oracle):
    rng = np.random.default_rng(1)
    so, T, lp = _case(rng, [5, 0, 7, 3])                   # one empty response
    adv = np.array([1.5, 9.0, -0.5, 2.0])
    o = oracle.tbpo(lp, lp, lp, so, adv, 1.0, EPS_H, DELTA_L, DELTA_H, CAP)
    assert np.all(o["r"] == 1) and np.all(o["w_clip"] == 1) and np.all(o["r_clip"] == 1) and np.all(o["in_band"] == 1)
    assert np.array_equal(o["obj_seq"], [1.5, 0.0, -0.5, 2.0])          # the empty response contributes nothing
    assert o["objective"] == (1.5 - 0.5 + 2.0) / 3                      # ... and does not count in the mean
    # d/dlp of exp(mean) at ratio 1 is 1/L per token, times A, over the 3 responses with tokens
    assert np.allclose(o["grad"][:5], 1.5 / (5 * 3), rtol=1e-15)
    assert np.allclose(o["grad"][5:12], -0.5 / (7 * 3), rtol=1e-15)
    assert np.allclose(o["grad"][12:], 2.0 / (3 * 3), rtol=1e-15)


def test_ratio_is_the_geometric_mean_of_token_probability_ratios(oracle):
    rng = np.random.default_rng(2)
    so, T, lp_old = _case(rng, [6, 9])
    lp_cur = lp_old + rng.normal(0, 1e-4, T)
    lp_smp = lp_old + rng.normal(0, 0.2, T)
    o = oracle.tbpo(lp_cur, lp_old, lp_smp, so, np.array([1.0, -1.0]), 1.0, 1.0, 1.0, 1.0, 1e9)   # bands and cap wide open
    for s, (lo, hi) in enumerate([(0, 6), (6, 15)]):
        p_cur, p_old, p_smp = np.exp(lp_cur[lo:hi]), np.exp(lp_old[lo:hi]), np.exp(lp_smp[lo:hi])
        geo = lambda p: math.prod(p) ** (1.0 / (hi - lo))                # pi(o|q) of the section
        assert math.isclose(o["r"][s], geo(p_cur) / geo(p_old), rel_tol=1e-12)
        assert math.isclose(o["w_clip"][s], geo(p_old) / geo(p_smp), rel_tol=1e-12)
        assert o["in_band"][s] == 1 and o["r_clip"][s] == o["r"][s]
    # token order inside a response does not matter
    perm = np.concatenate([rng.permutation(6), 6 + rng.permutation(9)])
    o2 = oracle.tbpo(lp_cur[perm], lp_old[perm], lp_smp[perm], so, np.array([1.0, -1.0]), 1.0, 1.0, 1.0, 1.0, 1e9)
    assert np.allclose(o2["r"], o["r"], rtol=1e-13) and np.allclose(o2["w_clip"], o["w_clip"], rtol=1e-13)


def test_bands_by_advantage_sign_and_the_cap(oracle):
    L = 4
    so = np.array([0, L, 2 * L, 3 * L, 4 * L, 5 * L, 6 * L], dtype=np.int32)
    lp_old = np.full(6 * L, -1.0)
    # per response: log-ratio of the current policy (constant per token, so r = exp(a) exactly)
    a = np.array([math.log(1.0002), math.log(1.01), math.log(0.5), math.log(1.0005), math.log(1.01), math.log(0.99)])
    lp_cur = lp_old + np.repeat(a, L)
    adv = np.array([1.0, 1.0, 1.0, -1.0, -1.0, -1.0])
    # mismatch: sampler 4x less likely on response 0 (w = 4 -> cap 2), 4x more likely on response 3 (w = 1/4 -> 1/2)
    lp_smp = lp_old.copy()
    lp_smp[0:L] -= math.log(4.0)
    lp_smp[3 * L:4 * L] += math.log(4.0)
    o = oracle.tbpo(lp_cur, lp_old, lp_smp, so, adv, 1.0, EPS_H, DELTA_L, DELTA_H, CAP)
    assert np.allclose(o["r"], np.exp(a), rtol=1e-14)
    # A >= 0: [0, 1 + eps_h]: 1.0002 inside, 1.01 cut to 1.0004, 0.5 inside (no lower bound)
    # A <  0: [1 - delta_l, 1 + delta_h]: 1.0005 inside, 1.01 cut to 1.0007, 0.99 cut to 0.9997
    assert list(o["in_band"]) == [1, 0, 1, 1, 0, 0]
    assert np.allclose(o["r_clip"], [1.0002, 1 + EPS_H, 0.5, 1.0005, 1 + DELTA_H, 1 - DELTA_L], rtol=1e-14)
    assert np.allclose(o["w_clip"], [2.0, 1, 1, 0.5, 1, 1], rtol=1e-14)
    want = np.array([2.0 * 1.0002, 1 + EPS_H, 0.5, -0.5 * 1.0005, -(1 + DELTA_H), -(1 - DELTA_L)])
    assert np.allclose(o["obj_seq"], want, rtol=1e-14)
    assert math.isclose(o["objective"], want.mean(), rel_tol=1e-14)
    # masked responses take no part in the update
    g = o["grad"].reshape(6, L)
    assert np.all(g[[1, 4, 5]] == 0) and np.all(g[[0, 2]] > 0) and np.all(g[3] < 0)
    # a lower bound for positive advantages (the experiment table's seq_clip_ratio_low) cuts response 2 as well
    o2 = oracle.tbpo(lp_cur, lp_old, lp_smp, so, adv, 0.0003, EPS_H, DELTA_L, DELTA_H, CAP)
    assert list(o2["in_band"]) == [1, 0, 0, 1, 0, 0] and math.isclose(o2["r_clip"][2], 1 - 0.0003, rel_tol=1e-14)


def test_gradient_matches_finite_differences(oracle):
    rng = np.random.default_rng(3)
    so, T, lp_old = _case(rng, [3, 5, 2, 4])
    lp_cur = lp_old + rng.normal(0, 0.02, T)
    lp_cur[8:10] += 1.0                                                  # response 2 far outside its band
    lp_smp = lp_old + rng.normal(0, 0.3, T)
    adv = np.array([0.7, -1.3, 2.0, 0.4])
    args = (so, adv, 1.0, 0.2, 0.1, 0.15, 1.5)
    o = oracle.tbpo(lp_cur, lp_old, lp_smp, *args)
    assert o["in_band"][2] == 0 and o["in_band"][[0, 1, 3]].all()
    h = 1e-6
    for t in range(T):
        up, dn = lp_cur.copy(), lp_cur.copy()
        up[t] += h
        dn[t] -= h
        fd = (oracle.tbpo(up, lp_old, lp_smp, *args)["objective"] - oracle.tbpo(dn, lp_old, lp_smp, *args)["objective"]) / (2 * h)
        assert abs(fd - o["grad"][t]) <= 1e-8 + 1e-6 * abs(o["grad"][t]), (t, fd, o["grad"][t])
