"""Pins of the oracle's router and grouping: full stable sort, all-ties inputs, softmax
identities."""
import numpy as np
import scipy.special
import torch

from paper_2604_07853_amd import synth


def _check(oracle, lg_bits, topk=8):
    T, E = lg_bits.shape
    ids, w = oracle.route(lg_bits, topk)
    lf = oracle.bf16_to_f64(lg_bits)
    for t in range(T):
        order = sorted(range(E), key=lambda e: (-lf[t, e], e))[:topk]
        assert list(ids[t]) == order
        sm = scipy.special.softmax(lf[t, order])       # softmax over the selected logits
        assert np.allclose(w[t], sm, rtol=1e-12, atol=0)
    assert np.allclose(w.sum(axis=1), 1.0, atol=1e-12)
    return ids, w


def test_random_and_tied_inputs(oracle):
    lg = synth.bits(synth.router_logits(300, 128, seed=1))
    ids, _ = _check(oracle, lg)
    lf = oracle.bf16_to_f64(lg)
    # bf16 logits collide: make sure this input really has ties at the 8th/9th boundary
    srt = -np.sort(-lf, axis=1)
    assert (srt[:, 7] == srt[:, 8]).sum() > 0
    allsame = np.full((4, 128), synth.bits(torch.tensor([0.5]).to(torch.bfloat16))[0], dtype=np.uint16)
    ids, w = _check(oracle, allsame)
    assert np.array_equal(ids, np.tile(np.arange(8, dtype=np.int32), (4, 1)))
    assert np.allclose(w, 0.125)
    few = synth.bits(torch.tensor(np.random.default_rng(0).integers(-1, 2, (64, 128)), dtype=torch.float32).to(torch.bfloat16))
    _check(oracle, few)
    _check(oracle, synth.bits(synth.router_logits(50, 16, seed=2)), topk=1)
    _check(oracle, synth.bits(synth.router_logits(50, 8, seed=3)), topk=8)


def test_no_renorm_is_plain_softmax(oracle):
    lg = synth.bits(synth.router_logits(10, 128, seed=4))
    ids, w = oracle.route(lg, 8, renorm=False)
    p = scipy.special.softmax(oracle.bf16_to_f64(lg), axis=1)
    assert np.allclose(w, np.take_along_axis(p, ids, axis=1), rtol=1e-12)


def test_grouping(oracle):
    lg = synth.bits(synth.router_logits(513, 128, seed=5, zipf_s=1.1))
    ids, _ = oracle.route(lg, 8)
    counts, offsets, pairs = oracle.group(ids, 128)
    assert np.array_equal(counts, np.bincount(ids.ravel(), minlength=128))
    assert offsets[0] == 0 and np.array_equal(np.diff(offsets), counts) and offsets[-1] == 513 * 8
    assert np.array_equal(np.sort(pairs), np.arange(513 * 8))
    exp_of_row = ids.ravel()[pairs]
    assert np.all(np.diff(exp_of_row) >= 0)
    want = np.argsort(ids.ravel(), kind="stable")      # (expert, t, slot) order
    assert np.array_equal(pairs, want.astype(np.int32))
    # skewed load: the Zipf bias concentrates tokens on few experts
    assert counts.max() > 20 * max(1, int(np.median(counts)))
