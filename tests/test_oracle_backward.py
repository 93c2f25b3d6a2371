"""Pins of the oracle's straight-through backward of the grouped W4A16 GEMM (paper section 3.1, item 2)."""
import numpy as np
import torch

from paper_2604_07853_amd import synth


def _case(oracle, E=3, N=48, K=256, rows=(7, 0, 12), seed=1):
    w = synth.normal_bf16((E, N, K), 0.02, seed=seed)
    codes, scales = oracle.quantize_int4(synth.bits(w))
    M = sum(rows)
    off = np.concatenate([[0], np.cumsum(rows)]).astype(np.int32)
    return codes, scales, off, M


def test_one_hot_gradient_returns_rows_of_the_dequantized_weight(oracle):
    E, N, K = 2, 32, 256
    codes, scales, _, _ = _case(oracle, E, N, K, (N, N))
    deq = oracle.dequant_int4(codes, scales)
    eye = synth.bits(torch.eye(N).to(torch.bfloat16))
    dy = np.concatenate([eye, eye])
    dx = oracle.qgemm_w4a16_dx(dy, codes, scales, np.array([0, N, 2 * N], dtype=np.int32))
    assert np.array_equal(dx[:N], deq[0].astype(np.float64)) and np.array_equal(dx[N:], deq[1].astype(np.float64))


def test_exact_integer_regime_equals_integer_matmuls(oracle):
    rng = np.random.default_rng(2)
    E, N, K, rows = 2, 32, 256, (9, 14)
    qi = rng.integers(-7, 8, size=(E, N, K))
    qi[:, :, ::128] = 7
    w = torch.tensor(qi * 0.25, dtype=torch.float32).to(torch.bfloat16)
    codes, scales = oracle.quantize_int4(synth.bits(w))
    M = sum(rows)
    off = np.array([0, rows[0], M], dtype=np.int32)
    dyi = rng.integers(-4, 5, size=(M, N))
    xi = rng.integers(-4, 5, size=(M, K))
    dy = synth.bits(torch.tensor(dyi, dtype=torch.float32).to(torch.bfloat16))
    x = synth.bits(torch.tensor(xi, dtype=torch.float32).to(torch.bfloat16))
    dx = oracle.qgemm_w4a16_dx(dy, codes, scales, off)
    dw = oracle.grouped_dw(dy, x, off, E)
    for e, (lo, hi) in enumerate([(0, rows[0]), (rows[0], M)]):
        assert np.array_equal(dx[lo:hi] * 4, (dyi[lo:hi].astype(np.int64) @ qi[e].astype(np.int64)).astype(np.float64))
        assert np.array_equal(dw[e], (dyi[lo:hi].T.astype(np.int64) @ xi[lo:hi].astype(np.int64)).astype(np.float64))


def test_adjoint_identity_and_finite_difference_of_the_forward(oracle):
    """<dY, Y> = <dX, X> = <dW, What> ties the two gradients to the forward; and the forward is linear in x, so its
    change along a direction d equals <dX, d> when dY holds the weights of a linear loss."""
    rng = np.random.default_rng(3)
    codes, scales, off, M = _case(oracle)
    E, N, K8 = codes.shape
    K = K8 * 8
    x = synth.normal_bf16((M + 5, K), 1.0, seed=4)
    rm = rng.permutation(M + 5)[:M].astype(np.int32)
    dy = synth.normal_bf16((M, N), 1.0, seed=5)
    xb, dyb = synth.bits(x), synth.bits(dy)
    y = oracle.qgemm_w4a16(xb, codes, scales, off, rm)
    dx = oracle.qgemm_w4a16_dx(dyb, codes, scales, off)
    dw = oracle.grouped_dw(dyb, xb, off, E, rm)
    dyf, xf = oracle.bf16_to_f64(dyb), oracle.bf16_to_f64(xb)
    what = oracle.dequant_int4(codes, scales).astype(np.float64)
    a = float((dyf * y).sum())
    assert np.isclose(a, float((dx * xf[rm]).sum()), rtol=1e-11) and np.isclose(a, float((dw * what).sum()), rtol=1e-11)
    # forward difference along a bf16 direction (linear map: exact up to double rounding)
    d = synth.normal_bf16((M + 5, K), 1.0, seed=6)
    x2 = (x.double() + d.double() * 2.0 ** -6)
    x2b = synth.bits(x2.to(torch.bfloat16))
    step = oracle.bf16_to_f64(x2b) - xf                      # the step actually taken after rounding to bf16
    y2 = oracle.qgemm_w4a16(x2b, codes, scales, off, rm)
    assert np.isclose(float((dyf * (y2 - y)).sum()), float((dx * step[rm]).sum()), rtol=1e-9)
    # dW against a plain einsum over each expert's rows
    for e in range(E):
        lo, hi = off[e], off[e + 1]
        assert np.allclose(dw[e], dyf[lo:hi].T @ xf[rm[lo:hi]], rtol=1e-13, atol=1e-300)
