"""Pins of the oracle's FP4 (e2m1, alpha = 6) cast and quantizer and of the two 4-bit-weight x 8-bit-activation
GEMMs (paper section 2.2: FP Quant constants; section 4.2 / the appendix on quantization schemes: W4A8)."""
import numpy as np
import torch

from paper_2604_07853_amd import synth

# the eight magnitudes of e2m1, written out from the format definition (bias 1, one subnormal)
E2M1 = [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]


def test_all_16_patterns_roundtrip_and_midpoints(oracle):
    codes = np.arange(16, dtype=np.uint8)
    vals = oracle.e2m1_decode(codes)
    assert list(vals[:8]) == E2M1 and list(vals[8:]) == [-v for v in E2M1]          # -0.0 == 0.0 compares equal
    assert np.signbit(vals[8])
    for c in range(16):
        if c == 8:
            continue                                                                 # -0 encodes as sign|0
        assert oracle.e2m1_encode(np.array([vals[c]]))[0] == c
    # midpoints between neighbours go to the even code; a hair off goes to the nearer one
    for c in range(7):
        mid = (E2M1[c] + E2M1[c + 1]) / 2
        assert oracle.e2m1_encode(np.array([mid]))[0] == (c if c % 2 == 0 else c + 1)
        assert oracle.e2m1_encode(np.array([mid * (1 - 1e-9)]))[0] == c
        assert oracle.e2m1_encode(np.array([mid * (1 + 1e-9)]))[0] == c + 1
        assert oracle.e2m1_encode(np.array([-mid]))[0] == 8 + (c if c % 2 == 0 else c + 1)
    # saturation at alpha = 6
    assert list(oracle.e2m1_encode(np.array([6.0, 6.5, 100.0, -7.0]))) == [7, 7, 7, 15]


def test_fp4_row_quantizer_against_brute_force(oracle):
    w = synth.normal_bf16((16, 256), 0.02, seed=3)
    wb = synth.bits(w).copy()
    wb[2, :] = 0
    codes, s = oracle.quantize_fp4_rows(wb)
    wf = oracle.bf16_to_f64(wb)
    am = np.abs(wf).max(axis=1)
    assert np.array_equal(s, am.astype(np.float32) / np.float32(6.0))
    assert s[2] == 0 and np.all(codes[2] == 0)
    dec = oracle.e2m1_decode(codes)
    assert np.all(np.abs(dec).max(axis=1)[am > 0] == 6.0)                           # the absmax element maps to +-6
    # brute force: the chosen value is a nearest one among the 15 distinct values, for the fp32 quotient
    grid = np.array(sorted(set(E2M1 + [-v for v in E2M1])))
    for r in (0, 5, 15):
        t = (wf[r].astype(np.float32) / s[r]).astype(np.float64)
        best = np.abs(t[:, None] - grid[None, :]).min(axis=1)
        assert np.all(np.abs(dec[r] - t) <= best * (1 + 1e-12) + 1e-300)
    # dequantization error: at most half the local spacing (<= 1 in units of s above 4, 0.25 below 2)
    err = np.abs(dec * s[:, None].astype(np.float64) - wf)
    assert np.all(err <= s[:, None].astype(np.float64) * 1.0 * (1 + 1e-6))


def test_fp4_and_w4a8_gemms_against_dense_numpy(oracle):
    rng = np.random.default_rng(4)
    E, N, K, rows = 3, 24, 256, (5, 0, 9)
    M = sum(rows)
    off = np.concatenate([[0], np.cumsum(rows)]).astype(np.int32)
    x = synth.normal_bf16((M, K), 1.0, seed=5)
    xq, sx = oracle.quantize_fp8_rows(synth.bits(x))
    w = synth.normal_bf16((E, N, K), 0.02, seed=6)
    rm = rng.permutation(M).astype(np.int32)
    xd = oracle.e4m3_decode(xq) * sx[:, None].astype(np.float64)
    # FP4 weights
    wq, sw = oracle.quantize_fp4_rows(synth.bits(w))
    wd = oracle.e2m1_decode(wq) * sw[..., None].astype(np.float64)
    got = oracle.qgemm_fp4w(xq, sx, wq, sw, off, rm)
    want = np.concatenate([xd[rm[off[e]:off[e + 1]]] @ wd[e].T for e in range(E)])
    assert np.allclose(got, want, rtol=1e-12, atol=1e-300)
    # int4 g128 weights
    c4, s4 = oracle.quantize_int4(synth.bits(w))
    w4 = oracle.dequant_int4(c4, s4).astype(np.float64)
    got = oracle.qgemm_w4a8(xq, sx, c4, s4, off, rm)
    want = np.concatenate([xd[rm[off[e]:off[e + 1]]] @ w4[e].T for e in range(E)])
    assert np.allclose(got, want, rtol=1e-12, atol=1e-300)
    # one-hot activation 448 e_k with scale 1: a column of the dequantized weight, exactly
    xq1 = np.zeros((K, K), dtype=np.uint8)
    xq1[np.arange(K), np.arange(K)] = 0x7e
    o1 = oracle.qgemm_w4a8(xq1, np.ones(K, dtype=np.float32), c4[:1], s4[:1], np.array([0, K], dtype=np.int32))
    assert np.array_equal(o1, 448.0 * w4[0].T)
    o2 = oracle.qgemm_fp4w(xq1, np.ones(K, dtype=np.float32), wq[:1], sw[:1], np.array([0, K], dtype=np.int32))
    assert np.array_equal(o2, 448.0 * wd[0].T)
