"""Pins of the oracle's integer quantizer (paper section 2.2, integer Quant/Dequant).

None of these re-type the oracle's fp32 formula: they use exact rational arithmetic,
hand-computable cases and invariants that any correct nearest-code quantizer satisfies.
"""
from fractions import Fraction

import numpy as np
import torch

from paper_2604_07853_amd import synth


def _f(bits16):
    return Fraction(float(np.array([bits16], dtype=np.uint16).astype(np.uint32).__lshift__(16).view(np.float32)[0]))


def _bf(vals):
    return synth.bits(torch.tensor(vals, dtype=torch.float32).to(torch.bfloat16))


def test_bf16_rounding_matches_torch(oracle):
    g = torch.Generator().manual_seed(11)
    x = torch.randn(4000, generator=g, dtype=torch.float64) * torch.logspace(-30, 30, 4000, dtype=torch.float64)
    # exact halfway cases between neighbouring bf16 values
    ties = torch.tensor([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -(2.0 + 2.0 ** -7), 0.0, 3.0e38], dtype=torch.float64)
    x = torch.cat([x, ties])
    # float64 -> float32 is exact for the ties; for the random part compare through float32
    x32 = x.to(torch.float32)
    want = synth.bits(x32.to(torch.bfloat16))
    got = oracle.bf16_from_f64(x32.double().numpy())
    assert np.array_equal(got, want)
    assert oracle.bf16_from_f64(np.array([1.0 + 2.0 ** -8]))[0] == 0x3F80      # tie -> even (down)
    assert oracle.bf16_from_f64(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 0x3F82  # tie -> even (up)


def test_nearest_code_and_scale_exact_rational(oracle):
    """Every code is the nearest integer multiple of the stored scale (ties to even) and the
    stored scale is the bf16 nearest to absmax/7, both checked in exact arithmetic."""
    w = synth.normal_bf16((6, 256), 0.02, seed=5)
    wb = synth.bits(w).copy()
    # plant exact ties: group 0 of row 0 gets absmax 7*2^-6 and half-integer multiples
    wb[0, :128] = _bf([0.0] * 128)
    planted = [7.0, 2.5, 3.5, -2.5, -3.5, 0.5, 1.5, -0.5, 6.5, -6.5, 4.5, 5.5]
    wb[0, :len(planted)] = _bf([v * 2.0 ** -6 for v in planted])
    codes, scales = oracle.quantize_int4(wb)
    q = oracle.unpack_int4(codes)
    for r in range(wb.shape[0]):
        for g in range(2):
            grp = wb[r, g * 128:(g + 1) * 128]
            am = max(abs(_f(b)) for b in grp)
            sb = int(scales[r, g])
            target = am / 7
            d = abs(_f(sb) - target)
            for nb in (sb - 1, sb + 1):
                assert d < abs(_f(nb) - target), "scale is not the nearest bf16 to absmax/7"
            S = _f(sb)
            for k in range(128):
                W = _f(grp[k])
                qq = int(q[r, g * 128 + k])
                assert -8 <= qq <= 7
                err = abs(W - S * qq)
                for alt in range(-8, 8):
                    e2 = abs(W - S * alt)
                    assert err <= e2
                    if e2 == err and alt != qq:
                        assert qq % 2 == 0, "tie not resolved to the even code"
    got = [int(v) for v in q[0, :len(planted)]]
    assert got == [7, 2, 4, -2, -4, 0, 2, 0, 6, -6, 4, 6]
    assert scales[0, 0] == _bf([2.0 ** -6])[0]


def test_invariants_random(oracle):
    w = synth.normal_bf16((64, 2048), 0.02, seed=0)
    wb = synth.bits(w)
    codes, scales = oracle.quantize_int4(wb)
    q = oracle.unpack_int4(codes).astype(np.float64)
    assert q.min() >= -8 and q.max() <= 7
    s = oracle.bf16_to_f64(scales)
    wf = oracle.bf16_to_f64(wb)
    deq = oracle.dequant_int4(codes, scales).astype(np.float64)
    assert np.array_equal(deq, np.repeat(s, 128, axis=1) * q)       # dequant = s*q exactly
    sfull = np.repeat(s, 128, axis=1)
    err = np.abs(deq - wf)
    wg = np.abs(wf).reshape(64, 16, 128)
    is_max = (wg == wg.max(axis=2, keepdims=True)).reshape(64, 2048)
    # |dequant(quant(w)) - w| <= s/2, except the absmax element, off by the scale's own
    # bf16 rounding: 7*s vs absmax differ by at most 7 * 2^-9 * s
    assert np.all(err[~is_max] <= sfull[~is_max] / 2)
    assert np.all(err[is_max] <= sfull[is_max] * 7 * 2.0 ** -8)
    assert np.all(np.abs(q[is_max]) == 7)                          # absmax element -> +-7


def test_idempotent_power_of_two_scales(oracle):
    rng = np.random.default_rng(3)
    q = rng.integers(-7, 8, size=(5, 512))
    q[:, ::128] = 7
    q[:, 1::128] = -7
    e = rng.integers(-12, 3, size=(5, 4))
    s = 2.0 ** e
    w = q * np.repeat(s, 128, axis=1)
    wb = synth.bits(torch.tensor(w, dtype=torch.float32).to(torch.bfloat16))
    assert np.array_equal(oracle.bf16_to_f64(wb), w)               # exactly representable
    codes, scales = oracle.quantize_int4(wb)
    assert np.array_equal(oracle.unpack_int4(codes), q.astype(np.int8))
    assert np.array_equal(oracle.bf16_to_f64(scales), s)


def test_hand_cases_and_packing(oracle):
    # constant group c -> every code 7, scale bf16(c/7)
    wb = _bf([0.37] * 128).reshape(1, 128)
    codes, scales = oracle.quantize_int4(wb)
    assert np.all(oracle.unpack_int4(codes) == 7)
    c = oracle.bf16_to_f64(wb)[0, 0]
    assert scales[0, 0] == oracle.bf16_from_f64(np.array([c / 7]))[0]
    # zero group -> scale 0, codes 0 (stored as 8 in every nibble)
    codes, scales = oracle.quantize_int4(np.zeros((1, 128), dtype=np.uint16))
    assert scales[0, 0] == 0 and np.all(codes == 0x88888888)
    # integers -7..7 times 2^-3: scale 2^-3, codes the integers; packing: element i of a
    # word sits in bits [4i, 4i+3] as q+8
    vals = list(range(-7, 1)) + list(range(0, 8)) + [0] * 112
    wb = _bf([v * 0.125 for v in vals]).reshape(1, 128)
    codes, scales = oracle.quantize_int4(wb)
    assert scales[0, 0] == _bf([0.125])[0]
    assert codes[0, 0] == 0x87654321 and codes[0, 1] == 0xFEDCBA98
    assert np.array_equal(oracle.unpack_int4(codes)[0, :16], np.array(vals[:16], dtype=np.int8))
    # negative absmax element -> -7, never -8
    wb = _bf([-1.0] + [0.5] * 127).reshape(1, 128)
    q = oracle.unpack_int4(oracle.quantize_int4(wb)[0])
    assert q[0, 0] == -7 and q.min() == -7
