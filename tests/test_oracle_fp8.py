"""Pins of the oracle's e4m3 cast and FP quantizer (paper section 2.2, FP Quant, alpha=448)."""
import numpy as np
import torch

from paper_2604_07853_amd import synth


def test_all_patterns_roundtrip(oracle):
    codes = np.arange(256, dtype=np.uint8)
    vals = oracle.e4m3_decode(codes)
    ref = torch.from_numpy(codes).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    finite = ~np.isnan(ref)
    assert np.array_equal(vals[finite], ref[finite]) and np.all(np.isnan(vals[~finite]))
    assert vals[0x7e] == 448.0 and vals[0x01] == 2.0 ** -9 and vals[0x08] == 2.0 ** -6
    for c in codes[finite]:
        if c == 0x80:
            continue                                   # -0 encodes as sign|0
        assert oracle.e4m3_encode(np.array([vals[c]]))[0] == c
        assert oracle.e4m3_encode(np.array([vals[c]]), fast=True)[0] == c


def test_midpoints_go_to_even_and_saturate(oracle):
    vals = oracle.e4m3_decode(np.arange(0x7f, dtype=np.uint8))
    mids = (vals[:-1] + vals[1:]) / 2
    enc = oracle.e4m3_encode(mids)
    for c, e in enumerate(enc):
        assert e == (c if c % 2 == 0 else c + 1)
    above = np.array([448.0, 449.0, 464.0, 480.0, 1e6, -1e6])
    assert list(oracle.e4m3_encode(above)) == [0x7e, 0x7e, 0x7e, 0x7e, 0x7e, 0xfe]
    # slightly off the midpoint goes to the nearer neighbour
    assert oracle.e4m3_encode(np.array([mids[40] * (1 - 1e-9)]))[0] == 40
    assert oracle.e4m3_encode(np.array([mids[40] * (1 + 1e-9)]))[0] == 41


def test_cast_matches_torch_in_range_and_fast_matches_slow(oracle):
    g = torch.Generator().manual_seed(2)
    x = (torch.randn(20000, generator=g) * torch.logspace(-4, 2.6, 20000)).clamp(-448, 448)
    want = x.to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = oracle.e4m3_encode(x.double().numpy())
    nz = want != 0x80                                  # torch keeps -0; value is the same
    assert np.array_equal(got[nz] & 0x7f, want[nz] & 0x7f)
    assert np.array_equal((got[nz] >> 7)[(want[nz] & 0x7f) != 0], (want[nz] >> 7)[(want[nz] & 0x7f) != 0])
    assert np.array_equal(oracle.e4m3_encode(x.double().numpy(), fast=True), got)


def test_row_quantizer(oracle):
    w = synth.normal_bf16((32, 768), 0.02, seed=9)
    wb = synth.bits(w).copy()
    wb[3, :] = 0
    codes, s = oracle.quantize_fp8_rows(wb)
    wf = oracle.bf16_to_f64(wb)
    am = np.abs(wf).max(axis=1)
    assert np.array_equal(s, (am.astype(np.float32) / np.float32(448.0)))
    assert s[3] == 0 and np.all(codes[3] == 0)
    dec = oracle.e4m3_decode(codes)
    assert np.all(np.abs(dec).max(axis=1)[am > 0] == 448.0)        # absmax element -> +-448
    deq = dec * s[:, None].astype(np.float64)
    # e4m3 has 4 significant bits: relative error <= 2^-4 on normals, absolute 2^-10*s below
    err = np.abs(deq - wf)
    bound = np.maximum(np.abs(wf) * 2.0 ** -4, s[:, None].astype(np.float64) * 2.0 ** -10) * (1 + 1e-6)
    assert np.all(err <= bound)
    # per-row codes equal torch's cast of the same fp32 quotient (in range by construction)
    r = 5
    t = (torch.from_numpy(wf[r].astype(np.float32)) / torch.tensor(s[r])).clamp(-448, 448)
    want = t.to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    nz = (want & 0x7f) != 0
    assert np.array_equal(codes[r][nz], want[nz])
