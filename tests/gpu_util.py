"""Helpers shared by the GPU parity tests."""
import numpy as np
import torch

from paper_2604_07853_amd import synth


def dev(t):
    return t.cuda()


def np_bits(t):
    return synth.bits(t)


def to_np(t):
    t = t.detach().cpu()
    if t.dtype == torch.bfloat16:
        return t.double().numpy()
    return t.numpy()


def norm_err(got, ref):
    """max |got - ref| / (|ref| + rms(ref)): relative error that stays meaningful near zero."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    rms = np.sqrt((ref ** 2).mean()) if ref.size else 0.0
    if ref.size == 0:
        return 0.0
    return float((np.abs(got - ref) / (np.abs(ref) + rms + 1e-300)).max())


def bf16_half_ulp(ref):
    """Half the spacing of bf16 (8 significant bits) at |ref|: the output format's own rounding."""
    a = np.abs(np.asarray(ref, dtype=np.float64))
    e = np.floor(np.log2(np.maximum(a, 2.0 ** -126)))
    return 2.0 ** (e - 8)


def norm_err_bf16(got, ref):
    """norm_err of a bf16 output after discounting the final rounding to bf16 itself, which any
    bf16 result (the oracle's too) carries: max (|got - ref| - half_ulp(ref))+ / (|ref| + rms)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if ref.size == 0:
        return 0.0
    rms = np.sqrt((ref ** 2).mean())
    # the undiscounted figure first: the bar itself (2e-3) plus the most a rounding to bf16 can add (2^-9 of the
    # binade top, i.e. below 2^-8 of the value)
    raw = float((np.abs(got - ref) / (np.abs(ref) + rms + 1e-300)).max())
    assert raw <= 2e-3 + 2.0 ** -8, "bf16 output off by %.3e before any discount" % raw
    d = np.maximum(np.abs(got - ref) - bf16_half_ulp(ref) * (1 + 1e-9), 0.0)
    return float((d / (np.abs(ref) + rms + 1e-300)).max())


def flip_fraction(got_bits, ref_bits):
    """Fraction of bf16 outputs whose bit pattern differs from the oracle's rounded output."""
    return float((np.asarray(got_bits) != np.asarray(ref_bits)).mean())


def bf16_ulp_diff(a_bits, b_bits):
    """Distance in bf16 ulps between two bit-pattern arrays (sign-magnitude aware)."""
    def key(x):
        x = x.astype(np.int32)
        return np.where(x & 0x8000, -(x & 0x7fff), x & 0x7fff)
    return np.abs(key(np.asarray(a_bits)) - key(np.asarray(b_bits)))


def int4_bit_pos(e):
    """Bit position of the low bit of element e of a packed word (include/qarl.h)."""
    return 3 + 4 * (e >> 1) + 16 * (e & 1) if e < 6 else (15 if e == 6 else 31)


def unblock_int4(codes, E, N, K):
    """Packed W4A16 codes as the library stores them (1 KiB blocks of 16 rows x 128 k, the elements of a
    word at the bit positions include/qarl.h lists, element 7 wrapping around the word) -> the oracle's
    packing: row-major words [E, N, K/8], element i of a word in nibble i.  Pure index permutation of
    words and bits."""
    w = np.ascontiguousarray(codes.detach().cpu().numpy()).view(np.uint32).reshape(E * N // 16, K // 128, 4, 16, 4)
    # [tile, g, q, c, i] -> [tile, c, g, q, i]
    w = np.ascontiguousarray(w.transpose(0, 3, 1, 2, 4)).reshape(E, N, K // 8)
    out = np.zeros_like(w)
    for el in range(8):
        p = int4_bit_pos(el)
        rot = (w >> np.uint32(p)) | (w << np.uint32((32 - p) % 32)) if p else w   # rotate right by p
        out |= (rot & np.uint32(15)) << np.uint32(4 * el)
    return out


def unblock_int4_torch(codes, E, N, K):
    """unblock_int4 with torch ops on the tensor's own device (int32 words in, int32 words out, same index
    permutation of words and bits): for comparisons over many whole layers."""
    w = codes.contiguous().view(torch.int32).reshape(E * N // 16, K // 128, 4, 16, 4)
    w = w.permute(0, 3, 1, 2, 4).contiguous().reshape(E, N, K // 8)
    out = torch.zeros_like(w)
    for el in range(8):
        p = int4_bit_pos(el)
        if p == 0:
            rot = w
        else:   # rotate right by p on the 32-bit pattern (arithmetic shifts: mask the sign extension away)
            rot = ((w >> p) & ((1 << (32 - p)) - 1)) | (w << (32 - p))
        out |= (rot & 15) << (4 * el)
    return out
