"""Seeded synthetic inputs shaped like the Qwen3-30B-A3B MoE workloads.

This module only draws random tensors (torch generators) and names the workload shapes.
It holds none of the method's arithmetic, so both the HIP path's tests and the CPU oracle
may take their inputs from it.  bf16 tensors are returned as torch tensors; `bits()` gives
the raw uint16 patterns as numpy for the oracle.
"""
import math

import numpy as np
import torch

# Qwen3-30B-A3B expert shapes: hidden H, experts E, top-k, expert intermediate I, vocab V.
H, E, TOPK, I, V, LAYERS = 2048, 128, 8, 768, 151936, 48
GROUP = 128


def _gen(seed, device):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def normal_bf16(shape, std, seed, device="cpu", mean=0.0):
    """bf16 tensor ~ N(mean, std) drawn in fp32 and rounded once to bf16."""
    g = _gen(seed, device)
    x = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
    if std != 1.0:
        x.mul_(std)
    if mean != 0.0:
        x.add_(mean)
    return x.to(torch.bfloat16)


def bits(t):
    """Raw bit patterns of a bf16 / int tensor as a numpy array (uint16 for bf16)."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    if t.dtype in (torch.float8_e4m3fn,):
        return t.view(torch.uint8).numpy()
    return t.numpy()


def from_bits(a, device="cpu"):
    """numpy uint16 bit patterns -> torch bf16 tensor."""
    a = np.ascontiguousarray(a, dtype=np.uint16)
    return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).to(device)


def router_logits(T, n_experts, seed, device="cpu", zipf_s=0.0):
    """bf16 router logits ~ N(0,1); with zipf_s > 0 a per-expert bias -s*ln(rank) is added
    in fp32 before the bf16 rounding, ranks being a seeded permutation of 1..E (the log of a
    Zipf(s) popularity), to skew the expert load."""
    g = _gen(seed, device)
    x = torch.randn((T, n_experts), generator=g, device=device, dtype=torch.float32)
    if zipf_s > 0.0:
        gp = _gen(seed + 7919, "cpu")
        rank = torch.randperm(n_experts, generator=gp).to(torch.float32) + 1.0
        x += (-zipf_s * torch.log(rank)).to(device)
    return x.to(torch.bfloat16)


def targets(T, vocab, seed, device="cpu"):
    g = _gen(seed, device)
    return torch.randint(0, vocab, (T,), generator=g, device=device, dtype=torch.int32)


def expert_weights(n_experts, hidden, inter, seed, device="cpu", std=0.02):
    """(gate_up [E, 2I, H], down [E, H, I]) bf16 ~ N(0, std)."""
    gu = normal_bf16((n_experts, 2 * inter, hidden), std, seed, device)
    dn = normal_bf16((n_experts, hidden, inter), std, seed + 1, device)
    return gu, dn


def perturb(w, std, seed):
    """Simulated optimizer update: bf16(float(w) + N(0, std))."""
    g = _gen(seed, w.device)
    n = torch.randn(w.shape, generator=g, device=w.device, dtype=torch.float32) * std
    return (w.float() + n).to(torch.bfloat16)


# The five workloads (sizes only; tensors are drawn by the callers with the seeds below).
CONFIGS = {
    "dense_w4a16": dict(M=16, N=768, K=2048, seed=0),
    "moe_decode_w4a16": dict(T=256, seed=1),
    "moe_prefill_w4a16": dict(T=16384, seqs=8, seq_len=2048, zipf_s=1.1, seed=2),
    "moe_fp8": dict(T=(256, 8192), seed=3),
    "stack48_requant_decode": dict(T=512, layers=48, noise_std=1e-4, seed=4),
}


def algorithmic_bytes_moe_w4a16(T, n_experts=E, hidden=H, inter=I, topk=TOPK):
    """Bytes one MoE layer must move at W4A16 g128: packed codes + bf16 scales of every
    expert once, x read, a written and read, out written."""
    per_expert = 3 * inter * hidden
    wbytes = n_experts * (per_expert // 2 + per_expert // GROUP * 2)
    act = T * hidden * 2 + 2 * T * topk * inter * 2 + T * hidden * 2
    return wbytes, act


def flops_moe(T, hidden=H, inter=I, topk=TOPK):
    return 2 * T * topk * 3 * inter * hidden
