"""qarl_token_logprob_static (the entry point for callers that cannot allocate: partials in the library's own
file-scope device array) against qarl_token_logprob with a caller workspace, through the C ABI: two calls in a
row, the second on a smaller input, so that the array still holds the first call's partials when the second runs."""
import numpy as np
import pytest
import torch

from paper_2604_07853_amd import synth
from gpu_util import np_bits

pytestmark = pytest.mark.gpu

TOL_LP = 1e-4


def test_static_scratch_logprob_matches_workspace_variant():
    from paper_2604_07853_amd import binding as q
    import oracle
    q.lib()
    H, V = 256, 20000
    w = synth.normal_bf16((V, H), 0.3, seed=11).cuda()
    for T, seed in ((700, 12), (37, 13)):                   # the second call is smaller than the first
        h = synth.normal_bf16((T, H), 1.0, seed=seed).cuda()
        tg = synth.targets(T, V, seed=seed + 10).cuda()
        want = q.qarl_token_logprob(h, w, tg)["logprob"]
        got = torch.full((T,), float("nan"), dtype=torch.float32, device="cuda")
        q.qarl_token_logprob_static(h, w, tg, got)
        torch.cuda.synchronize()
        assert torch.equal(got, want), T                    # same kernels, same partial layout: same bits
        rows = np.arange(T) if T <= 64 else np.linspace(0, T - 1, 48).astype(np.int64)
        ref = oracle.token_logprob(np_bits(h)[rows], np_bits(w), tg.cpu().numpy()[rows])
        assert np.abs(got.cpu().numpy()[rows].astype(np.float64) - ref).max() <= TOL_LP
    # beyond the array's size the call refuses, with the limit in the message, and launches nothing
    assert q.qarl_token_logprob_static_limit() == 4 << 20
    Tbig = 4 * (4 << 20) // (4 * (2 * ((V + 255) // 256) + 1))
    hb = torch.zeros((Tbig, H), dtype=torch.bfloat16, device="cuda")
    tb = torch.zeros((Tbig,), dtype=torch.int32, device="cuda")
    ob = torch.empty((Tbig,), dtype=torch.float32, device="cuda")
    with pytest.raises(q.QarlError) as ei:
        q.qarl_token_logprob_static(hb, w, tb, ob)
    assert ei.value.status == q.QARL_ERR_WORKSPACE and "built-in scratch" in str(ei.value)
