"""The C-ABI library loads and exports every symbol include/qarl.h declares (no GPU needed)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_all_declared_symbols():
    from paper_2604_07853_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):
        build.build()
    lib = ctypes.CDLL(binding.LIB_PATH)
    header = open(os.path.join(ROOT, "include", "qarl.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(qarl_[a-z0-9_]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_workspace_queries_and_host_side_validation():
    from paper_2604_07853_amd import binding as q
    L = q.lib()
    d4 = q.qarl_qweight(q.QARL_W4A16_G128, 128, 2048, 768, 128, 16, 16)
    d8 = q.qarl_qweight(q.QARL_FP8_E4M3_CH, 128, 2048, 768, 0, 16, 16)
    by = ctypes.byref
    assert L.qarl_qgemm_workspace_bytes(by(d8), 2048, 2048, q.QARL_EPI_COMBINE) == 2048 * 2048 * 4
    assert L.qarl_qgemm_workspace_bytes(by(d8), 2048, 2048, q.QARL_EPI_NONE) == 0
    assert L.qarl_qgemm_workspace_bytes(by(d4), 2048, 2048, q.QARL_EPI_NONE) == 2048 * 6 * 4
    assert L.qarl_qgemm_workspace_bytes(by(d4), 2048, 2048, q.QARL_EPI_COMBINE) == 2048 * 2048 * 4 + 2048 * 6 * 4
    assert L.qarl_logprob_workspace_bytes(16384, 2048, 151936) == (2 * 594 + 1) * 16384 * 4
    # argument errors are reported before any launch, so they can be checked without a GPU
    d = q.qarl_qweight(q.QARL_W4A16_G128, 1, 32, 100, 128, 16, 16)
    assert L.qarl_quantize_weights(ctypes.c_void_p(16), ctypes.byref(d), None) == q.QARL_ERR_UNSUPPORTED
    assert b"K % 128" in L.qarl_last_error()
    d = q.qarl_qweight(q.QARL_W4A16_G128, 1, 32, 128, 64, 16, 16)
    assert L.qarl_quantize_weights(ctypes.c_void_p(16), ctypes.byref(d), None) == q.QARL_ERR_UNSUPPORTED
    d = q.qarl_qweight(q.QARL_W4A16_G128, 1, 32, 128, 128, 8, 16)
    assert L.qarl_quantize_weights(ctypes.c_void_p(16), ctypes.byref(d), None) == q.QARL_ERR_ALIGNMENT
    assert L.qarl_moe_route(None, 4, 100, 8, 1, None, None, None, None, None, None, None) == q.QARL_ERR_UNSUPPORTED
    assert L.qarl_moe_route(None, -1, 128, 8, 1, None, None, None, None, None, None, None) == q.QARL_ERR_INVALID_ARG
