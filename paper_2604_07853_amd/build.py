"""Compile the HIP library (gfx950) into paper_2604_07853_amd/libqarl.so with hipcc.

Every source becomes an object file under paper_2604_07853_amd/_build/ (compiled in parallel; an object is
reused when it is newer than its source and every header, unless force=True), then one link step.
"""
import os
import shutil
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libqarl.so")
SOURCES = ["api.hip", "quantize.hip", "route.hip", "qgemm_stream_fp8.hip", "qgemm_stream_w4.hip", "qgemm_tile.hip", "qgemm_backward.hip",
           "qgemm_tile_fp8.hip", "combine.hip", "logprob.hip", "tbpo.hip"]
# packed fp32 operations are switched off for all device code
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
         "-packed-fp32-ops", "-Wall"]
NOISE = "is not a recognized feature for this target"


def hipcc():
    return shutil.which("hipcc") or "/opt/rocm/bin/hipcc"


def _run(cmd):
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if NOISE not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed: %s\n%s" % (" ".join(cmd[-3:]), err))
    return err


def build(verbose=False, force=False, jobs=None):
    os.makedirs(OBJ, exist_ok=True)
    headers = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith((".hpp", ".h"))]
    headers.append(os.path.join(HERE, "..", "include", "qarl.h"))
    newest_header = max(os.path.getmtime(h) for h in headers)
    todo, objs = [], []
    for s in SOURCES:
        src, obj = os.path.join(CSRC, s), os.path.join(OBJ, s.replace(".hip", ".o"))
        objs.append(obj)
        if force or not os.path.exists(obj) or os.path.getmtime(obj) < max(os.path.getmtime(src), newest_header):
            todo.append([hipcc()] + FLAGS + ["-c", src, "-o", obj])
    jobs = jobs or min(8, os.cpu_count() or 1)
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        msgs = list(pool.map(_run, todo))
    if todo or not os.path.exists(LIB):
        msgs.append(_run([hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs))
    if verbose:
        for m in msgs:
            if m.strip():
                print(m)
    return LIB


if __name__ == "__main__":
    import sys
    print(build(verbose=True, force="--force" in sys.argv))
