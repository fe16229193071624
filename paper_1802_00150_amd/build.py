"""Compile the HIP sources under csrc/ into paper_1802_00150_amd/libamq.so for gfx950.

hipcc cross-compiles without a GPU.  Objects go to _build/ (not tracked); the shared library
stays in-tree next to this file so that it travels with the source tree.
"""
import concurrent.futures as cf
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(ROOT, "_build")
LIB = os.path.join(HERE, "libamq.so")

SOURCES = ["amq_api.hip", "amq_quantize.hip", "amq_gemm.hip", "amq_bmv.hip", "amq_mfma.hip", "amq_mfma4.hip", "amq_mfma4w.hip", "amq_lstm_seqg.hip", "amq_cells.hip", "amq_lm.hip", "amq_baselines.hip"]
# packed-fp32 instructions are disabled on purpose; -ffp-contract=off keeps single binary32
# operations single (the code-assignment comparison must round like the reference arithmetic).
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall",
               "-Wno-unused-command-line-argument"]


def _headers():
    hs = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    hs.append(os.path.join(ROOT, "include", "amq.h"))
    return hs


def _compile(src, force):
    obj = os.path.join(OBJ_DIR, os.path.splitext(src)[0] + ".o")
    path = os.path.join(CSRC, src)
    newest = max(os.path.getmtime(p) for p in [path, *_headers()])
    if not force and os.path.exists(obj) and os.path.getmtime(obj) >= newest:
        return obj
    subprocess.check_call(["hipcc", *HIPCC_FLAGS, "-c", path, "-o", obj])
    return obj


def build(force: bool = False, jobs: int = 4) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    with cf.ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda s: _compile(s, force), SOURCES))
    if force or not os.path.exists(LIB) or any(os.path.getmtime(o) > os.path.getmtime(LIB) for o in objs):
        tmp = LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", tmp])
        os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
