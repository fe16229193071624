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
# profiling build: the same sources with -DAMQ_PHASE_TIMING (in-kernel phase timers and the extra entry
# point amq_debug_set_phase_buffer); loaded instead of libamq.so when AMQ_LIBRARY names it
LIB_PHASES = os.path.join(HERE, "libamq_phases.so")

SOURCES = ["amq_api.hip", "amq_quantize.hip", "amq_gemm.hip", "amq_bmv.hip", "amq_mfma.hip", "amq_mfma4.hip", "amq_mfma4w.hip", "amq_step.hip", "amq_lstm_seqg.hip", "amq_cells.hip", "amq_lm.hip", "amq_baselines.hip"]
# packed-fp32 instructions are disabled on purpose; -ffp-contract=off keeps single binary32
# operations single (the code-assignment comparison must round like the reference arithmetic).
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall",
               "-Wno-unused-command-line-argument"]


def _headers():
    hs = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    hs.append(os.path.join(ROOT, "include", "amq.h"))
    return hs


def _compile(src, force, obj_dir, extra):
    obj = os.path.join(obj_dir, os.path.splitext(src)[0] + ".o")
    path = os.path.join(CSRC, src)
    newest = max(os.path.getmtime(p) for p in [path, *_headers()])
    if not force and os.path.exists(obj) and os.path.getmtime(obj) >= newest:
        return obj
    # (the host pass of hipcc warns that it does not know the packed-fp32 feature; harmless)
    r = subprocess.run(["hipcc", *HIPCC_FLAGS, *extra, "-c", path, "-o", obj], stderr=subprocess.PIPE, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if err.strip():
        sys.stderr.write(err + "\n")
    if r.returncode != 0:
        raise subprocess.CalledProcessError(r.returncode, r.args)
    return obj


def build(force: bool = False, jobs: int = 4, phase_timing: bool = False) -> str:
    lib = LIB_PHASES if phase_timing else LIB
    obj_dir = os.path.join(OBJ_DIR, "phases") if phase_timing else OBJ_DIR
    extra = ["-DAMQ_PHASE_TIMING"] if phase_timing else []
    os.makedirs(obj_dir, exist_ok=True)
    with cf.ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda s: _compile(s, force, obj_dir, extra), SOURCES))
    if force or not os.path.exists(lib) or any(os.path.getmtime(o) > os.path.getmtime(lib) for o in objs):
        tmp = lib + ".tmp.%d" % os.getpid()
        subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", tmp])
        os.replace(tmp, lib)
    return lib


if __name__ == "__main__":
    print(build(force="--force" in sys.argv, phase_timing="--phase-timing" in sys.argv))
