"""Compile the CPU oracle (plain C) into oracle/libamq_oracle.so with gcc.

Test infrastructure only; the GPU library never links or loads this.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "amq_oracle.c")
LIB = os.path.join(HERE, "libamq_oracle.so")

# -ffp-contract=off: single binary32 operations must stay single operations.
FLAGS = ["-O3", "-std=gnu99", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-shared", "-fPIC",
         "-Wall", "-Wextra"]


# The same source under AddressSanitizer and UndefinedBehaviorSanitizer (a second library, used only by
# the sanitizer test: a process that loads it must have the sanitizer run-time preloaded).
LIB_SANITIZED = os.path.join(HERE, "libamq_oracle_san.so")
SANITIZE_FLAGS = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
                  "-fno-sanitize-recover=undefined"]


def build(force: bool = False, sanitize: bool = False) -> str:
    lib = LIB_SANITIZED if sanitize else LIB
    if not force and os.path.exists(lib) and os.path.getmtime(lib) >= os.path.getmtime(SRC):
        return lib
    flags = [f for f in FLAGS if f != "-O3"] + SANITIZE_FLAGS if sanitize else FLAGS
    tmp = lib + ".tmp.%d" % os.getpid()
    subprocess.check_call(["gcc", *flags, SRC, "-o", tmp, "-lm"])
    os.replace(tmp, lib)
    return lib


def sanitizer_runtime() -> str:
    """Path of gcc's AddressSanitizer run-time (to preload into a process that loads the sanitized library)."""
    return subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()


if __name__ == "__main__":
    print(build(force="--force" in sys.argv, sanitize="--sanitize" in sys.argv))
