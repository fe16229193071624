"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer: the oracle's own pin tests
are run again in a child process against a sanitized build of oracle/amq_oracle.c (the sanitizer
run-time preloaded), so that an out-of-bounds access, a use of uninitialised stack, a signed overflow
or a misaligned access in the code every parity claim rests on fails a test."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

PIN_TESTS = ["tests/test_oracle_quantizer.py", "tests/test_oracle_products.py", "tests/test_oracle_baselines.py",
             "tests/test_oracle_ternary.py", "tests/test_oracle_lm.py"]


def test_oracle_pins_hold_under_address_and_undefined_behaviour_sanitizers():
    from oracle import build
    build.build(sanitize=True)
    env = dict(os.environ)
    env.update({"AMQ_ORACLE_SANITIZE": "1", "LD_PRELOAD": build.sanitizer_runtime(),
                # python itself leaks by design and is not built for the link-order check
                "ASAN_OPTIONS": "detect_leaks=0:verify_asan_link_order=0:abort_on_error=1",
                "UBSAN_OPTIONS": "halt_on_error=1:print_stacktrace=1", "OMP_NUM_THREADS": "4"})
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider",
                        *PIN_TESTS], cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True,
                       timeout=1500)
    tail = r.stdout[-3000:]
    assert r.returncode == 0, tail
    assert "ERROR: AddressSanitizer" not in r.stdout and "runtime error:" not in r.stdout, tail
    assert " passed" in tail
