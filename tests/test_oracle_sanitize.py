"""The oracle's C under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only).

Builds oracle/liboracle_san.so (`python oracle/build.py --sanitize`) and runs a slice of the oracle's own pins
against it in a child process with libasan preloaded: an out-of-bounds index, a use of uninitialised stack
through a wrong length, signed overflow or a misaligned access anywhere in the oracle's loops ends that process
with a report instead of a quietly wrong number.
"""
import os
import subprocess
import sys

import pytest

from oracle import build as oracle_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PINS = ["tests/test_oracle_scores.py", "tests/test_oracle_prune.py", "tests/test_oracle_evict.py",
        "tests/test_oracle_evict_ex.py", "tests/test_oracle_attention.py", "tests/test_oracle_loop.py",
        "tests/test_oracle_shared.py"]


@pytest.mark.skipif("PE_ORACLE_SANITIZE" in os.environ or "PE_ORACLE_LIB" in os.environ,
                    reason="already inside a child run")
def test_oracle_pins_under_asan_ubsan():
    lib = oracle_build.build(force=True, sanitize=True)
    assert os.path.exists(lib)
    asan = oracle_build.asan_runtime()
    if not os.path.exists(asan):
        pytest.skip("gcc's libasan.so not found")
    preload = asan + (":" + os.environ["LD_PRELOAD"] if os.environ.get("LD_PRELOAD") else "")   # keep what is there
    env = dict(os.environ, PE_ORACLE_SANITIZE="1", LD_PRELOAD=preload, OMP_NUM_THREADS="2",
               ASAN_OPTIONS="detect_leaks=0:abort_on_error=0:exitcode=97",
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    r = subprocess.run([sys.executable, "-m", "pytest"] + PINS + ["-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider"],
                       cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    tail = "\n".join(r.stdout.splitlines()[-40:])
    assert r.returncode == 0, tail
    assert "passed" in tail and "runtime error" not in r.stdout and "AddressSanitizer" not in r.stdout, tail
