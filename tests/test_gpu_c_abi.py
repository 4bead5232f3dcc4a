"""The C ABI is usable from plain C: a C program (tests/c_abi/pe_c_smoke.c, built by the package's build step
with gcc against libpe.so and the HIP runtime) allocates device memory itself, calls the library, and checks
closed-form results on the host."""
import os
import subprocess

import pytest

from paper_2509_04377_amd import build as pe_build

pytestmark = pytest.mark.gpu


def test_plain_c_caller():
    print("case plain C caller", flush=True)
    if not os.path.exists(pe_build.C_SMOKE_BIN):      # normally built in-tree beforehand; gcc only, about a second
        pe_build.build_c_smoke()
    r = subprocess.run([pe_build.C_SMOKE_BIN], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, (r.returncode, r.stdout, r.stderr)
    assert "pe_c_smoke ok" in r.stdout
