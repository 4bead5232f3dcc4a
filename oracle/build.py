"""Compile the C oracle (test infrastructure) into oracle/liboracle.so with gcc.

    python oracle/build.py              the library the tests load
    python oracle/build.py --sanitize   a second library, oracle/liboracle_san.so, built with
                                        -fsanitize=address,undefined (CPU only); a process that is to load it
                                        needs libasan preloaded (see tests/test_oracle_sanitize.py)
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRCS = [os.path.join(HERE, "pe_oracle.c"), os.path.join(HERE, "pe_oracle_shared.c")]
LIB = os.path.join(HERE, "liboracle.so")
LIB_SAN = os.path.join(HERE, "liboracle_san.so")


def build(force: bool = True, sanitize: bool = False) -> str:
    lib = LIB_SAN if sanitize else LIB
    if not force and os.path.exists(lib) and os.path.getmtime(lib) >= max(os.path.getmtime(f) for f in SRCS):
        return lib
    tmp = lib + ".tmp.%d" % os.getpid()
    flags = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
             "-fno-omit-frame-pointer"] if sanitize else ["-O2"]
    cmd = ["gcc", "-std=c11"] + flags + ["-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
                                         "-ffp-contract=off", "-o", tmp] + SRCS + ["-lm"]
    subprocess.run(cmd, check=True)
    os.replace(tmp, lib)
    return lib


def asan_runtime() -> str:
    """Path of gcc's libasan.so (to be preloaded by a process that loads the sanitized oracle)."""
    out = subprocess.run(["gcc", "-print-file-name=libasan.so"], check=True, stdout=subprocess.PIPE, text=True)
    return os.path.realpath(out.stdout.strip())


if __name__ == "__main__":
    print(build(sanitize="--sanitize" in sys.argv))
