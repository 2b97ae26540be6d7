"""Build the C oracle into oracle/libssm_oracle.so with gcc (test infrastructure only)."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "ssm_oracle.c")
LIB = os.path.join(HERE, "libssm_oracle.so")


SAN_LIB = os.path.join(HERE, "libssm_oracle_san.so")


def sanitized() -> bool:
    """SSM_ORACLE_SANITIZE=1 in the environment: the oracle is built with AddressSanitizer and UBSan and that build
    is the one loaded (the process must then have the gcc sanitizer runtime preloaded; tests/test_sanitizers.py does)."""
    return os.environ.get("SSM_ORACLE_SANITIZE", "") == "1"


def build(force: bool = False) -> str:
    lib = SAN_LIB if sanitized() else LIB
    if not force and os.path.exists(lib) and os.path.getmtime(lib) >= os.path.getmtime(SRC):
        return lib
    # No -march=native: the library travels to a machine whose CPU may differ.
    # No -ffast-math: the oracle is the definition, evaluated in strict fp64.
    opt = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"] if sanitized() else ["-O2"]
    cmd = ["gcc"] + opt + ["-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
                           "-ffp-contract=off", SRC, "-o", lib + ".tmp", "-lm"]
    subprocess.run(cmd, check=True)
    os.replace(lib + ".tmp", lib)
    return lib


if __name__ == "__main__":
    print(build(force=True))
