"""Compile the CPU oracle (plain C, OpenMP) into oracle/liboracle.so with gcc."""
from __future__ import annotations

import pathlib
import subprocess

HERE = pathlib.Path(__file__).resolve().parent
LIB = HERE / "liboracle.so"


def build(force: bool = True) -> pathlib.Path:
    src = HERE / "xp_oracle.c"
    hdr = HERE / "xp_oracle.h"
    if not force and LIB.exists() and LIB.stat().st_mtime >= max(src.stat().st_mtime, hdr.stat().st_mtime):
        return LIB
    cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-o", str(LIB), str(src), "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


def build_selftest(out_dir) -> pathlib.Path:
    """The oracle and its closed-form self-test (selftest.c) as one executable under AddressSanitizer and
    UndefinedBehaviorSanitizer: running it stops at the first access outside an operand buffer."""
    exe = pathlib.Path(out_dir) / "oracle_selftest"
    cmd = ["gcc", "-std=c11", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-Wall", "-Wextra", "-o", str(exe), str(HERE / "selftest.c"), str(HERE / "xp_oracle.c"), "-lm"]
    subprocess.run(cmd, check=True)
    return exe


if __name__ == "__main__":
    print(build())
