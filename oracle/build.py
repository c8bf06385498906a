"""Compile the C oracle into oracle/liblcrwmd_oracle.so with gcc (host only, no GPU code)."""
from __future__ import annotations

import pathlib
import subprocess

HERE = pathlib.Path(__file__).resolve().parent
SRC = HERE / "rwmd_oracle.c"
LIB = HERE / "liblcrwmd_oracle.so"


def build(force: bool = True) -> pathlib.Path:
    if not force and LIB.exists() and LIB.stat().st_mtime >= SRC.stat().st_mtime:
        return LIB
    # x86-64-v3 (AVX2) rather than -march=native: the library is built on one host and may be loaded on another;
    # contraction off, so the wider instruction set changes speed only, never a rounding
    cmd = ["gcc", "-std=c99", "-O3", "-march=x86-64-v3", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-o", str(LIB), str(SRC), "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
