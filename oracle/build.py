"""Compile the CPU oracle (test infrastructure) into two shared objects:
liborc64.so (double arithmetic, the reference) and liborc32.so (float)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "specbound_oracle.c")
FLAGS = ["-O2", "-march=x86-64-v3", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared",
         "-std=c11", "-Wall", "-Wextra", "-Wno-unused-parameter"]


def lib_path(bits: int) -> str:
    return os.path.join(HERE, f"liborc{bits}.so")


def build(force: bool = True) -> None:
    for bits, defs in ((64, []), (32, ["-DORC_F32"])):
        out = lib_path(bits)
        if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(SRC):
            continue
        subprocess.check_call(["gcc", *FLAGS, *defs, SRC, "-o", out, "-lm"])


if __name__ == "__main__":
    build()
    print("built", lib_path(64), lib_path(32))
