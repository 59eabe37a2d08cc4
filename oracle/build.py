"""Builds the CPU oracle's shared libraries with g++ (no GPU toolchain involved).

    python -m oracle.build

Two builds of the same source: fp32 accumulation (`liboracle.so`, the oracle)
and double accumulation (`liboracle_f64.so`, used only to bound the oracle's own
rounding).  No fast-math, no FMA contraction: results are run-to-run identical.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "fi_oracle.cpp")
FLAGS = ["-O3", "-march=x86-64-v3", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared", "-std=c++17", "-Wall"]


def build(force: bool = True) -> None:
    for name, extra in (("liboracle.so", []), ("liboracle_f64.so", ["-DORC_ACC=double"])):
        out = os.path.join(HERE, name)
        if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(SRC):
            continue
        subprocess.check_call(["g++", *FLAGS, *extra, SRC, "-o", out])


if __name__ == "__main__":
    build()
    print("oracle built")
