"""Compile the CPU oracles into shared objects beside their sources (g++, no fast-math, no FMA contraction):
oracle/libbca_oracle.so (bucket-wise clip + Adam / LAMB) and oracle/liblbs_oracle.so (load-balancing simulation)."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "bca_oracle.cpp")
LIB = os.path.join(HERE, "libbca_oracle.so")
LBS_SRC = os.path.join(HERE, "lbs_oracle.cpp")
LBS_LIB = os.path.join(HERE, "liblbs_oracle.so")


def build(force: bool = True, src: str = SRC, out: str = LIB) -> str:
    if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(src):
        return out
    cmd = ["g++", "-O2", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math",
           "-Wall", "-Wextra", "-o", out, src]
    subprocess.run(cmd, check=True)
    return out


def build_lbs(force: bool = True, src: str = LBS_SRC, out: str = LBS_LIB) -> str:
    return build(force, src, out)


def build_all() -> None:
    build()
    build_lbs()


if __name__ == "__main__":
    print(build())
    print(build_lbs())
