"""Compile the C part of the CPU oracle with gcc (test infrastructure; not part of the product path)."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(_HERE, "gate_order.c")
LIB = os.path.join(_HERE, "liboracle_gate.so")


def build(force: bool = False) -> str:
    """Build liboracle_gate.so next to its source; returns the library path."""
    if force or not os.path.exists(LIB) or os.path.getmtime(LIB) < os.path.getmtime(SRC):
        # -ffp-contract=off: the only fused operation must be the explicit fmaf() call.
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math",
               "-o", LIB, SRC, "-lm"]
        subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
