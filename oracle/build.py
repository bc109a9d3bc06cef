"""Compile the C oracle (TEST INFRASTRUCTURE) into two shared libraries:
libd3oracle_f64.so (double arithmetic, the parity reference) and
libd3oracle_f32.so (float arithmetic).  Plain gcc, no fast-math, so every sum
keeps its written order."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
VARIANTS = {"f64": "double", "f32": "float"}


def lib_path(variant: str) -> str:
    return os.path.join(HERE, f"libd3oracle_{variant}.so")


def build(force: bool = False) -> None:
    src = os.path.join(HERE, "d3_oracle.c")
    hdr = os.path.join(HERE, "d3_oracle.h")
    newest = max(os.path.getmtime(src), os.path.getmtime(hdr))
    for variant, ctype in VARIANTS.items():
        out = lib_path(variant)
        if not force and os.path.exists(out) and os.path.getmtime(out) >= newest:
            continue
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-Wall", "-Wno-maybe-uninitialized", f"-DD3O_REAL={ctype}", "-o", out, src, "-lm"]
        subprocess.run(cmd, check=True)


if __name__ == "__main__":
    build(force=True)
    print("built", [lib_path(v) for v in VARIANTS])
