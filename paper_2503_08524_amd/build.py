"""Build the D^3 HIP library for gfx950: hipcc cross-compiles every source under
csrc/ into paper_2503_08524_amd/libd3.so (no GPU needed to build)."""
from __future__ import annotations

import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libd3.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

BUILD_DIR = os.path.join(HERE, "_build")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # scalar fp32 only
    "-Wall", "-Wno-unused-function",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")) + glob.glob(os.path.join(CSRC, "*.cpp")))


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    deps = sources() + glob.glob(os.path.join(CSRC, "*.h")) + [os.path.join(HERE, "..", "include", "d3.h")]
    return max(os.path.getmtime(p) for p in deps) > os.path.getmtime(LIB)


def build(force: bool = True, verbose: bool = False) -> str:
    if not force and not is_stale():
        return LIB
    extra = os.environ.get("D3_BUILD_DEFINES", "").split()          # e.g. "-DD3_GEMV_DEPTH=4" for tuning experiments
    out_path = os.environ.get("D3_BUILD_OUT", LIB)
    # one object per source, compiled side by side, then one link
    os.makedirs(BUILD_DIR, exist_ok=True)
    tag = os.path.splitext(os.path.basename(out_path))[0]

    def compile_one(src):
        obj = os.path.join(BUILD_DIR, tag + "_" + os.path.basename(src) + ".o")
        r = subprocess.run([HIPCC] + FLAGS + extra + ["-x", "hip", "-c", src, "-o", obj], capture_output=True, text=True)
        return obj, r

    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as pool:
        results = list(pool.map(compile_one, sources()))
    out = "\n".join(r.stdout + r.stderr for _, r in results)
    if any(r.returncode != 0 for _, r in results):
        raise RuntimeError("hipcc failed:\n" + out)
    res = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC"] + [o for o, _ in results] + ["-o", out_path],
                         capture_output=True, text=True)
    out = "\n".join(ln for ln in (out + res.stdout + res.stderr).splitlines() if "packed-fp32-ops" not in ln)
    if res.returncode != 0:
        raise RuntimeError("hipcc link failed:\n" + out)
    if verbose and out.strip():
        print(out, file=sys.stderr)
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose=True))
