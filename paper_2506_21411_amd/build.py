"""Builds libdchag.so (HIP, gfx950) in-tree with hipcc.  `python -m paper_2506_21411_amd.build`."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdchag.so")
SOURCES = [os.path.join(CSRC, "dchag_api.hip")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # no packed-fp32 code generation
    "-Wall", "-Wno-unused-function",
]


def build(verbose: bool = True, out: str = LIB, defines=()) -> str:
    """Compiles the library to `out` (default: the in-tree libdchag.so); `defines` are extra -D macros (the timing
    probes of the GEMM core, which must never be built into the in-tree library)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if defines and os.path.abspath(out) == os.path.abspath(LIB):
        raise ValueError("a build with extra defines needs its own --out file")
    cmd = [hipcc] + HIPCC_FLAGS + ["-D" + d for d in defines] + ["-o", out] + SOURCES
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if verbose and out.strip():
        print(out, flush=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    return out


if __name__ == "__main__":
    import argparse
    ap = argparse.ArgumentParser()
    ap.add_argument("--out", default=LIB)
    ap.add_argument("--define", action="append", default=[], help="extra macro, e.g. DCHAG_GEMM_PROBE=8 (needs --out)")
    a = ap.parse_args()
    build(out=a.out, defines=a.define)
    sys.exit(0)
