"""Builds libpicospec.so (gfx950) in-tree with hipcc.  Run as ``python -m paper_2603_19133_amd.build``."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpicospec.so")
SOURCES = ["api.hip", "compress.hip", "verify.hip", "residual.hip", "downlink.hip", "wire.hip", "selfcheck.hip", "noalloc.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# packed-fp32 instructions are switched off (scalar fp32 code only); the compiler's rewrite of
# same-address LDS atomics into a wave-wide scan is switched off (the compress kernel issues one
# atomic per passing element on purpose: a few lanes each, no vector ALU work)
# (-Wno-unused-lambda-capture: two lambdas name a register they pass to inline assembly in their capture lists on purpose)
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-Wall", "-Wno-unused-lambda-capture",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-mllvm", "-amdgpu-atomic-optimizer-strategy=None"]


def build(verbose: bool = False, extra: list[str] | None = None, out: str | None = None) -> str:
    """Compiles the library (to `out` instead of the in-tree libpicospec.so, if given)."""
    out = out or LIB
    cmd = [HIPCC, *FLAGS, *(extra or []), "-o", out, *[os.path.join(CSRC, s) for s in SOURCES]]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed:\n{err}")
    if verbose and err.strip():
        print(err, file=sys.stderr)
    return out


if __name__ == "__main__":
    print(build(verbose=True))
