"""Compile the HIP library in-tree for gfx950: `python -m paper_2509_24381_amd.build`."""
from __future__ import annotations

import os
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
SRCS = [os.path.join(PKG_DIR, "csrc", "rserve_prefill.hip"),   # kernels + the prefill ABI
        os.path.join(PKG_DIR, "csrc", "rserve_sched.cpp")]     # host-only scheduler / tracker ABI
LIB = os.path.join(PKG_DIR, "librserve_prefill.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
    # keep the compiler from forming packed fp32 VALU ops
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def build(verbose: bool = True) -> str:
    """Cross-compiles csrc/ into librserve_prefill.so (no GPU needed) and returns its path."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + SRCS + ["-o", LIB + ".tmp"]
    if verbose:
        print("[build]", " ".join(cmd), flush=True)
    proc = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in proc.stderr.splitlines() if noise not in l)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err, file=sys.stderr)
    os.replace(LIB + ".tmp", LIB)
    return LIB


if __name__ == "__main__":
    print(build())
