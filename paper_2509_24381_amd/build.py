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


# Host code under AddressSanitizer and UndefinedBehaviorSanitizer (the device code is compiled as usual: sanitizers are
# for the host pass only, so each -fsanitize sits behind -Xarch_host).  The runtime is linked dynamically: a process that
# loads the library through ctypes must have the ASan runtime preloaded (see asan_runtime()).
SANITIZE_FLAGS = [
    "-O1", "-g", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
    "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer", "-shared-libsan",
]


def asan_runtime() -> str:
    """Path of the AddressSanitizer runtime that matches hipcc's clang (to be put in LD_PRELOAD)."""
    import glob
    hits = sorted(glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so"))
    if not hits:
        raise RuntimeError("no libclang_rt.asan-x86_64.so under /opt/rocm/lib/llvm")
    return hits[-1]


def build(verbose: bool = True, sanitize_host_to: str = "") -> str:
    """Cross-compiles csrc/ into librserve_prefill.so (no GPU needed) and returns its path.

    With `sanitize_host_to` the library is written to that path instead, its host code instrumented with ASan + UBSan
    (a checking build for the CPU tests; the in-tree library is left alone)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if sanitize_host_to:
        flags = [f for f in HIPCC_FLAGS if f != "-O3"] + SANITIZE_FLAGS
        cmd = [hipcc] + flags + SRCS + ["-o", sanitize_host_to]
        if verbose:
            print("[build]", " ".join(cmd), flush=True)
        proc = subprocess.run(cmd, capture_output=True, text=True)
        if proc.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + proc.stderr)
        return sanitize_host_to
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
