"""Builds libtq.so (host encoder + validator + gfx950 kernels) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libtq.so")
SOURCES = ["tq_encode.cpp", "tq_blob.cpp", "tq_device.hip", "tq_listing.hip"]
HEADERS = ["tq_format.h", "tq_kernels_common.h", "tq_kernel_dot.h", "tq_strip_decode.h", "tq_kernel_ring.h", "tq_kernel_strip.h",
           os.path.join("..", "..", "include", "tq.h")]


def hipcc_command(out: str):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    return [
        hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-pthread",
        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # keep hipcc from emitting packed fp32 ops
        "-Wall", "-Wno-unused-command-line-argument",
        *[os.path.join(CSRC, s) for s in SOURCES], "-o", out,
    ]


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(os.path.join(CSRC, f)) > t for f in SOURCES + HEADERS)


def build_libtq(force: bool = True, verbose: bool = False) -> str:
    if not force and not is_stale():
        return LIB
    tmp = LIB + f".tmp{os.getpid()}"
    cmd = hipcc_command(tmp)
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed ({res.returncode}):\n{err}")
    if verbose and err.strip():
        print(err, file=sys.stderr)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build_libtq(force=True, verbose=True))
