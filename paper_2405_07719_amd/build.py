"""Build libusp.so (the C-ABI library) in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libusp.so")
SOURCES = ["usp_api.cpp", "layout_a2a.hip", "lse_merge.hip", "block_attn_fwd.hip", "block_attn_bwd.hip"]
# measurement aid for bench.py only (matrix-core calibration loops): a library of its own, not part of the product
CALIB_LIB = os.path.join(PKG, "libusp_calib.so")
CALIB_SOURCES = ["calib_mfma.hip"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-fvisibility=hidden",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # no packed-fp32 VALU forms
    "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
    "-DUSP_BUILDING=1",
]


def _compile(sources, lib, verbose, extra) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    srcs = [os.path.join(CSRC, s) for s in sources]
    cmd = [hipcc, *FLAGS, *extra, "-x", "hip", *srcs, "-o", lib]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l and "is not a recognized feature" not in l)
    if verbose and out.strip():
        print(out)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    return lib


def build(verbose: bool = True, extra=()) -> str:
    _compile(CALIB_SOURCES, CALIB_LIB, verbose, extra)
    return _compile(SOURCES, LIB, verbose, extra)


if __name__ == "__main__":
    build(extra=sys.argv[1:])
