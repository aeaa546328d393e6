"""Build the gfx950 shared library ``libattn_fwd.so`` in-tree with hipcc.

``python -m paper_2510_14719_amd.build`` compiles every HIP source for gfx950
(hipcc cross-compiles; no GPU is needed) and links the C-ABI library next to
this file.  Nothing is built at import time or inside tests.
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(HERE, "libattn_fwd.so")

SOURCES = ["attn_fwd_kernel.hip", "attn_fwd_fp8_kernel.hip", "mfma_probe.hip", "attn_api.cpp", "gemm_nt_kernel.hip", "gemm_nt_fp8_kernel.hip", "gemm_api.cpp"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed-fp32 VALU forms are kept out of every kernel of this library
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def build(extra_defines=(), out: str = LIB, verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, "-I", INCLUDE, "-I", CSRC]
    cmd += ["-D%s" % d for d in extra_defines]
    cmd += ["-x", "hip"] + [os.path.join(CSRC, s) for s in SOURCES]
    tmp = out + ".tmp.%d" % os.getpid()
    cmd += ["-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    log = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + log)
    if verbose and log.strip():
        print(log)
    os.replace(tmp, out)
    return out


if __name__ == "__main__":
    build(extra_defines=sys.argv[1:], verbose=True)
    print("built", LIB)
