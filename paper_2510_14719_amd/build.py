"""Build the gfx950 shared library ``libattn_fwd.so`` in-tree with hipcc.

``python -m paper_2510_14719_amd.build`` compiles every HIP source for gfx950
(hipcc cross-compiles; no GPU is needed) and links the C-ABI library next to
this file.  Nothing is built at import time or inside tests.

Every source is compiled to an object of its own (in parallel) under ``_build/``
and the objects are linked; an object is reused when it is newer than its source
and every header, and was made with the same flags (``force`` recompiles all).
"""
from __future__ import annotations

import hashlib
import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(HERE, "libattn_fwd.so")
OBJ_DIR = os.path.join(HERE, "_build")

SOURCES = ["attn_fwd_kernel.hip", "attn_fwd_pipe_kernel.hip", "attn_fwd_fp8_kernel.hip", "mfma_probe.hip", "attn_api.cpp",
           "gemm_nt_kernel.hip", "gemm_nt_fp8_kernel.hip", "gemm_api.cpp"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed-fp32 VALU forms are kept out of every kernel of this library
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    log = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + log)
    if verbose and log.strip():
        print(log)


def _text_with_includes(path: str, seen=None) -> str:
    """The text of a source and of every header of this library it includes (directly or not)."""
    seen = set() if seen is None else seen
    if path in seen or not os.path.exists(path):
        return ""
    seen.add(path)
    text = open(path).read()
    for name in re.findall(r'#include\s+"([^"]+)"', text):
        for d in (CSRC, INCLUDE):
            text += _text_with_includes(os.path.join(d, name), seen)
    return text


def build(extra_defines=(), out: str = LIB, verbose: bool = False, force: bool = False, jobs: int = 8) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    base = [*HIPCC_FLAGS, "-I", INCLUDE, "-I", CSRC]
    headers = [os.path.join(d, f) for d in (CSRC, INCLUDE) for f in os.listdir(d) if f.endswith((".h", ".inc"))]
    newest_header = max(os.path.getmtime(h) for h in headers)

    def compile_one(src):
        path = os.path.join(CSRC, src)
        # a define only matters to the sources that mention its macro: the others share their objects with the
        # default build (a sweep variant then recompiles one or two files, not the library)
        text = _text_with_includes(path)
        flags = base + ["-D%s" % d for d in extra_defines if re.search(r"\b%s\b" % re.escape(d.split("=")[0]), text)]
        tag = hashlib.sha1(" ".join([hipcc] + flags).encode()).hexdigest()[:12]
        odir = os.path.join(OBJ_DIR, tag)
        os.makedirs(odir, exist_ok=True)
        obj = os.path.join(odir, src + ".o")
        if not force and os.path.exists(obj) and os.path.getmtime(obj) > max(os.path.getmtime(path), newest_header):
            return obj
        tmp = obj + ".tmp.%d.%d" % (os.getpid(), abs(hash(out)) % 100000)
        _run([hipcc, *flags, "-x", "hip", "-c", path, "-o", tmp], verbose)
        os.replace(tmp, obj)
        return obj

    # the assembly loop of the 64-rows-per-wave attention kernel is generated text: refresh it when its generator is newer
    gen, inc = os.path.join(CSRC, "gen_attn_mb2_loop.py"), os.path.join(CSRC, "attn_mb2_loop.inc")
    if not os.path.exists(inc) or os.path.getmtime(inc) < os.path.getmtime(gen):
        _run([sys.executable, gen, inc], verbose)

    with ThreadPoolExecutor(max_workers=max(1, jobs)) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    tmp = out + ".tmp.%d" % os.getpid()
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", tmp], verbose)
    os.replace(tmp, out)
    return out


if __name__ == "__main__":
    build(extra_defines=[a for a in sys.argv[1:] if a != "--force"], verbose=True, force="--force" in sys.argv[1:])
    print("built", LIB)
