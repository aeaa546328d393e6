"""Sweep of the kernels' schedule parameters (the counterpart of the paper's study of the aref depth D
and the MMA issue depth P, Section 5.5, and of its ablation, Section 5.6).

The knobs are compile-time constants of the HIP sources, so a sweep is two steps:

    python -m paper_2510_14719_amd.sweep build [--op attn|gemm|...] # anywhere hipcc runs (no GPU needed)
    python -m paper_2510_14719_amd.sweep run   [--op attn|gemm|...] ...  # on the GPU: times every built variant

``build`` compiles one shared library per grid point into ``sweep_variants/`` next to this file; ``run``
loads each through ctypes, checks a few sampled outputs of every variant against the default build's
output (bit-identical or within rounding of it -- a variant that computes something else is reported, not
timed) and prints one JSON line per variant plus a table.

What the axes stand for on gfx950:
  attention  ATTN_FWIN          LDS fragments requested ahead of their MFMA inside a burst (the paper's P)
             ATTN_COPY_GROUP    which waves produce (issue the global -> LDS copies): 0 all, 2 group A, 1 group B
             ATTN_SUMCHAINS     independent row-sum chains of the softmax
             ATTN_PERSISTENT    persistent launch with the static tile schedule (causal d = 128)
  attn_fp8   ATTN8_FWIN         the same for the 8-bit-float kernel
             ATTN8_INTERLEAVE   softmax of tile j issued in slices between the MFMAs of U_{j-1} and T_{j+1} (1: the
                                in-wave software pipeline of the paper's Algorithm 1) or after them as one block (0)
             ATTN8_STAGES       depth of the LDS ring (the paper's D): copies run STAGES - 2 tiles ahead
             ATTN8_COPIES_IN_PASS copies issued one by one behind MFMAs of the pass (1) or all right after the barrier (0)
  gemm       GEMM_STAGES        depth of the LDS ring (the paper's D): 4 or 5
             GEMM_CONFIG        0: chosen by K; 1: 8 waves x (128 x 64); 2: the same with paired copies (two stages
                                issued together so that both halves of a memory line are requested back to back);
                                3: 4 waves x (128 x 128); 4: the same with paired copies
             GEMM_TAIL_READS    LDS requests allowed in flight across the tile boundary
  gemm_fp8   GEMM8_STAGES, GEMM8_TAIL_READS, GEMM8_CONFIG   the same for the 8-bit-float kernel
             GEMM8_COPY_PHASE   copies behind the odd (1) or the even (0) MFMAs of a K tile
             GEMM8_CONFIG       0: chosen by K; 1: 8 waves x (128 x 64); 2: the same with paired copies (two stages
                                issued together so that both halves of a memory line are requested back to back);
                                3: 4 waves x (128 x 128); 4: the same with paired copies
"""
from __future__ import annotations

import argparse
import ctypes
import itertools
import json
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
VARIANT_DIR = os.path.join(HERE, "sweep_variants")

GRIDS = {
    "attn": {"ATTN_FWIN": [1, 2, 4, 8], "ATTN_COPY_GROUP": [0, 2, 1], "ATTN_SUMCHAINS": [2, 4]},
    "attn_causal": {"ATTN_PERSISTENT": [0, 1], "ATTN_FWIN": [2, 4]},
    "attn_fp8": {"ATTN8_FWIN": [1, 2, 3], "ATTN8_INTERLEAVE": [1, 0], "ATTN8_STAGES": [4, 8], "ATTN8_COPIES_IN_PASS": [1, 0]},
    "gemm": {"GEMM_CONFIG": [0, 1, 2, 3, 4], "GEMM_STAGES": [4, 5], "GEMM_TAIL_READS": [3, 0]},
    "gemm_fp8": {"GEMM8_CONFIG": [0, 1, 2, 3, 4], "GEMM8_STAGES": [4, 5], "GEMM8_TAIL_READS": [3, 0]},
}
DEFAULTS = {"ATTN8_FWIN": 2, "ATTN8_INTERLEAVE": 1, "ATTN8_STAGES": 4, "ATTN8_COPIES_IN_PASS": 1, "ATTN_FWIN": 2, "ATTN_COPY_GROUP": 0, "ATTN_SUMCHAINS": 4, "ATTN_PERSISTENT": 1,
            "GEMM_STAGES": 4, "GEMM_CONFIG": 0, "GEMM_TAIL_READS": 3,
            "GEMM8_STAGES": 4, "GEMM8_TAIL_READS": 3, "GEMM8_COPY_PHASE": 1, "GEMM8_CONFIG": 0}


def grid_points(op: str):
    """All combinations of the grid of ``op`` as dicts, the default point first."""
    g = GRIDS[op]
    keys = list(g)
    pts = [dict(zip(keys, vals)) for vals in itertools.product(*(g[k] for k in keys))]
    pts.sort(key=lambda p: (not all(p[k] == DEFAULTS[k] for k in keys), [p[k] for k in keys]))
    return pts


def variant_name(op: str, point: dict) -> str:
    return op + "__" + "__".join("%s-%s" % (k.split("_", 1)[1].lower(), point[k]) for k in sorted(point))


def variant_path(op: str, point: dict) -> str:
    return os.path.join(VARIANT_DIR, "lib%s.so" % variant_name(op, point))


def cmd_build(args) -> int:
    from concurrent.futures import ThreadPoolExecutor
    from . import build as lib_build
    os.makedirs(VARIANT_DIR, exist_ok=True)
    jobs = []
    for op in args.ops:
        for p in grid_points(op):
            jobs.append((["%s=%s" % kv for kv in p.items()], variant_path(op, p)))
    with ThreadPoolExecutor(max(1, args.jobs)) as ex:
        for out in ex.map(lambda j: lib_build.build(extra_defines=j[0], out=j[1]), jobs):
            print("built", os.path.relpath(out, HERE), flush=True)
    return 0


def _load(path):
    lib = ctypes.CDLL(path)
    vp, ci, cf = ctypes.c_void_p, ctypes.c_int, ctypes.c_float
    lib.attn_fwd.restype = ci
    lib.attn_fwd.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, cf, ci, vp, ci]
    lib.attn_fwd_fp8.restype = ci
    lib.attn_fwd_fp8.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, cf, ci, vp, ci]
    lib.gemm_nt.restype = ci
    lib.gemm_nt.argtypes = [vp, vp, vp, ci, ci, ci, vp, ci]
    lib.gemm_nt_fp8.restype = ci
    lib.gemm_nt_fp8.argtypes = [vp, vp, vp, ci, ci, ci, vp, ci]
    return lib


def cmd_run(args) -> int:
    import numpy as np
    import torch
    from . import binding, inputs as I
    if not torch.cuda.is_available():
        print("sweep run: no GPU visible", file=sys.stderr)
        return 3
    binding.load_library()          # torch's HIP runtime first, as for the product library
    stream = torch.cuda.current_stream().cuda_stream
    rows = []
    for op in args.ops:
        if op == "gemm":
            M = N = 8192
            K = args.K
            a_bits, b_bits = I.make_ab(M, N, K, I.FP16, 7000 + K)
            a = torch.from_numpy(a_bits.view("int16")).cuda()
            b = torch.from_numpy(b_bits.view("int16")).cuda()
            out = torch.empty((M, N), dtype=torch.int16, device="cuda")
            flops, what = 2.0 * M * N * K, "gemm_nt M=N=8192 K=%d fp16" % K
            call = lambda lib: lib.gemm_nt(a.data_ptr(), b.data_ptr(), out.data_ptr(), M, N, K, stream, 0)
            view = lambda: out.view(torch.float16)[::509, ::263].float().cpu().numpy()
        elif op == "gemm_fp8":
            M = N = 8192
            K = args.K
            a_bits, b_bits = I.make_ab(M, N, K, I.E4M3, 7000 + K)
            a, b = torch.from_numpy(a_bits).cuda(), torch.from_numpy(b_bits).cuda()
            out = torch.empty((M, N), dtype=torch.int16, device="cuda")
            flops, what = 2.0 * M * N * K, "gemm_nt_fp8 M=N=8192 K=%d" % K
            call = lambda lib: lib.gemm_nt_fp8(a.data_ptr(), b.data_ptr(), out.data_ptr(), M, N, K, stream, 0)
            view = lambda: out.view(torch.float16)[::509, ::263].float().cpu().numpy()
        elif op == "attn_fp8":
            w = I.FP8_WORKLOADS[args.fp8_workload]
            q, k, v = (torch.from_numpy(x).cuda() for x in I.make_workload(w))
            out = torch.empty((w.B, w.H, w.N, w.d), dtype=torch.int16, device="cuda")
            lse = torch.empty((w.B, w.H, w.N), dtype=torch.float32, device="cuda")
            flops, what = w.flops, w.name
            call = lambda lib: lib.attn_fwd_fp8(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), lse.data_ptr(),
                                                w.B, w.H, w.N, w.d, w.scale, int(w.causal), stream, 0)
            view = lambda: np.concatenate([out.view(torch.float16)[:, :, ::251, ::7].float().cpu().numpy().ravel(),
                                           lse[:, :, ::251].cpu().numpy().ravel()])
        else:
            w = I.WORKLOADS[args.causal_workload if op == "attn_causal" else args.workload]
            q, k, v = (torch.from_numpy(x.view("int16")).cuda() for x in I.make_workload(w))
            out = torch.empty_like(q)
            lse = torch.empty((w.B, w.H, w.N), dtype=torch.float32, device="cuda")
            flops, what = w.flops, w.name
            call = lambda lib: lib.attn_fwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), lse.data_ptr(),
                                            w.B, w.H, w.N, w.d, w.scale, int(w.causal), stream, w.dtype)
            dt = torch.float16 if w.dtype == I.FP16 else torch.bfloat16
            view = lambda: np.concatenate([out.view(dt)[:, :, ::251, ::7].float().cpu().numpy().ravel(),
                                           lse[:, :, ::251].cpu().numpy().ravel()])
        reference = None
        for p in grid_points(op):
            path = variant_path(op, p)
            if not os.path.exists(path):
                print("sweep run: %s is not built (run `sweep build` first)" % os.path.relpath(path, HERE), file=sys.stderr)
                continue
            lib = _load(path)
            out.zero_()
            if reference is None:
                # the first variant of a group also warms the device up: about half a second of launches, so that
                # its timing is taken at the settled clock like everyone else's
                import time
                t_end = time.perf_counter() + 0.5
                while time.perf_counter() < t_end:
                    for _ in range(10):
                        call(lib)
                    torch.cuda.synchronize()
            for _ in range(args.warmup):
                rc = call(lib)
            torch.cuda.synchronize()
            if rc != 0:
                print("sweep run: %s returned %d" % (variant_name(op, p), rc), file=sys.stderr)
                continue
            sample = view()
            if reference is None:
                reference = sample              # the default point comes first
            agree = bool(np.allclose(sample, reference, rtol=2e-2, atol=2e-2)) and bool(np.isfinite(sample).all())
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(args.steps):
                call(lib)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / args.steps
            rec = {"op": op, "workload": what, "knobs": p, "ms": ms, "tflops": flops / ms * 1e-9,
                   "default": all(p[k] == DEFAULTS[k] for k in p), "agrees_with_default": agree}
            rows.append(rec)
            print(json.dumps(rec), flush=True)
    print()
    for r in rows:
        print("%-12s %-28s %-58s %8.4f ms %8.1f TFLOP/s%s%s" % (
            r["op"], r["workload"], " ".join("%s=%s" % kv for kv in r["knobs"].items()), r["ms"], r["tflops"],
            "  (default)" if r["default"] else "", "" if r["agrees_with_default"] else "  OUTPUT DIFFERS"))
    return 0


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(prog="python -m paper_2510_14719_amd.sweep")
    sub = ap.add_subparsers(dest="cmd", required=True)
    for name in ("build", "run"):
        sp = sub.add_parser(name)
        sp.add_argument("--op", dest="ops", action="append", choices=sorted(GRIDS), help="default: all")
        if name == "build":
            sp.add_argument("--jobs", type=int, default=4)
        else:
            sp.add_argument("--workload", default="c4")
            sp.add_argument("--causal-workload", default="c5")
            sp.add_argument("--fp8-workload", default="f4")
            sp.add_argument("--K", type=int, default=16384)
            sp.add_argument("--steps", type=int, default=50)
            sp.add_argument("--warmup", type=int, default=15)
    args = ap.parse_args(argv)
    if not args.ops:
        args.ops = sorted(GRIDS)
    return cmd_build(args) if args.cmd == "build" else cmd_run(args)


if __name__ == "__main__":
    sys.exit(main())
