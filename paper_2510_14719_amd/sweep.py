"""Sweep of the kernels' schedule parameters (the counterpart of the paper's study of the aref depth D
and the MMA issue depth P, Section 5.5, and of its ablation, Section 5.6).

The knobs are compile-time constants of the HIP sources, so a sweep is two steps:

    python -m paper_2510_14719_amd.sweep build [--op attn|gemm|...] # anywhere hipcc runs (no GPU needed)
    python -m paper_2510_14719_amd.sweep run   [--op attn|gemm|...] ...  # on the GPU: times every built variant

``build`` compiles one shared library per grid point into ``sweep_variants/`` next to this file; ``run``
loads each through ctypes, times it and prints one JSON line per variant plus a table.  ``run`` also compares a
few sampled outputs of every variant with the default point's (a smoke check that flags a variant computing
something else; it exits non-zero when one differs, fails or is missing).  The check that counts, every
variant against the CPU oracle within the library's tolerances, lives in ``tests/test_gpu_sweep_variants.py``
(the package itself never imports the oracle); ``build --test-variants`` builds just the points that test
loads.  ``run --only NAME`` runs one variant, e.g. under ``rocprofv3 --pmc`` for its counters.

What the axes stand for on gfx950:
  attn_schedule (d = 128)
             ATTN_CFG_PIPE      0: two wave groups half a period apart (attn_fwd_kernel.hip, the default);
                                1: the coarse-grained pipeline of the paper's Algorithm 1 inside every wave
                                   (attn_fwd_pipe_kernel.hip): the softmax of tile j between the MFMAs of U_{j-1} and T_{j+1}
             ATTNP_CFG_NW       (pipe only) 8 waves of 32 query rows (two per SIMD), or 4 waves of 64 rows (one per SIMD,
                                O and Q in the accumulation registers, the steady state a generated assembly loop)
             ATTNP_INTERLEAVE   (pipe only) 1: softmax in slices between the MFMAs; 0: after them as one block
             ATTNP_FWIN         (pipe only) LDS fragments requested ahead of their MFMAs
             The 16-bit two-group kernel fixes its ring depth (4 stages: the protocol and the 160 KiB LDS), its tile
             (64 keys) and its eight waves by construction (static_asserts in the source); the in-wave kernel is
             the variant with another ring (5 stages) and, as ATTNP_CFG_NW = 4, with four waves of 64 rows.
  attn_waves ATTN_CFG_NW        waves per workgroup of the two-group kernel: 8 (two groups, 256 query rows) or 12 (THREE groups
                                of four waves, one wave of each per SIMD, 384 query rows, 168 registers per wave: the
                                middle group splits its softmax around its burst, so that a SIMD sees three bursts per
                                tile back to back)
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
    "attn_schedule": {"ATTN_CFG_PIPE": [0, 1], "ATTNP_CFG_NW": [8, 4], "ATTNP_INTERLEAVE": [1, 0], "ATTNP_FWIN": [3, 2]},
    "attn_waves": {"ATTN_CFG_NW": [8, 12]},
    "attn": {"ATTN_FWIN": [1, 2, 4, 8], "ATTN_COPY_GROUP": [0, 2, 1], "ATTN_SUMCHAINS": [2, 4]},
    "attn_causal": {"ATTN_PERSISTENT": [0, 1], "ATTN_FWIN": [2, 4]},
    "attn_fp8": {"ATTN8_FWIN": [1, 2, 3], "ATTN8_INTERLEAVE": [1, 0], "ATTN8_STAGES": [4, 8], "ATTN8_COPIES_IN_PASS": [1, 0]},
    "gemm": {"GEMM_CONFIG": [0, 1, 2, 3, 4], "GEMM_STAGES": [4, 5], "GEMM_TAIL_READS": [3, 0]},
    "gemm_fp8": {"GEMM8_CONFIG": [0, 1, 2, 3, 4], "GEMM8_STAGES": [4, 5], "GEMM8_TAIL_READS": [3, 0]},
}
DEFAULTS = {"ATTN_CFG_NW": 8, "ATTN_CFG_PIPE": 0, "ATTNP_CFG_NW": 8, "ATTNP_INTERLEAVE": 1, "ATTNP_FWIN": 3, "ATTN8_FWIN": 2, "ATTN8_INTERLEAVE": 1, "ATTN8_STAGES": 4, "ATTN8_COPIES_IN_PASS": 1, "ATTN_FWIN": 2, "ATTN_COPY_GROUP": 0, "ATTN_SUMCHAINS": 4, "ATTN_PERSISTENT": 1,
            "GEMM_STAGES": 4, "GEMM_CONFIG": 0, "GEMM_TAIL_READS": 3,
            "GEMM8_STAGES": 4, "GEMM8_TAIL_READS": 3, "GEMM8_COPY_PHASE": 1, "GEMM8_CONFIG": 0}


# The non-default points that tests/test_gpu_sweep_variants.py checks against the oracle (two per operation).
TEST_VARIANTS = {
    "attn_schedule": [{"ATTN_CFG_PIPE": 1, "ATTNP_CFG_NW": 8, "ATTNP_INTERLEAVE": 1, "ATTNP_FWIN": 3},
                      {"ATTN_CFG_PIPE": 1, "ATTNP_CFG_NW": 8, "ATTNP_INTERLEAVE": 0, "ATTNP_FWIN": 2},
                      {"ATTN_CFG_PIPE": 1, "ATTNP_CFG_NW": 4, "ATTNP_INTERLEAVE": 1, "ATTNP_FWIN": 3}],
    "attn_waves": [{"ATTN_CFG_NW": 12}],
    "attn": [{"ATTN_FWIN": 4, "ATTN_COPY_GROUP": 2, "ATTN_SUMCHAINS": 2}, {"ATTN_FWIN": 1, "ATTN_COPY_GROUP": 1, "ATTN_SUMCHAINS": 4}],
    "attn_causal": [{"ATTN_PERSISTENT": 0, "ATTN_FWIN": 2}, {"ATTN_PERSISTENT": 1, "ATTN_FWIN": 4}],
    "attn_fp8": [{"ATTN8_FWIN": 3, "ATTN8_INTERLEAVE": 0, "ATTN8_STAGES": 4, "ATTN8_COPIES_IN_PASS": 1},
                 {"ATTN8_FWIN": 1, "ATTN8_INTERLEAVE": 1, "ATTN8_STAGES": 8, "ATTN8_COPIES_IN_PASS": 0}],
    "gemm": [{"GEMM_CONFIG": 1, "GEMM_STAGES": 5, "GEMM_TAIL_READS": 0}, {"GEMM_CONFIG": 4, "GEMM_STAGES": 4, "GEMM_TAIL_READS": 3}],
    "gemm_fp8": [{"GEMM8_CONFIG": 2, "GEMM8_STAGES": 5, "GEMM8_TAIL_READS": 0}, {"GEMM8_CONFIG": 3, "GEMM8_STAGES": 4, "GEMM8_TAIL_READS": 3}],
}


def grid_points(op: str):
    """All combinations of the grid of ``op`` as dicts, the default point first.  (For attn_schedule the pipe-only
    knobs only vary with ATTN_CFG_PIPE = 1.)"""
    g = GRIDS[op]
    keys = list(g)
    pts = [dict(zip(keys, vals)) for vals in itertools.product(*(g[k] for k in keys))]
    if op == "attn_schedule":
        # the knobs of the in-wave kernel only vary where it is selected; with four waves its steady state is the
        # generated assembly loop, which has its own fragment window and is interleaved by construction
        pts = [p for p in pts if (p["ATTN_CFG_PIPE"] == 1 or all(p[k] == DEFAULTS[k] for k in keys if k != "ATTN_CFG_PIPE"))
               and (p["ATTNP_CFG_NW"] == 8 or (p["ATTNP_INTERLEAVE"] == 1 and p["ATTNP_FWIN"] == 3))]
    pts.sort(key=lambda p: (not all(p[k] == DEFAULTS[k] for k in keys), [p[k] for k in keys]))
    return pts


def variant_name(op: str, point: dict) -> str:
    return op + "__" + "__".join("%s-%s" % (k.split("_", 1)[1].lower(), point[k]) for k in sorted(point))


def variant_path(op: str, point: dict) -> str:
    return os.path.join(VARIANT_DIR, "lib%s.so" % variant_name(op, point))


def build_test_variants(jobs: int = 4, verbose: bool = False):
    """Build the points of TEST_VARIANTS (what the GPU test of the variants loads).  Returns their paths."""
    from concurrent.futures import ThreadPoolExecutor
    from . import build as lib_build
    os.makedirs(VARIANT_DIR, exist_ok=True)
    todo = [(["%s=%s" % kv for kv in p.items()], variant_path(op, p)) for op, pts in TEST_VARIANTS.items() for p in pts]
    with ThreadPoolExecutor(max(1, jobs)) as ex:
        outs = list(ex.map(lambda j: lib_build.build(extra_defines=j[0], out=j[1], jobs=2), todo))
    if verbose:
        for o in outs:
            print("built", os.path.relpath(o, HERE), flush=True)
    return outs


def cmd_build(args) -> int:
    from concurrent.futures import ThreadPoolExecutor
    from . import build as lib_build
    if args.test_variants:
        build_test_variants(args.jobs, verbose=True)
        return 0
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
    problems = 0                    # variants that are missing, fail to run or disagree with the default point
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
        else:               # attn, attn_causal, attn_schedule, attn_waves
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
            is_default = all(p[k] == DEFAULTS[k] for k in p)
            if args.only and variant_name(op, p) != args.only and not is_default:
                continue
            if not os.path.exists(path):
                print("sweep run: %s is not built (run `sweep build` first)" % os.path.relpath(path, HERE), file=sys.stderr)
                problems += 1
                if is_default:
                    print("sweep run: without the default point of %s nothing can be compared; skipping the operation" % op, file=sys.stderr)
                    break
                continue
            lib = _load(path)
            out.zero_()
            rc = call(lib)          # (also the case --warmup 0)
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
                problems += 1
                continue
            sample = view()
            if reference is None:
                reference = sample              # the default point comes first
            agree = bool(np.allclose(sample, reference, rtol=2e-2, atol=2e-2)) and bool(np.isfinite(sample).all())
            problems += 0 if agree else 1
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(args.steps):
                call(lib)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / args.steps
            rec = {"op": op, "workload": what, "variant": variant_name(op, p), "knobs": p, "ms": ms, "tflops": flops / ms * 1e-9,
                   "default": is_default, "agrees_with_default": agree}
            rows.append(rec)
            print(json.dumps(rec), flush=True)
    print()
    for r in rows:
        print("%-12s %-28s %-58s %8.4f ms %8.1f TFLOP/s%s%s" % (
            r["op"], r["workload"], " ".join("%s=%s" % kv for kv in r["knobs"].items()), r["ms"], r["tflops"],
            "  (default)" if r["default"] else "", "" if r["agrees_with_default"] else "  OUTPUT DIFFERS"))
    if problems:
        print("sweep run: %d variant(s) missing, failing or differing from the default point" % problems, file=sys.stderr)
        return 1
    return 0


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(prog="python -m paper_2510_14719_amd.sweep")
    sub = ap.add_subparsers(dest="cmd", required=True)
    for name in ("build", "run"):
        sp = sub.add_parser(name)
        sp.add_argument("--op", dest="ops", action="append", choices=sorted(GRIDS), help="default: all")
        if name == "build":
            sp.add_argument("--jobs", type=int, default=4)
            sp.add_argument("--test-variants", action="store_true", help="only the points the GPU test of the variants loads")
        else:
            sp.add_argument("--only", default=None, help="run the default point and this variant only (a name as printed in the JSON lines)")
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
