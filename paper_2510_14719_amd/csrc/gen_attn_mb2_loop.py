#!/usr/bin/env python3
"""Generator of the hand-scheduled steady-state loop of the 64-rows-per-wave attention kernel
(``attn_fwd_pipe_kernel.hip`` with four waves per workgroup, one per SIMD).

Why assembly: in this form a wave owns a SIMD and 512 registers, the O accumulators and the Q fragments
live in the accumulation registers, the scores and probabilities in the vector registers, and the vector
work of the softmax has to sit in the shadow of the wave's own MFMAs, a few instructions behind each.
The compiler gives all MFMA results of a function one register class and re-derives the interleaving on
its own; neither fits.  So the loop body is emitted here, instruction by instruction, with fixed
registers, and included by the kernel as one ``asm volatile`` statement; everything outside the steady
state (prologue, the slow softmax path, a wave's last tile, the epilogue) stays C++.

What one pass (iteration j, scores of parity P = j & 1) does is what ``pass`` of the C++ kernel does:
  wait for the copies of stage j, barrier, then 64 MFMAs -- U_{j-1} (O^T += V^T P^T, P of tile j-1) on 16 V^T
  fragments, T_{j+1} (S^T = K Q^T into the scores of parity P^1) on 16 K fragments, every fragment feeding
  the MFMAs of both 32-query blocks in snake order -- and between them
    * the fast softmax of tile j (scores of parity P): p = exp2(s*c - m*c), round, pack, row sums;
      no maximum (see the kernel source), a word of P rewritten only after the last MFMA that reads its
      previous content,
    * the 8 global -> LDS copies of stage j+2 (scalar address arithmetic, tiles clamped to the sequence end),
    * the LDS fragment reads, six fragments ahead of their MFMAs and across the barrier (the stage a pass reads
      became visible one barrier earlier, so the previous pass requests the first fragments);
  at the end the overflow test of the row sums: a lane whose sum is not <= 16384 leaves the loop with the
  redo flag set (the scores of tile j are still in their registers).
The loop is unrolled by two (parity 1, then 0), entered with an odd j and left when j > j_end.

Register contract with the C++ side (all fixed):
  a[0:127]    O[mb][db]      16 registers each, (mb*4 + db)*16
  a[128:191]  Q[mb][kk]      4 registers each, 128 + (mb*8 + kk)*4
  v[0:127]    S[par][mb][kb] 16 registers each, ((par*2 + mb)*2 + kb)*16
  v[128:159]  P[mb][word]    128 + mb*16 + word
  v[160:163]  -m*c of block 0, 1; running row sum of block 0, 1
  v200..v203  per-lane byte offsets: K fragment reads, V^T fragment reads (incl. the V half of a stage), K copy, V copy
  s[36:37] K of the head, s[38:39] V of the head, s40 j (in/out), s41 j_end, s42 scale*log2(e), s43 LDS base,
  s44 wave index, s45 N, s46 redo flag (out)
  clobbered: v164..v199, v204..v225, s47..s63, vcc, scc, m0

Usage: ``python gen_attn_mb2_loop.py [out.inc]`` writes the include file with the two loops (fp16, bf16) as
string-literal macros.  ``--check`` assembles them with llvm-mc for gfx950 first.
"""
from __future__ import annotations

import os
import subprocess
import sys

# Development switches (timing experiments only: the results are wrong with any of them set)
X_NO_VALU = bool(os.environ.get("MB2_NO_VALU"))
X_NO_COPY = bool(os.environ.get("MB2_NO_COPY"))
X_NO_EXP = bool(os.environ.get("MB2_NO_EXP"))
X_NO_LDS = bool(os.environ.get("MB2_NO_LDS"))
X_VALU_FORM = int(os.environ.get("MB2_VALU_FORM", "0"))    # 1: temporaries only; 3: P words not written; 4: scores not read
X_ONLY = os.environ.get("MB2_ONLY", "")                    # keep only these kinds of vector instructions (comma list); "ov": plain FMAs on temporaries
X_T_AGPR = bool(os.environ.get("MB2_T_AGPR"))
X_SUM = os.environ.get("MB2_SUM", "add")                   # row sums: "dot" = v_dot2c on the packed pair, "add" = two fp32 adds              # T accumulates in a[192:255] instead of the S registers

KB, KK, DB, MB = 2, 8, 4, 2
TILE_BYTES = 64 * 256
STAGE_BYTES = 2 * TILE_BYTES
LPG = 8                     # copies per wave and stage (4 K pieces, 4 V pieces)
RING = 8                    # fragment registers: RING fragments of 4 registers
FWIN = 6                    # fragments requested ahead (LDS reads in flight: at most 2 * FWIN <= 15, the counter's range)
VALU_BUDGET = 28            # vector-ALU cycles placed behind one MFMA (an MFMA occupies the pipe for 32)
VALU_BUDGET_BF16 = 34       # bf16 carries two more instructions per score pair (the rounded row sums): the vector ALU is its bound
COST = {"fma": 5, "exp": 9, "cvt": 5, "dot": 5, "add": 5}

S_BASE = lambda par, mb, kb: ((par * 2 + mb) * 2 + kb) * 16
PW = lambda mb, w: 128 + mb * 16 + w
NEGMC = lambda mb: 160 + mb
LRUN = lambda mb: 162 + mb
SUM = lambda mb: 164 + mb
TMP0 = 168                  # 8 pairs of temporaries
FRAG = [184, 188, 192, 196, 208, 212, 216, 220]    # the fragment ring
V_KRD, V_VRD, V_KCP, V_VCP, V_MAX = 200, 201, 202, 203, 206
V_SK = {1: 204, 0: 224}     # LDS address of this lane's K fragment reads, by parity of the pass (the next pass's is set up
V_SV = {1: 205, 0: 225}     # while the current one still reads), and of its V^T fragment reads
O_BASE = lambda mb, db: (mb * 4 + db) * 16
Q_BASE = lambda mb, kk: 128 + (mb * 8 + kk) * 4


def vr(b, n=1):
    return "v%d" % b if n == 1 else "v[%d:%d]" % (b, b + n - 1)


def ar(b, n):
    return "a[%d:%d]" % (b, b + n - 1)


def gen_pass(P: int, el: str, uid: str):
    """Instruction list of one pass on the scores of parity P."""
    mfma = "v_mfma_f32_32x32x16_%s" % el
    cvt = "v_cvt_pk_%s_f32" % el
    dot = "v_dot2c_f32_%s" % el
    ones = "0x3c003c00" if el == "f16" else "0x3f803f80"
    out = []
    emit = out.append

    # ---- top: wait, barrier.  The first FWIN fragments were requested by the previous pass (the stage this pass
    # reads became visible one barrier earlier), the scalar work for the copies follows the first MFMAs.
    emit("s_waitcnt vmcnt(%d)" % LPG)
    emit("s_barrier")
    top_salu = [
        "s_add_i32 s49, s40, 2",
        "s_and_b32 s49, s49, 3",
        "s_lshl_b32 s49, s49, 15",
        "s_add_i32 s49, s49, s43",
        "s_add_i32 s49, s49, s57",                  # LDS address of this wave's first piece of the stage written
        "s_add_i32 s50, s40, 4",                    # K tile j+4, V tile j+2: first row min(t*64, N-64), 256 B per row
        "s_lshl_b32 s50, s50, 6",
        "s_min_i32 s50, s50, s47",
        "s_lshl_b32 s50, s50, 8",
        "s_add_i32 s50, s50, s56",
        "s_add_u32 s52, s36, s50",
        "s_addc_u32 s53, s37, 0",
        "s_add_i32 s51, s40, 2",
        "s_lshl_b32 s51, s51, 6",
        "s_min_i32 s51, s51, s47",
        "s_lshl_b32 s51, s51, 8",
        "s_add_i32 s51, s51, s56",
        "s_add_u32 s54, s38, s51",
        "s_addc_u32 s55, s39, 0",
    ] + ["v_mov_b32 %s, 0" % vr(SUM(0) + r) for r in range(2 if X_SUM == "dot" else 4)]
    # the addresses of the NEXT pass's fragment reads (it reads stage j), set up half way through this one
    next_addr = [
        "s_and_b32 s48, s40, 3",
        "s_lshl_b32 s48, s48, 15",
        "s_add_i32 s48, s48, s43",
        "v_add_u32 %s, s48, %s" % (vr(V_SK[P ^ 1]), vr(V_KRD)),
        "v_add_u32 %s, s48, %s" % (vr(V_SV[P ^ 1]), vr(V_VRD)),
    ]

    # ---- fragments: 0..15 V^T (U), 16..31 K (T); 32 .. 32+FWIN-1 are fragments 0 .. FWIN-1 of the next pass
    NF = 32
    lds_queue = []                                  # fragment index of every LDS read still counted, in issue order
    for f0 in range(FWIN):                          # requested by the previous pass (or by the loop's prologue)
        lds_queue.extend([f0, f0] if f0 < 16 else [f0])

    def fetch(f, out_list=None, queue=lds_queue):
        e = emit if out_list is None else out_list.append
        par = P if f < NF else P ^ 1
        g = f % NF
        r = FRAG[f % RING]
        if X_NO_LDS and f >= 4:
            return
        if g < 16:
            kb, ks, db = g // 8, (g // 4) % 2, g % 4
            off = db * 4096 + (kb * 32 + ks * 16) * 64
            e("ds_read_b64_tr_b16 %s, %s offset:%d" % (vr(r, 2), vr(V_SV[par]), off))
            e("ds_read_b64_tr_b16 %s, %s offset:%d" % (vr(r + 2, 2), vr(V_SV[par]), off + 512))
            queue.extend([f, f])
        else:
            idx = g - 16
            kb, kk = idx % 2, idx // 2
            off = ((kk >> 1) * 4 + kb * 2) * 1024 + (kk & 1) * 512
            e("ds_read_b128 %s, %s offset:%d" % (vr(r, 4), vr(V_SK[par]), off))
            queue.append(f)

    def wait_frag(f):
        # LDS reads return in order: everything up to the last read of fragment f must be back
        if X_NO_LDS and f >= 4:
            return
        last = max(i for i, g in enumerate(lds_queue) if g == f)
        emit("s_waitcnt lgkmcnt(%d)" % (len(lds_queue) - 1 - last))
        del lds_queue[:last + 1]

    # ---- the vector work of the fast softmax as micro-operations with earliest MFMA slots
    steps = [(q, mb) for q in range(16) for mb in range(MB)]
    ops = []                                        # per step: list of (kind, text)
    for s, (q, mb) in enumerate(steps):
        kb, t = q // 8, q % 8
        sreg = S_BASE(P, mb, kb) + 2 * t
        x0, x1 = TMP0 + (s % 8) * 2, TMP0 + (s % 8) * 2 + 1
        first_c = (q // 4 + 1) * DB * MB            # first slot after the last MFMA of U reading word q of the blocks
        src0, src1, ng, wdst = vr(sreg), vr(sreg + 1), vr(NEGMC(mb)), vr(PW(mb, q))
        if X_VALU_FORM in (1, 4):
            src0, src1 = vr(x0), vr(x1)
        if X_VALU_FORM == 1:
            ng = vr(x0)
        if X_VALU_FORM in (1, 3):
            wdst = vr(207)
        # (kind, text, earliest slot, indices of the operations of the step it needs; each at least one slot earlier)
        step_ops = [
            ("fma", "v_fma_f32 %s, s42, %s, %s" % (vr(x0), src0, ng), 0, []),
            ("fma", "v_fma_f32 %s, s42, %s, %s" % (vr(x1), src1, ng), 0, []),
            ("exp", "v_exp_f32 %s, %s" % (vr(x0), vr(x0)), 0, [0]),
            ("exp", "v_exp_f32 %s, %s" % (vr(x1), vr(x1)), 0, [1]),
            ("cvt", "%s %s, %s, %s" % (cvt, wdst, vr(x0), vr(x1)), first_c, [2, 3]),
        ]
        # row sums (two chains per block).  Not v_dot2c: the dot instructions go through the matrix pipe and every one
        # stalls the MFMA stream (measured: 32 of them cost a pass 450 cycles).  fp16: the two unrounded values are added;
        # bf16: the ROUNDED ones (a bf16 is the upper half of its fp32), so that the rounding of numerator and
        # denominator cancels on rows that a few keys dominate.
        if X_SUM == "dot":
            step_ops.append(("dot", "%s %s, %s, %s" % (dot, vr(SUM(mb)), ones, wdst), 0, [4]))
        elif el == "f16":
            step_ops.append(("add", "v_add_f32 %s, %s, %s" % (vr(SUM(mb)), vr(SUM(mb)), vr(x0)), 0, [2]))
            step_ops.append(("add", "v_add_f32 %s, %s, %s" % (vr(SUM(mb) + 2), vr(SUM(mb) + 2), vr(x1)), 0, [3]))
        else:
            step_ops.append(("add", "v_lshlrev_b32 %s, 16, %s" % (vr(x0), wdst), 0, [4]))
            step_ops.append(("add", "v_and_b32 %s, 0xffff0000, %s" % (vr(x1), wdst), 0, [4]))
            step_ops.append(("add", "v_add_f32 %s, %s, %s" % (vr(SUM(mb)), vr(SUM(mb)), vr(x0)), 0, [5]))
            step_ops.append(("add", "v_add_f32 %s, %s, %s" % (vr(SUM(mb) + 2), vr(SUM(mb) + 2), vr(x1)), 0, [6]))
        ops.append(step_ops)
    nxt = [0] * len(steps)                          # next micro-operation of every step
    NOPS = len(ops[0])
    done_slot = [[-1] * NOPS for _ in steps]        # slot in which each was emitted


    def emit_valu(slot, budget):
        used = 0
        if X_NO_VALU:
            for s in range(len(steps)):
                nxt[s] = NOPS
            return
        for s in range(len(steps)):
            # the temporaries of step s are those of step s-8: start only when that one has finished
            if s >= 8 and nxt[s] == 0 and nxt[s - 8] < NOPS:
                break
            while nxt[s] < NOPS:
                i = nxt[s]
                kind, text, earliest, deps = ops[s][i]
                if slot < earliest or any(done_slot[s][d] < 0 or done_slot[s][d] >= slot for d in deps):
                    break
                if used + COST[kind] > budget:
                    return
                if X_ONLY == "ov":
                    t0 = TMP0 + (s * 6 + i) % 16
                    emit("v_fma_f32 %s, %s, s42, 0.5" % (vr(t0), vr(t0)))
                elif not X_ONLY or kind in X_ONLY.split(","):
                    emit(text if not (X_NO_EXP and kind == "exp") else text.replace("v_exp_f32", "v_mov_b32"))
                used += COST[kind]
                done_slot[s][i] = slot
                nxt[s] += 1

    # ---- copies: piece c after MFMA 2 + 8c
    def emit_copy(c):
        if X_NO_COPY:
            return
        i = c % 4
        src, lane, dst = ("s52", V_KCP, 0) if c < 4 else ("s54", V_VCP, TILE_BYTES)
        hi = "s53" if c < 4 else "s55"
        emit("s_add_u32 s58, %s, %d" % (src, i * 4096))
        emit("s_addc_u32 s59, %s, 0" % hi)
        emit("s_add_i32 s60, s49, %d" % (dst + i * 1024))
        emit("s_mov_b32 m0, s60")
        emit("s_nop 0")
        emit("global_load_lds_dwordx4 %s, s[58:59]" % vr(lane))

    slot = 0
    for f in range(NF):
        if f + FWIN == NF:                          # from here on the requests go to the next pass's stage
            for l in next_addr:
                emit(l)
        fetch(f + FWIN)
        wait_frag(f)
        r = FRAG[f % RING]
        for i in range(MB):
            mb = (MB - 1 - i) if (f & 1) else i
            if f < 16:
                kb, ks, db = f // 8, (f // 4) % 2, f % 4
                o = O_BASE(mb, db)
                emit("%s %s, %s, %s, %s" % (mfma, ar(o, 16), vr(r, 4), vr(PW(mb, kb * 8 + ks * 4), 4), ar(o, 16)))
            else:
                idx = f - 16
                kb, kk = idx % 2, idx // 2
                sb = S_BASE(P ^ 1, mb, kb)
                if X_T_AGPR:
                    ab = 192 + (mb * 2 + kb) * 16
                    emit("%s %s, %s, %s, %s" % (mfma, ar(ab, 16), vr(r, 4), ar(Q_BASE(mb, kk), 4), "0" if kk == 0 else ar(ab, 16)))
                else:
                    emit("%s %s, %s, %s, %s" % (mfma, vr(sb, 16), vr(r, 4), ar(Q_BASE(mb, kk), 4), "0" if kk == 0 else vr(sb, 16)))
            if slot % 8 == 2:
                emit_copy(slot // 8)
            budget = VALU_BUDGET if el == "f16" else VALU_BUDGET_BF16
            if slot < 2:                            # the scalar work of the pass top, in two halves behind the first two MFMAs
                half = (len(top_salu) + 1) // 2
                for l in top_salu[slot * half:(slot + 1) * half]:
                    emit(l)
                budget = 8
            emit_valu(slot, budget)
            slot += 1
    # whatever vector work is left goes behind the last MFMA, slot by slot (keeps the one-slot distances)
    while any(n < NOPS for n in nxt):
        emit("s_nop 1")                             # (no MFMA in between any more: a transcendental's result needs the distance)
        emit_valu(slot, 1000)
        slot += 1
    assert X_NO_LDS or sorted(set(lds_queue)) == list(range(NF, NF + FWIN)), lds_queue    # exactly the next pass's first fragments are in flight

    # ---- end of the pass: overflow test of the two row sums, running sums, next j
    if X_SUM != "dot":
        emit("v_add_f32 %s, %s, %s" % (vr(SUM(0)), vr(SUM(0)), vr(SUM(0) + 2)))
        emit("v_add_f32 %s, %s, %s" % (vr(SUM(1)), vr(SUM(1)), vr(SUM(1) + 2)))
    emit("v_cmp_nle_f32 vcc, %s, %s" % (vr(SUM(0)), vr(V_MAX)))
    emit("v_cmp_nle_f32_e64 s[60:61], %s, %s" % (vr(SUM(1)), vr(V_MAX)))
    emit("s_or_b64 s[60:61], vcc, s[60:61]")
    emit("s_cmp_lg_u64 s[60:61], 0")
    emit("s_cbranch_scc1 L_mb2_redo_%s" % uid)
    emit("v_add_f32 %s, %s, %s" % (vr(LRUN(0)), vr(LRUN(0)), vr(SUM(0))))
    emit("v_add_f32 %s, %s, %s" % (vr(LRUN(1)), vr(LRUN(1)), vr(SUM(1))))
    emit("s_add_i32 s40, s40, 1")
    emit("s_cmp_gt_i32 s40, s41")
    emit("s_cbranch_scc1 L_mb2_done_%s" % uid)
    return out


def gen_loop(el: str, uid: str):
    out = []
    out.append("s_add_i32 s47, s45, -64")                      # N - 64
    out.append("s_lshl_b32 s56, s44, 6")                       # wave * 64: this wave's feature group inside a source row
    out.append("s_lshl_b32 s57, s44, 12")                      # wave * 4096: its pieces inside a K or V slot
    out.append("v_mov_b32 %s, 0x46800000" % vr(V_MAX))         # 16384.0
    # the first pass (odd j, parity 1) reads stage j-1, visible since the last barrier: request its first fragments
    out.append("s_add_i32 s48, s40, -1")
    out.append("s_and_b32 s48, s48, 3")
    out.append("s_lshl_b32 s48, s48, 15")
    out.append("s_add_i32 s48, s48, s43")
    out.append("v_add_u32 %s, s48, %s" % (vr(V_SK[1]), vr(V_KRD)))
    out.append("v_add_u32 %s, s48, %s" % (vr(V_SV[1]), vr(V_VRD)))
    for f0 in range(FWIN):
        r = FRAG[f0 % RING]
        kb, ks, db = f0 // 8, (f0 // 4) % 2, f0 % 4
        off = db * 4096 + (kb * 32 + ks * 16) * 64
        out.append("ds_read_b64_tr_b16 %s, %s offset:%d" % (vr(r, 2), vr(V_SV[1]), off))
        out.append("ds_read_b64_tr_b16 %s, %s offset:%d" % (vr(r + 2, 2), vr(V_SV[1]), off + 512))
    out.append("L_mb2_top_%s:" % uid)
    out += gen_pass(1, el, uid)
    out += gen_pass(0, el, uid)
    out.append("s_branch L_mb2_top_%s" % uid)
    out.append("L_mb2_redo_%s:" % uid)
    out.append("s_mov_b32 s46, 1")
    out.append("s_branch L_mb2_out_%s" % uid)
    out.append("L_mb2_done_%s:" % uid)
    out.append("s_mov_b32 s46, 0")
    out.append("L_mb2_out_%s:" % uid)
    out.append("s_waitcnt lgkmcnt(0)")                          # the fragments requested for a pass that does not come
    # the code that follows may read S and O at once; it does not know that MFMAs wrote them
    out += ["s_nop 15"] * 4
    return out


CLOBBER_V = list(range(164, 200)) + list(range(204, 226))
CLOBBER_S = list(range(47, 64))


def write_inc(path: str):
    with open(path, "w") as fh:
        fh.write("// Generated by gen_attn_mb2_loop.py -- do not edit.  The steady-state loop of the 64-rows-per-wave attention\n")
        fh.write("// kernel as assembly text (register contract and schedule: see the generator).\n")
        for el in ("f16", "bf16"):
            lines = gen_loop(el, "%=")
            fh.write("#define ATTN_MB2_LOOP_%s \\\n" % el.upper())
            for l in lines:
                fh.write('    "%s\\n\\t" \\\n' % l)
            fh.write('    ""\n')
        fh.write("#define ATTN_MB2_LOOP_CLOBBERS \\\n    ")
        extra = ['"a%d"' % r for r in range(192, 256)] if X_T_AGPR else []
        fh.write(", ".join(['"v%d"' % r for r in CLOBBER_V] + extra + ['"s%d"' % r for r in CLOBBER_S] + ['"vcc"', '"scc"', '"m0"', '"memory"']))
        fh.write("\n")


def check():
    """Assemble both loops with llvm-mc for gfx950 (syntax and encodability only)."""
    mc = "/opt/rocm/llvm/bin/llvm-mc"
    for el in ("f16", "bf16"):
        text = "\n".join(gen_loop(el, "x")) + "\n"
        res = subprocess.run([mc, "-arch=amdgcn", "-mcpu=gfx950", "-filetype=null"], input=text, text=True,
                             stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
        if res.returncode != 0 or "error" in res.stdout:
            sys.stderr.write(res.stdout[:4000])
            raise SystemExit("llvm-mc rejected the %s loop" % el)
    lines = gen_loop("f16", "x")
    n_mfma = sum(1 for l in lines if l.startswith("v_mfma"))
    n_valu = sum(1 for l in lines if l.startswith("v_") and not l.startswith("v_mfma"))
    print("ok: %d instructions per two passes, %d MFMAs, %d other vector instructions" % (len(lines), n_mfma, n_valu))


if __name__ == "__main__":
    args = [a for a in sys.argv[1:] if a != "--check"]
    if "--check" in sys.argv[1:]:
        check()
    write_inc(args[0] if args else os.path.join(os.path.dirname(os.path.abspath(__file__)), "attn_mb2_loop.inc"))
