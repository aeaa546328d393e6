"""Host-side model of the LDS ring protocol of the 16-bit attention kernel (no GPU, no library).

Ring of four stages; stage s holds K tile s+1 and V tile s (stage -1 only brings K tile 0).  The prologue
issues stages -1, 0, 1 and waits for all of them.  At barrier j every wave has waited for all of its copies
but the latest stage's; after it, the copies of stage j+2 go out.  Wave group A multiplies [U_{j-1}, T_j] from
stage j-1 after barrier j; group B multiplies [U_j, T_{j+1}] from stage j after barrier j (and T_0 from stage
-1 right after the prologue).  Checked for 1 ... 40 tiles: every stage is complete (waited for by the issuing
wave before the barrier) when it is read, and a slot is only overwritten after the barrier that follows the
last read of the stage it held.
"""
import os

CSRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2510_14719_amd", "csrc")
STAGES = 4


def replay(nt, lpg):
    issued = []                 # (stage, barrier index after which it was issued; -1 = prologue)
    complete = 0
    reads = []                  # (stage, index of the last barrier passed before the read, group)

    def issue(stage, after_barrier):
        for _ in range(lpg):
            issued.append((stage, after_barrier))

    def stage_complete(stage):
        idx = [i for i, c in enumerate(issued) if c[0] == stage]
        return bool(idx) and max(idx) < complete

    for s in (-1, 0, 1):
        issue(s, -1)
    complete = len(issued)                                   # wait for everything, then a barrier
    reads.append((-1, -1, "B"))                              # group B: T_0 before its first barrier
    for j in range(nt):
        # wait_stage(j): all but the latest stage's copies (everything when no further stage follows), barrier j
        complete = max(complete, len(issued) - (lpg if j + 1 < nt else 0))
        a_stage = j - 1                                      # group A reads stage j-1 (T_0: stage -1 at j = 0)
        b_stage = j
        assert stage_complete(a_stage), "group A, tile %d of %d: stage %d not complete" % (j, nt, a_stage)
        assert stage_complete(b_stage) or b_stage > nt - 1, "group B, tile %d of %d: stage %d not complete" % (j, nt, b_stage)
        reads.append((a_stage, j, "A"))
        reads.append((b_stage, j, "B"))
        if j + 2 < nt:
            issue(j + 2, j)
    # U of the last tile: group A reads stage nt-1 after barrier nt (or, when nt_w == nt, without a further barrier: the
    # stage was complete at barrier nt-1 already, which is what is checked here)
    assert stage_complete(nt - 1)
    reads.append((nt - 1, nt - 1, "A"))
    # slot reuse: a copy of stage s issued after barrier b overwrites stage s - STAGES; every read of that stage must
    # have happened before barrier b, i.e. after a barrier with a smaller index, by a wave that reaches barrier b later
    for stage, after in issued:
        old = stage - STAGES
        for rs, rb, grp in reads:
            if rs == old:
                assert rb < after, "stage %d (issued after barrier %d) overwrites stage %d read by group %s after barrier %d" % (stage, after, old, grp, rb)
    return len(issued)


def test_ring_protocol():
    for lpg in (2, 4, 8):
        for nt in range(1, 41):
            assert replay(nt, lpg) == (3 + max(nt - 2, 0)) * lpg


def test_sources_spell_out_what_the_model_assumes():
    src = open(os.path.join(CSRC, "attn_fwd_kernel.hip")).read()
    for needle in ["issue_stage(-1);\n        issue_stage(0);\n        issue_stage(1);",
                   "if (j + 1 < nt) wait_vmcnt<LPG>(); else wait_vmcnt<0>();",
                   "mfma_burst(std::true_type{}, std::true_type{}, stage_ptr(j - 1));",
                   "mfma_burst(std::true_type{}, std::true_type{}, stage_ptr(j));",
                   "issue_stage(j + 2);"]:
        assert needle in src, "attn_fwd_kernel.hip no longer contains `%s`" % needle
