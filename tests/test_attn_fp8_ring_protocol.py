"""Host-side model of the LDS ring protocol of the 8-bit-float attention kernel (no GPU, no library).

Ring of STAGES stages (4 or 8), AHEAD = STAGES - 2.  Stage s holds K tile s+2 and V tile s.  The prologue
issues stages -2 ... AHEAD-1 and waits for all but the last AHEAD-1 of them (stages <= 0 complete), barrier.
step(j): wait for all of the wave's copies except those of the at most AHEAD-1 stages after stage j, barrier j,
then issue stage j+AHEAD (while it is <= last_stage = max(AHEAD-1, nt-1)).  After barrier j a wave reads stage
j-1 and, at the end of the iteration (or for the last tile's second contraction), stage j.  T_0 reads stage -2
right after the prologue.  Checked for 1 ... 40 tiles: a stage is complete when it is read, and a slot is only
overwritten after the barrier that follows the last read of the stage it held.
"""
import os

import pytest

CSRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2510_14719_amd", "csrc")


def replay(nt, ppw, stages):
    ahead = stages - 2
    last_stage = max(ahead - 1, nt - 1)
    issued, reads = [], []          # (stage, after barrier), (stage, after barrier)
    complete = 0

    def issue(stage, after):
        for _ in range(ppw):
            issued.append((stage, after))

    def stage_complete(stage):
        idx = [i for i, c in enumerate(issued) if c[0] == stage]
        return bool(idx) and max(idx) < complete

    for s in range(-2, ahead):
        issue(s, -1)
    complete = len(issued) - (ahead - 1) * ppw
    for s in (-2, -1, 0):
        assert stage_complete(s)
    reads.append((-2, -1))                                   # T_0
    for j in range(nt):
        n_out = min(j + ahead - 1, last_stage) - j           # stages after j that may stay in flight
        complete = max(complete, len(issued) - max(n_out, 0) * ppw)
        assert stage_complete(j - 1) and stage_complete(j), "tile %d of %d, %d stages" % (j, nt, stages)
        reads.append((j - 1, j))
        reads.append((j, j))
        if j + ahead <= last_stage:
            issue(j + ahead, j)
    assert all(s <= last_stage for s, _ in issued)
    complete = len(issued)
    for stage, after in issued:
        old = stage - stages
        for rs, rb in reads:
            if rs == old:
                assert rb < after, "stage %d (issued after barrier %d) overwrites stage %d, read after barrier %d" % (stage, after, old, rb)
    return len(issued)


@pytest.mark.parametrize("stages", [4, 8])
def test_ring_protocol(stages):
    for ppw in (1, 2, 4):
        for nt in range(1, 41):
            ahead = stages - 2
            assert replay(nt, ppw, stages) == (max(ahead - 1, nt - 1) + 3) * ppw


def test_sources_spell_out_what_the_model_assumes():
    src = open(os.path.join(CSRC, "attn_fwd_fp8_kernel.hip")).read()
    for needle in ["for (int s0 = -2; s0 < AHEAD; ++s0) issue_stage(s0);",
                   "const int last_stage = max(AHEAD - 1, nt - 1);",
                   "const int n_out = min(j + AHEAD - 1, last_stage) - j;",
                   "if (n_out >= AHEAD - 1) wait_vmcnt<(AHEAD - 1) * PPW>();",
                   "else wait_vmcnt<0>();",
                   "const int s = j + AHEAD;",
                   "pass(NO, Y, NO, NO, P1, stage_ptr(-2), 0);",
                   "pass(Y, Y, Y, Y, P1, stage_ptr(j - 1), j);",
                   "pass(Y, NO, NO, NO, parx, stage_ptr(j), j + 1);"]:
        assert needle in src, "attn_fwd_fp8_kernel.hip no longer contains `%s`" % needle
