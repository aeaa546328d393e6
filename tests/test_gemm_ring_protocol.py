"""Host-side model of the LDS ring protocols of the matrix-product kernels (no GPU, no library).

The kernels track their global -> LDS copies with a counter of copies in flight (a wait for "all but the
last n" completes the older ones, in issue order) and one workgroup barrier per K tile.  This test replays
the order of issues, waits, barriers and fragment reads that the kernel sources spell out and checks the
two properties the protocol exists for, for every number of K tiles from 1 to 40 and both wave layouts:

  * every copy of a stage has been waited for, by the wave that issued it, before the barrier that
    precedes the first read of that stage (all waves run the same sequence, so one wave stands for all);
  * a ring slot is overwritten only by a copy issued after the barrier that follows the last read of the
    stage it held.

The literal wait expressions the model assumes are also looked up in the sources, so that a change of the
kernel without a change of the model fails here.
"""
import os
import re

import pytest

CSRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2510_14719_amd", "csrc")


class Wave:
    """The copy bookkeeping of one wave: issue order, what has been waited for, what each slot holds."""

    def __init__(self, stages):
        self.stages = stages
        self.issued = []            # (stage, piece, tile during which it was issued; -1 = prologue)
        self.complete = 0           # the first `complete` issued copies are known to have landed
        self.slot_stage = {}        # slot -> stage of the copy most recently issued into it

    def issue(self, stage, piece, tile, last_read_tile_of):
        slot = stage % self.stages
        prev = self.slot_stage.get(slot)
        if prev is not None and prev != stage:
            # the stage that sat in this slot must not be read any more: its reads end with tile
            # last_read_tile_of(prev), and this copy is issued during `tile`, after that tile's successor's barrier
            assert last_read_tile_of(prev) < tile, "slot %d: stage %d overwritten during tile %d while stage %d is still read" % (slot, stage, tile, prev)
        self.slot_stage[slot] = stage
        self.issued.append((stage, piece, tile))

    def wait(self, n):
        self.complete = max(self.complete, len(self.issued) - n)

    def stage_complete(self, stage):
        idx = [i for i, c in enumerate(self.issued) if c[0] == stage]
        return bool(idx) and max(idx) < self.complete


def run_paired(nk, lpg):
    """Five stages; even tiles issue stages j+4 and j+5 alternately, one copy per slot; the fragments of tile
    j+1 are read during tile j; waits: all but 2*lpg (even j) or all but 2*lpg+1 (odd j)."""
    w = Wave(5)
    clamp = lambda s: min(s, nk - 1)
    # a stage s is read as "fragments of tile s": during tile s-1 (stage 0: in the prologue); the last tile re-reads itself
    last_read = lambda s: s - 1 if s < nk else -1          # stages past the end are never read
    for s in range(4):
        for i in range(lpg):
            w.issue(s, i, -1, last_read)
    w.wait(3 * lpg)
    assert w.stage_complete(0)
    for j in range(nk):
        w.wait(2 * lpg if j % 2 == 0 else 2 * lpg + 1)
        # barrier j: every wave has waited as above, so stage min(j+1, nk-1) must be complete
        assert w.stage_complete(clamp(j + 1)), "tile %d of %d: stage %d read before its copies were waited for" % (j, nk, clamp(j + 1))
        if j % 2 == 0:
            for q in range(2 * lpg):
                w.issue(j + 4 + (q & 1), q >> 1, j, last_read)
    w.wait(0)
    return len(w.issued)


def run_unpaired(nk, lpg, stages):
    """`stages` stages, copies stages-1 tiles ahead, one stage per tile; steady-state wait: all but
    (ahead-2)*lpg; draining tiles wait for what is left."""
    ahead = stages - 1
    w = Wave(stages)
    last_read = lambda s: s - 1
    for s in range(min(ahead, nk)):
        for i in range(lpg):
            w.issue(s, i, -1, last_read)
    w.wait((min(ahead, nk) - 1) * lpg)
    assert w.stage_complete(0)
    for j in range(nk):
        steady = j + ahead < nk
        if steady:
            w.wait((ahead - 2) * lpg)
        elif ahead > 3 and j + 3 < nk:
            w.wait(2 * lpg)
        elif j + 2 < nk:
            w.wait(lpg)
        else:
            w.wait(0)
        if j + 1 < nk:
            assert w.stage_complete(j + 1), "tile %d of %d: stage %d not complete" % (j, nk, j + 1)
        if j + ahead < nk:
            for i in range(lpg):
                w.issue(j + ahead, i, j, last_read)
    assert w.complete == len(w.issued)
    return len(w.issued)


@pytest.mark.parametrize("lpg", [4, 8])              # 8 waves: 4 copies per wave and stage; 4 waves: 8
def test_paired_ring(lpg):
    for nk in range(1, 41):
        n = run_paired(nk, lpg)
        assert n == 4 * lpg + ((nk + 1) // 2) * 2 * lpg


@pytest.mark.parametrize("stages", [4, 5])
@pytest.mark.parametrize("lpg", [4, 8])
def test_unpaired_ring(lpg, stages):
    for nk in range(1, 41):
        assert run_unpaired(nk, lpg, stages) == nk * lpg


def test_model_detects_a_short_wait_and_an_early_overwrite():
    # the same replay with one copy fewer waited for, or with the pair issued one tile early, must fail
    w = Wave(5)
    last_read = lambda s: s - 1
    for s in range(4):
        for i in range(4):
            w.issue(s, i, -1, last_read)
    w.wait(3 * 4 + 1)
    assert not w.stage_complete(0)
    with pytest.raises(AssertionError):
        w2 = Wave(5)
        for s in range(5):
            for i in range(4):
                w2.issue(s, i, -1, last_read)
        w2.issue(5, 0, 0, last_read)          # slot of stage 0 during tile 0 is fine (its fragments were read in the prologue) ...
        w2.issue(6, 0, 0, last_read)          # ... but stage 1 is read during tile 0


@pytest.mark.parametrize("fname,prefix", [("gemm_nt_kernel.hip", "G_"), ("gemm_nt_fp8_kernel.hip", "H_")])
def test_sources_spell_out_the_waits_the_model_assumes(fname, prefix):
    src = open(os.path.join(CSRC, fname)).read()
    L = prefix + "LPG"
    for needle in ["wait_vmcnt<3 * %s>();" % L,
                   "if (EVEN) wait_vmcnt<2 * %s>(); else wait_vmcnt<2 * %s + 1>();" % (L, L),
                   "if (STEADY) wait_vmcnt<(%sAHEAD - 2) * %s>(); else wait_next_stage(j);" % (prefix, L),
                   "__builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0): this wave's reads of stage j are complete"]:
        assert needle in src, "%s no longer contains `%s`" % (fname, needle)
    # paired issue: stage j + 4 + parity, piece index from the slot number
    assert re.search(r"issue_piece_any\(j \+ 4 \+ \(", src)
