"""Model check of the kernel's LDS ring protocol against the paper's aref rules (Section 3.2, Fig. 4):
a slot is *put* only while empty, *got* only while full, and becomes empty again when every consumer
has signalled *consumed*.  The model replays, for one workgroup, what the two wave groups of
``attn_fwd_kernel`` do around each barrier (which stage they copy into, which stage their MFMA burst
reads) and asserts that no rule's premise is ever violated, for every tile count including those
smaller than the ring."""
import itertools

import pytest

STAGES = 4


class Slot:
    def __init__(self):
        self.full = False
        self.tile = None        # (k_tile, v_tile) held
        self.readers = 0        # outstanding gets not yet consumed

    def put(self, tile):
        assert not self.full and self.readers == 0, "put into a slot that is full or still being read"
        self.full, self.tile = True, tile

    def get(self, want):
        assert self.full, "get from an empty slot"
        assert self.tile == want, "slot holds %r, wanted %r" % (self.tile, want)
        self.readers += 1

    def consumed(self):
        assert self.readers > 0
        self.readers -= 1

    def release(self):
        assert self.readers == 0
        self.full = False


def stage_of(s):
    return (s + STAGES) % STAGES


def run_model(nt, nt_w_a, nt_w_b):
    """Stage s holds (K tile s+1, V tile s).  Copies of stage j+2 are issued after barrier j; group A's
    burst of iteration j reads stage j-1 (U_{j-1}, T_j), group B's reads stage j (U_j, T_{j+1})."""
    ring = [Slot() for _ in range(STAGES)]
    landed = {}
    log = []

    def issue(s):
        slot = ring[stage_of(s)]
        if slot.full:
            slot.release()          # legal only if nobody reads it: release() asserts that
        slot.put((s + 1, s))
        landed[s] = True

    for s in (-1, 0, 1):
        issue(s)
    # prologue barrier; group B's T_0 reads stage -1
    ring[stage_of(-1)].get((0, -1)); ring[stage_of(-1)].consumed()
    pending_a = None                # group A's reads of iteration j finish before barrier j+1
    for j in range(nt + 1):
        if j < nt:
            # barrier j: everybody's reads of earlier iterations are complete
            assert landed.get(j - 1) and landed.get(j), "barrier %d passed before its stages landed" % j
            if j + 2 < nt:
                issue(j + 2)        # overwrites stage j-2
        # group A: U_{j-1}, T_j from stage j-1
        do_u, do_t = j >= 1 and j - 1 < nt_w_a, j < nt_w_a
        if do_u or do_t:
            ring[stage_of(j - 1)].get((j, j - 1)); ring[stage_of(j - 1)].consumed()
            log.append(("A", j, do_u, do_t))
        # group B: C_j, then U_j, T_{j+1} from stage j
        if j < nt and j < nt_w_b:
            ring[stage_of(j)].get((j + 1, j)); ring[stage_of(j)].consumed()
            log.append(("B", j, True, j + 1 < nt_w_b))
    return log


@pytest.mark.parametrize("nt", list(range(1, 12)))
def test_ring_rules_hold_for_every_tile_count(nt):
    log = run_model(nt, nt, nt)
    # every tile's T and U happen exactly once per group
    for grp in "AB":
        us = sorted(j - 1 if grp == "A" else j for g, j, u, t in log if g == grp and u)
        assert us == list(range(nt))
    ta = sorted(j for g, j, u, t in log if g == "A" and t)
    tb = sorted(j + 1 for g, j, u, t in log if g == "B" and t)
    assert ta == list(range(nt)) and tb == list(range(1, nt))   # group B's T_0 is the prologue


@pytest.mark.parametrize("nt,a,b", [(nt, a, b) for nt in (1, 2, 5, 9) for a, b in itertools.product(range(1, nt + 1), repeat=2) if a <= b])
def test_ring_rules_hold_with_causal_idle_tails(nt, a, b):
    run_model(nt, a, b)


def test_model_catches_a_too_shallow_ring():
    global STAGES
    old = STAGES
    STAGES = 3
    try:
        with pytest.raises(AssertionError):
            run_model(6, 6, 6)
    finally:
        STAGES = old
