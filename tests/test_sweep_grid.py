"""Host logic of the schedule-parameter sweep: the grids contain the compiled-in defaults, the default
point is enumerated first (the run step takes its output as the reference), names are unique and every
knob of a grid exists in the HIP sources with the default the sweep assumes."""
import os
import re

from paper_2510_14719_amd import sweep

CSRC = os.path.join(os.path.dirname(os.path.abspath(sweep.__file__)), "csrc")


def test_default_point_first_and_names_unique():
    for op, grid in sweep.GRIDS.items():
        pts = sweep.grid_points(op)
        n = 1
        for vals in grid.values():
            n *= len(vals)
        if op == "attn_schedule":       # the knobs of the in-wave kernel only vary where that kernel is selected
            n = 1 + 4 + 1               # the default, eight waves x (interleave, window), four waves
        assert len(pts) == n
        assert all(pts[0][k] == sweep.DEFAULTS[k] for k in grid)
        names = [sweep.variant_name(op, p) for p in pts]
        assert len(set(names)) == n
        assert all(re.fullmatch(r"[a-z0-9_\-]+", x) for x in names)


def test_knobs_exist_in_sources_with_the_assumed_defaults():
    text = "".join(open(os.path.join(CSRC, f)).read() for f in os.listdir(CSRC) if f.endswith((".hip", ".h", ".cpp")))
    for knob, default in sweep.DEFAULTS.items():
        m = re.search(r"#ifndef %s\s*\n#define %s (\d+)" % (knob, knob), text)
        assert m, "knob %s is not an overridable #define of the sources" % knob
        assert int(m.group(1)) == default, knob


def test_the_variants_the_gpu_test_loads_are_non_default_grid_points():
    for op, pts in sweep.TEST_VARIANTS.items():
        assert len(pts) >= 2 or len(sweep.GRIDS[op]) == 1 and len(next(iter(sweep.GRIDS[op].values()))) == 2
        names = {sweep.variant_name(op, p) for p in sweep.grid_points(op)}
        for p in pts:
            assert sweep.variant_name(op, p) in names
            assert not all(p[k] == sweep.DEFAULTS[k] for k in p)
