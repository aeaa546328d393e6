"""Host-side checks of the generated assembly loop of the 64-rows-per-wave attention kernel
(``csrc/gen_attn_mb2_loop.py`` -> ``csrc/attn_mb2_loop.inc``): it assembles for gfx950, the committed include
file is what the generator writes, it only writes the registers its contract names, a word of P is rewritten
only after the last MFMA that reads it, and its scalar address arithmetic -- emulated here instruction by
instruction -- keeps every global -> LDS copy inside the sequence and inside the LDS ring, issues one barrier
per pass and terminates, for sequences of whole tiles and ragged ones."""
import importlib.util
import os
import re
import shutil
import subprocess

import pytest

CSRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2510_14719_amd", "csrc")


@pytest.fixture(scope="module")
def gen():
    spec = importlib.util.spec_from_file_location("gen_attn_mb2_loop", os.path.join(CSRC, "gen_attn_mb2_loop.py"))
    g = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(g)
    return g


def test_committed_include_file_is_current(gen, tmp_path):
    out = tmp_path / "loop.inc"
    gen.write_inc(str(out))
    assert out.read_text() == open(os.path.join(CSRC, "attn_mb2_loop.inc")).read(), \
        "attn_mb2_loop.inc is stale: run python paper_2510_14719_amd/csrc/gen_attn_mb2_loop.py"


@pytest.mark.parametrize("el", ["f16", "bf16"])
def test_loop_assembles_for_gfx950(gen, el):
    mc = "/opt/rocm/llvm/bin/llvm-mc"
    if not os.path.exists(mc):
        mc = shutil.which("llvm-mc")
    if not mc:
        pytest.skip("no llvm-mc in this environment")
    text = "\n".join(gen.gen_loop(el, "t")) + "\n"
    res = subprocess.run([mc, "-arch=amdgcn", "-mcpu=gfx950", "-filetype=null"], input=text, text=True,
                         stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
    assert res.returncode == 0 and "error" not in res.stdout, res.stdout[:2000]


def _regs(tok):
    m = re.match(r"^([vsa])\[(\d+):(\d+)\]$", tok)
    if m:
        return m.group(1), range(int(m.group(2)), int(m.group(3)) + 1)
    m = re.match(r"^([vsa])(\d+)$", tok)
    if m:
        return m.group(1), [int(m.group(2))]
    return None, []


@pytest.mark.parametrize("el", ["f16", "bf16"])
def test_loop_writes_only_the_registers_of_its_contract(gen, el):
    written = {"v": set(), "s": set(), "a": set()}
    for l in gen.gen_loop(el, "t"):
        if l.endswith(":") or l.split()[0] in ("s_waitcnt", "s_barrier", "s_nop", "s_branch", "s_cbranch_scc1", "s_cmp_gt_i32",
                                               "s_cmp_lg_u64", "global_load_lds_dwordx4"):
            continue
        dst = l.partition(" ")[2].split(",")[0].strip()
        c, r = _regs(dst)
        if c:
            written[c].update(r)
        else:
            assert dst in ("vcc", "m0"), l
    in_out_v = set(range(0, 164))                     # S, P, the softmax state
    assert written["v"] <= in_out_v | set(gen.CLOBBER_V)
    assert not written["v"] & {200, 201, 202, 203}, "the per-lane offsets are inputs"
    assert written["s"] <= {40, 46} | set(gen.CLOBBER_S)
    assert written["a"] <= set(range(0, 128)), "only O is accumulated; Q (a128..a191) is read"


@pytest.mark.parametrize("el", ["f16", "bf16"])
def test_p_words_are_rewritten_after_their_last_reader(gen, el):
    """A word of P (v128..v159) is the B operand of U's MFMAs and the destination of the pass's conversions."""
    for par in (0, 1):
        last_read, written_at = {}, {}
        for i, l in enumerate(gen.gen_pass(par, el, "t")):
            if l.startswith("v_mfma") and "a[" in l.split(",")[0]:          # U: accumulates into O
                _, r = _regs(l.split(",")[2].strip())
                for x in r:
                    last_read[x] = i
            elif l.startswith("v_cvt_pk"):
                _, r = _regs(l.partition(" ")[2].split(",")[0].strip())
                for x in r:
                    written_at[x] = i
        assert set(written_at) == set(range(128, 160)) == set(last_read)
        assert all(written_at[x] > last_read[x] for x in written_at)


def _emulate(lines, N, wave, j0, j_end):
    """The scalar side of the loop: returns (final SGPRs, copies as (j, global base, LDS address, lane-offset register), barriers)."""
    labels = {l[:-1]: i for i, l in enumerate(lines) if l.endswith(":")}
    KBASE, VBASE = 0x10000000, 0x20000000
    s = {36: KBASE, 37: 0, 38: VBASE, 39: 0, 40: j0, 41: j_end, 43: 0, 44: wave, 45: N}
    scc = m0 = pc = barriers = steps = 0
    copies = []

    def val(t):
        t = t.strip()
        if re.match(r"^s\d+$", t):
            return s[int(t[1:])]
        return int(t, 0) & 0xffffffff

    def sgn(x):
        return x - (1 << 32) if x & 0x80000000 else x

    while pc < len(lines):
        steps += 1
        assert steps < 400000, "the loop does not terminate"
        l = lines[pc]
        pc += 1
        if l.endswith(":"):
            continue
        op, _, rest = l.partition(" ")
        a = [x.strip() for x in rest.split(",")]
        if op == "s_add_i32":
            s[int(a[0][1:])] = (sgn(val(a[1])) + sgn(val(a[2]))) & 0xffffffff
        elif op == "s_add_u32":
            t = val(a[1]) + val(a[2]); scc = t >> 32; s[int(a[0][1:])] = t & 0xffffffff
        elif op == "s_addc_u32":
            t = val(a[1]) + val(a[2]) + scc; scc = t >> 32; s[int(a[0][1:])] = t & 0xffffffff
        elif op == "s_and_b32":
            s[int(a[0][1:])] = val(a[1]) & val(a[2])
        elif op == "s_lshl_b32":
            s[int(a[0][1:])] = (val(a[1]) << val(a[2])) & 0xffffffff
        elif op == "s_min_i32":
            s[int(a[0][1:])] = min(sgn(val(a[1])), sgn(val(a[2]))) & 0xffffffff
        elif op == "s_mov_b32":
            if a[0] == "m0":
                m0 = val(a[1])
            else:
                s[int(a[0][1:])] = val(a[1])
        elif op == "s_cmp_gt_i32":
            scc = int(sgn(val(a[0])) > sgn(val(a[1])))
        elif op == "s_cmp_lg_u64":
            scc = 0                                  # no overflow of the row sums in this emulation
        elif op == "s_cbranch_scc1":
            if scc:
                pc = labels[a[0]]
        elif op == "s_branch":
            pc = labels[a[0]]
        elif op == "global_load_lds_dwordx4":
            m = re.match(r"s\[(\d+):(\d+)\]", a[1])
            copies.append((s[40], s[int(m.group(1))] | (s[int(m.group(2))] << 32), m0, a[0]))
        elif op == "s_barrier":
            barriers += 1
        else:
            assert op.startswith(("s_or_b64", "s_waitcnt", "s_nop", "v_", "ds_")), l
    return s, copies, barriers


@pytest.mark.parametrize("N", [129, 192, 256, 577, 1000, 2309, 4096, 16384])
def test_scalar_address_arithmetic(gen, N):
    lines = gen.gen_loop("f16", "t")
    nt = (N + 63) // 64
    j_end = nt - 2
    for wave in range(4):
        for j0 in [j for j in (1, 3, max(1, (j_end // 2) | 1)) if j <= j_end]:
            s, copies, barriers = _emulate(lines, N, wave, j0, j_end)
            assert s[40] == j_end + 1 and s[46] == 0, "leaves with j = j_end + 1 and no redo"
            assert barriers == j_end - j0 + 1, "one barrier per pass"
            assert len(copies) == 8 * barriers, "eight copies per pass"
            for (j, base, lds, lane_reg) in copies:
                is_k = lane_reg == "v202"
                off = base - (0x10000000 if is_k else 0x20000000)
                # a piece is 16 rows x 64 B of the source: the lanes add up to 15 rows and 3 columns of 16 B
                assert 0 <= off and off + 15 * 256 + 3 * 16 + 16 <= N * 256, ("copy outside the sequence", N, wave, j, off, is_k)
                assert 0 <= lds and lds + 1024 <= 4 * 32768, ("copy outside the LDS ring", lds)
                # the stage written is j + 2, the K half first
                assert lds // 32768 == (j + 2) % 4 and ((lds % 32768) >= 16384) == (not is_k)
