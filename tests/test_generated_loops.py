"""The generated instruction streams (csrc/gen_attn_loop.py, csrc/gen_attn_bwd_loop.py) obey the rules the
hardware does not enforce, checked on the emitted text itself (asm_emit.check_stream): every register filled
by an LDS read is covered by an s_waitcnt before its first use, MFMA results are not touched by the VALU
within 11 wait states, VALU results not read by an MFMA within 2, transcendental results not used by the
next instruction, one wait state between a scalar write of m0 and a direct global->LDS load.  The main path
is walked through the first iteration and twice round the four loop bodies (loop-carried distances), and
once through every out-of-line section (mask pre-pass, exact-maximum pass, ragged loads, the last iteration
of each ring phase, the single-tile exit).  Also: the library build's
generated files are exactly what the generators emit, with or without stray environment variables."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2512_18134_amd", "csrc")
sys.path.insert(0, CSRC)

import asm_emit  # noqa: E402
import gen_attn_bwd_loop  # noqa: E402
import gen_attn_loop  # noqa: E402

FWD = [(name, dt) for name in gen_attn_loop.CONFIGS for dt in ("bf16", "f16")]


def fwd_lines(name, dtype="bf16"):
    g = gen_attn_loop.Gen(name, dtype=dtype)
    g.generate()
    return [l.replace("%=", "") for l in g.lines]


@pytest.mark.parametrize("name,dtype", FWD)
def test_forward_main_path_twice_round(name, dtype):
    lines = fwd_lines(name, dtype)
    path = asm_emit.walk(lines, loop_label="BODY0_", loop_visits=2)
    n_mfma = sum(1 for l in path if l.startswith("v_mfma"))
    g = gen_attn_loop.Gen(name)
    # the first iteration (K Q^T only), bodies 1..3, then two full rounds of the four bodies
    assert n_mfma == g.NQKG * g.QB + 11 * g.NM
    assert asm_emit.check_stream(path) == len(path)


def clamped_loads(g, tag):
    """Branches an iteration takes when its loads are the clamped ones: out of line from the first load slot
    (all of them at once when every load has a slot of its own, K then V otherwise), past the other slots."""
    if g.LS == 0:
        return ["KSLOW%s_" % tag, "VSLOW%s_" % tag]
    return ["KSLOW%s_" % tag] + ["LD%d_%s_" % (n, tag) for n in range(1, 2 * g.NLD)]


@pytest.mark.parametrize("name", list(gen_attn_loop.CONFIGS))
@pytest.mark.parametrize("b", range(4))
def test_forward_out_of_line_sections(name, b):
    lines = fwd_lines(name)
    g = gen_attn_loop.Gen(name)
    # each detour is taken the first time its branch is met (body b of the first round; the bodies are
    # alike, so b = 1..3 also cover a detour with loop-carried state before it), then the loop goes on
    for detour in (["SLOW%d_" % b], ["SPECIAL%d_" % b] + clamped_loads(g, b),
                   ["SPECIAL%d_" % b, "NOMASK%d_" % b] + clamped_loads(g, b)):
        path = asm_emit.walk(lines, take=detour, loop_label="BODY0_", loop_visits=2)
        assert asm_emit.check_stream(path) == len(path)
        assert sum(1 for l in path if l.startswith("v_mfma")) == g.NQKG * g.QB + 11 * g.NM
    # the last iteration (with and without the mask pre-pass and the exact-maximum pass) ends the loop:
    # P V of the tile before, then P V of the last tile
    for detour in (["SPECIAL%d_" % b, "TOPL%d_" % b, "DONE_"], ["SPECIAL%d_" % b, "NOMASK%d_" % b, "TOPL%d_" % b, "DONE_"],
                   ["SPECIAL%d_" % b, "TOPL%d_" % b, "SLOWL%d_" % b, "DONE_"]):
        path = asm_emit.walk(lines, take=detour, loop_label="BODY0_", loop_visits=2)
        assert asm_emit.check_stream(path) == len(path)
        assert path[-1].startswith("s_nop") and any(l.startswith("s_mov_b32 m0, s") for l in path[-4:])
        tail = [l for l in path if l.startswith("v_mfma")][-2 * g.NPVG * g.QB:]
        after = path[max(k for k, l in enumerate(path) if l == "s_barrier"):]
        assert all(", 0" not in l for l in tail) and not any(l.startswith("global_load_lds") for l in after)


@pytest.mark.parametrize("name", list(gen_attn_loop.CONFIGS))
def test_forward_first_iteration_and_single_tile(name):
    lines = fwd_lines(name)
    g = gen_attn_loop.Gen(name)
    for detour in (["SLOWF_"], ["SPECIALF_"] + clamped_loads(g, "F"), ["SPECIALF_", "NOMASKF_"] + clamped_loads(g, "F")):
        path = asm_emit.walk(lines, take=detour, loop_label="BODY0_", loop_visits=1)
        assert asm_emit.check_stream(path) == len(path)
    # a launch with one tile: the first iteration (its loads clamped), then straight to P(0) V(0)
    path = asm_emit.walk(lines, take=["SPECIALF_", "SLOWF_"] + clamped_loads(g, "F") + ["SPECIAL1_", "EXIT1_", "DONE_"])
    assert asm_emit.check_stream(path) == len(path)
    assert sum(1 for l in path if l.startswith("v_mfma")) == (g.NQKG + g.NPVG) * g.QB
    assert path[-1].startswith("s_nop") and any(l.startswith("s_mov_b32 m0, s") for l in path[-4:])


@pytest.mark.parametrize("name", list(gen_attn_loop.CONFIGS))
def test_forward_load_slots_see_the_flag_the_iteration_started_with(name):
    """SCC is set once per iteration (loads reach past S_kv or not) and read by every load slot: nothing
    between the top of the iteration and the last load slot may write it, every path issues each of the
    iteration's 2 NLD direct loads exactly once, and the out-of-line loads come back with the flag set."""
    lines = [l.strip() for l in fwd_lines(name)]
    g = gen_attn_loop.Gen(name)
    keeps_scc = ("s_waitcnt", "s_nop", "s_barrier", "s_mov_b32", "s_cbranch_scc1")
    for tag in ("F", "0", "1", "2", "3"):
        top = lines.index("TOP%s_:" % tag)
        slot_labels = ["KRET%s_:" % tag] + (["VRET%s_:" % tag] if g.LS == 0 else
                                            ["LD%d_%s_:" % (n, tag) for n in range(1, 2 * g.NLD)])
        end = max(lines.index(l) for l in slot_labels)
        region = [l for l in lines[top:end] if not l.endswith(":")]
        for l in region:
            assert not l.startswith("s_") or l.split()[0] in keeps_scc, l
        assert sum(l.startswith("s_cbranch_scc1") for l in region) == len(slot_labels)
        assert sum(l.startswith("global_load_lds") for l in region) == 2 * g.NLD
        # the clamped loads: one iteration through them, counted between its barrier and the next
        path = asm_emit.walk(lines, take=["SPECIAL%s_" % tag] + clamped_loads(g, tag), loop_label="BODY0_", loop_visits=2)
        slow = lines.index("KSLOW%s_:" % tag)
        k = next(i for i, l in enumerate(path) if l == lines[slow + 1] and path[i:i + 3] == lines[slow + 1:slow + 4])
        before = max(i for i in range(k) if path[i] == "s_barrier")
        after = min(i for i in range(k, len(path)) if path[i] == "s_barrier" or i == len(path) - 1)
        assert sum(l.startswith("global_load_lds") for l in path[before:after]) == 2 * g.NLD
        ret = lines.index("s_branch KRET%s_" % tag, slow)
        assert lines[ret - 1].startswith("s_cmp_ge_i32 s%d, s%d" % (g.s_j, g.s_tload))


def scalar_run(g, lines, n, n_wave, t_full, j_mask):
    """Barriers and direct loads of one wave's run through the loop, by barrier interval."""
    sg = {g.s_ntiles: n, g.s_nw: n_wave, g.s_tfull: t_full, g.s_jmask: j_mask, g.s_skvm1: max(t_full, 1) * g.BN - 1,
          g.s_ldsk: 1 << 20, g.s_ldsv: 1 << 21, g.s_kbase: 0, g.s_vbase: 0}
    ev = asm_emit.run_scalar(lines, sg, g.BN, g.TB, {"k": (g.s_kbase, g.s_kptr), "v": (g.s_vbase, g.s_vptr)})
    intervals = []
    for e in ev:
        if e[0] == "barrier":
            intervals.append([])
        else:
            assert intervals, "a load before the first barrier"
            intervals[-1].append(e[1:])
    return intervals


@pytest.mark.parametrize("name", list(gen_attn_loop.CONFIGS))
def test_forward_wave_without_rows_for_the_last_tiles_keeps_step(name):
    """Causal launches: a wave whose rows end before the workgroup's tiles do stops computing after its own
    last tile.  Whatever its tile count, it meets the same number of barriers as a wave that computes every
    tile (one per tile: anything else hangs the workgroup), and between the same two barriers it issues the
    same direct loads (tensor, tile, ring stage), so that the other waves find their operands."""
    g = gen_attn_loop.Gen(name)
    g.generate()
    lines = [l.replace("%=", "") for l in g.lines]
    for n in (1, 2, 3, 4, 5, 6, 7, 9, 13):
        for t_full in (n, n - 1):
            for j_mask in sorted({0, n // 2, n - 1, n}):
                full = scalar_run(g, lines, n, n, t_full, j_mask)
                assert len(full) == n
                for j, loads in enumerate(full):     # iteration j brings K(j+4) and V(j+2), the last one nothing
                    want = [("k", j + 4, j % 4)] * g.NLD + [("v", j + 2, (j + 2) % 4)] * g.NLD
                    if j == n - 1 and n > 1:         # (the first iteration is not specialised: it always loads)
                        want = []
                    got = sorted((w, t, ((a - ((1 << 20) if w == "k" else (1 << 21))) // g.TB)) for w, t, a in loads)
                    assert got == sorted(want), (n, t_full, j_mask, j)
                for n_wave in range(1, n):
                    part = scalar_run(g, lines, n, n_wave, t_full, j_mask)
                    assert len(part) == n, (n, n_wave, t_full, j_mask)
                    assert [sorted(x) for x in part] == [sorted(x) for x in full], (n, n_wave, t_full, j_mask)


@pytest.mark.parametrize("name", list(gen_attn_loop.CONFIGS))
def test_forward_early_finish_sections_obey_the_hazard_rules(name):
    lines = fwd_lines(name)
    g = gen_attn_loop.Gen(name)
    for b in range(4):
        # the wave's last tile in ring phase b and its owed loads, then three iterations of standing by: two
        # with loads, one without
        path = asm_emit.walk(lines, take=["SPECIAL%d_" % b, "TOPL%d_" % b, "OWED%d_" % b, "STANDBYNEXT_"],
                             loop_label="STANDBY_", loop_visits=3)
        assert asm_emit.check_stream(path) == len(path)
        tail = path[[i for i, l in enumerate(path) if l.startswith("s_branch AFTERLAST_")][0]:]
        assert sum(l == "s_barrier" for l in tail) == 3
        assert sum(l.startswith("global_load_lds") for l in tail) == 2 * 2 * g.NLD
    # a wave with rows for the first tile only
    path = asm_emit.walk(lines, take=["SPECIALF_"] + clamped_loads(g, "F") + ["SPECIAL1_", "EXIT1_"],
                         loop_label="STANDBY_", loop_visits=2)
    assert asm_emit.check_stream(path) == len(path)


BWD = [(ko, d, dt) for ko in (True, False) for d in (64, 128) for dt in ("bf16", "f16")]


@pytest.mark.parametrize("key_owner,d,dtype", BWD)
def test_backward_sweeps(key_owner, d, dtype):
    g = gen_attn_bwd_loop.Gen(key_owner, d, dtype=dtype)
    g.generate()
    lines = [l.replace("%=", "") for l in g.lines]
    path = asm_emit.walk(lines, loop_label="BODY0_", loop_visits=2)
    assert sum(1 for l in path if l.startswith("v_mfma")) == 2 * g.NST * g.NM
    assert asm_emit.check_stream(path) == len(path)
    for b in range(g.NST):
        for detour in (["MASKLO%d_" % b], ["MASKHI%d_" % b], ["SLOW%d_" % b], ["MASKLO%d_" % b, "MASKHI%d_" % b, "SLOW%d_" % b],
                       ["EXIT%d_" % b]):
            path = asm_emit.walk(lines, take=detour, loop_label="BODY0_", loop_visits=2)
            assert asm_emit.check_stream(path) == len(path)


def test_checker_catches_planted_mistakes():
    lines = fwd_lines("d128")
    path = asm_emit.walk(lines, loop_label="BODY0_", loop_visits=2)
    # a wait removed: the fragment of the next MFMA is then read while its LDS read is in flight
    i = [k for k, l in enumerate(path) if l.startswith("s_waitcnt lgkmcnt")][5]
    with pytest.raises(AssertionError):
        asm_emit.check_stream(path[:i] + path[i + 1:])
    # a VALU read of a score block moved right behind the MFMA that produces it
    k = [k for k, l in enumerate(path) if l.startswith("v_mfma") and ", 0" not in l and "v[128:143]" in l.split(",")[0]]
    with pytest.raises(AssertionError):
        asm_emit.check_stream(path[:k[0] + 1] + ["v_add_f32 v250, v128, v128"] + path[k[0] + 1:])
    # the filler between an m0 write and its load removed
    j = [k for k, l in enumerate(path) if l.startswith("global_load_lds")][0]
    with pytest.raises(AssertionError):
        asm_emit.check_stream(path[:j - 1] + path[j:])
    # exp result consumed by the very next instruction
    x = [k for k, l in enumerate(path) if l.startswith("v_exp_f32")][0]
    dst = path[x].split()[1].rstrip(",")
    with pytest.raises(AssertionError):
        asm_emit.check_stream(path[:x + 1] + ["v_add_f32 v250, %s, %s" % (dst, dst)] + path[x + 1:])


def test_build_output_is_the_generators_output_and_ignores_the_environment(tmp_path):
    from paper_2512_18134_amd import build
    env = dict(os.environ, ATTN_GEN_EXP="novalu", ATTN_GEN_BWD_EXP="nolds", ATTN_GEN_TAU="3", ATTN_GEN_PFD="2")
    code = ("import sys; sys.path.insert(0, %r)\nfrom paper_2512_18134_amd import build\n"
            "build.generate_sources(out_dir=%r)\n" % (ROOT, str(tmp_path)))
    subprocess.run([sys.executable, "-c", code], check=True, env=env)
    committed = os.path.join(CSRC, "generated")
    names = sorted(os.listdir(str(tmp_path)))
    assert names == sorted(f for f in os.listdir(committed) if f.endswith(".inc")) and len(names) >= 17
    for fn in names:
        assert open(os.path.join(str(tmp_path), fn)).read() == open(os.path.join(committed, fn)).read(), fn
