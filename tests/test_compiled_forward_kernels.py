"""Checks on the compiled forward kernels (hipcc -S of csrc/attn_fwd.hip).

1. The forward kernels that load Q straight into registers do so with asm statements the compiler cannot see
into (csrc/attn_fwd_asm.h: one hand-placed s_waitcnt covers them, so that the wait for Q is not a wait for
every K/V tile behind it).  The compiler therefore believes the destination registers are valid at once.  This
test compiles the forward source to gfx950 assembly and follows every path from those loads: no instruction
may touch a destination register before a vector-memory wait that covers the loads has been passed.

2. The code around the hand-scheduled loop must not spill vector registers to scratch memory: a reload is followed
by a wait for every load in flight, the K/V tiles of the stream included, which costs the short launches a quarter
of their time.  (The 8-wave D = 128 loop assigns all 256 VGPRs itself; the few spills around it are known.)"""
import os
import re
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
RANGE = re.compile(r"\bv\[(\d+):(\d+)\]|\bv(\d+)\b")
MAX_TILE_LOADS = 20   # a wait for at most this many loads in flight is one of the kernel's waits behind the Q loads


def vgprs(text):
    out = set()
    for m in RANGE.finditer(text):
        if m.group(1):
            out.update(range(int(m.group(1)), int(m.group(2)) + 1))
        else:
            out.add(int(m.group(3)))
    return out


def kernels_of(asm_text):
    """{kernel name: [instructions and labels]} of the attn_fwd_asm_kernel instantiations."""
    out, cur = {}, None
    for line in asm_text.split("\n"):
        m = re.match(r"^(_ZN4attn19attn_fwd_asm_kernel\S+):", line)
        if m:
            cur = m.group(1)
            out[cur] = []
            continue
        if cur is None:
            continue
        if line.startswith(".Lfunc_end"):
            cur = None
            continue
        s = line.split(";")[0].strip()
        if s and (not s.startswith(".") or s.endswith(":")):
            out[cur].append(s)
    return out


def touched_before_wait(ins):
    """Instructions that read or write a register with an asm Q load in flight, on any path."""
    label = {s[:-1]: i for i, s in enumerate(ins) if s.endswith(":")}
    state = [None] * len(ins)
    work, bad, n_loads = [(0, frozenset())], set(), 0
    while work:
        i, pend = work.pop()
        while i < len(ins):
            if state[i] is not None and pend <= state[i]:
                break
            state[i] = pend if state[i] is None else state[i] | pend
            pend = state[i]
            s = ins[i]
            if s.endswith(":"):
                i += 1
                continue
            op = s.split()[0]
            if op == "global_load_dwordx4" and s.split()[1].startswith("v["):
                pend = pend | frozenset(vgprs(s.split(",")[0]))
                n_loads += 1
            elif op == "s_waitcnt" and "vmcnt" in s:
                if int(re.search(r"vmcnt\((\d+)\)", s).group(1)) <= MAX_TILE_LOADS:
                    pend = frozenset()
            elif pend and not op.startswith("global_load_lds") and vgprs(s) & pend:
                bad.add((i, s))
            if op == "s_branch":
                i = label[s.split()[1]]
                continue
            if op.startswith("s_cbranch"):
                work.append((label[s.split()[1]], pend))
            if op == "s_endpgm":
                break
            i += 1
    return sorted(bad), n_loads


def test_checker_sees_a_planted_early_use():
    ins = ["global_load_dwordx4 v[4:7], v[0:1], off offset:0", "s_cbranch_scc1 L1", "v_mov_b32 v9, v8",
           "L1:", "s_waitcnt vmcnt(4)", "v_mov_b32 v9, v5", "s_endpgm"]
    assert touched_before_wait(ins) == ([], 1)
    early = ins[:3] + ["v_mov_b32 v10, v6"] + ins[3:]
    assert [s for _, s in touched_before_wait(early)[0]] == ["v_mov_b32 v10, v6"]
    # a wait for the compiler's own loads only (many tile loads may still be in flight) does not count
    weak = [s.replace("vmcnt(4)", "vmcnt(40)") for s in ins]
    assert [s for _, s in touched_before_wait(weak)[0]] == ["v_mov_b32 v9, v5"]


@pytest.fixture(scope="module", params=["product", "debug"])
def compiled(request, tmp_path_factory):
    """Assembly text of attn_fwd.hip, built like the product library or like the debug library."""
    from paper_2512_18134_amd import build
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("hipcc is not installed")
    out = str(tmp_path_factory.mktemp(request.param) / "fwd.s")
    flags = [f for f in build.HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    if request.param == "debug":
        flags.append("-DATTN_DEBUG_ENTRY_POINTS")
    src = os.path.join(ROOT, "paper_2512_18134_amd", "csrc", "attn_fwd.hip")
    subprocess.run([hipcc] + flags + ["-S", "--cuda-device-only", "-o", out, src], check=True,
                   stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
    return open(out).read()


def test_no_scratch_around_the_hand_scheduled_loops(compiled):
    meta = compiled[compiled.index("amdhsa.kernels:"):]
    seen = 0
    for block in meta.split("  - .agpr_count:")[1:]:
        name = re.search(r"\.name:\s+(\S+)", block).group(1)
        m = re.search(r"attn_fwd_asm_kernelILi(\d+)ELi(\d)ELi(\d)ELi(\d)E", name)
        if not m:
            continue
        d, qb, sb, nw = (int(x) for x in m.groups())
        scratch = int(re.search(r"\.private_segment_fixed_size:\s+(\d+)", block).group(1))
        spills = int(re.search(r"\.vgpr_spill_count:\s+(\d+)", block).group(1))
        if d == 64 and nw == 4:
            # two of these workgroups share a CU: a wave may use half a SIMD's registers (VGPRs + AGPRs)
            assert int(re.search(r"\.vgpr_count:\s+(\d+)", block).group(1)) <= 256, name
        if d == 128 and qb == 1:
            assert scratch <= 64, (name, scratch)      # the loop that leaves the compiler no VGPR
        else:
            assert scratch == 0 and spills == 0, (name, scratch, spills)
        seen += 1
    assert seen >= 20


def test_no_use_of_q_registers_before_the_wait(compiled):
    kernels = kernels_of(compiled)
    assert len(kernels) >= 20                      # every tiling, causal or not, both element types, split-KV
    with_asm_loads = 0
    for name, ins in kernels.items():
        bad, n_loads = touched_before_wait(ins)
        assert not bad, (name, bad[:5])
        with_asm_loads += n_loads > 0
    assert with_asm_loads >= 8                     # the tilings without an LDS staging area for Q
