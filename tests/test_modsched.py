"""The modulo-scheduling model against the paper's running example (Section 3.1, Fig. 1)
and on the measured gfx950 costs."""
import math

from paper_2512_18134_amd import modsched as ms


def test_paper_running_example():
    g = ms.paper_toy()
    M, I, L = ms.schedule(g)
    # the paper's figure: initiation interval 2, schedule length 4
    assert (I, L) == (2, 4)
    assert ms.is_valid(g, M, I)
    # in order: one iteration every 3 cycles; pipelined: one every 2 after the prologue
    assert ms.in_order_interval(g) == 3
    # the single-iteration optimum M(P)=1, M(O)=2 respects the dependences but O collides
    # with S on the tensor core (0 = 2 mod 2): exactly the paper's remark
    bad = {"S": 0, "P": 1, "O": 2}
    assert all(bad[v] + I * dl >= bad[u] + d for u, v, d, dl in g.edges)
    assert not ms.is_valid(g, bad, I)
    # the schedule the paper draws (P and O each one cycle later than that optimum) is valid
    assert ms.is_valid(g, {"S": 0, "P": 2, "O": 3}, 2)
    # I = 1 is impossible: two tensor-core instructions per iteration on one tensor core
    assert ms.res_mii(g) == 2
    assert ms.optimal_modulo_schedule(g, 1, 8) is None


def test_prologue_steady_state_structure():
    g = ms.paper_toy()
    M = {"S": 0, "P": 2, "O": 3}
    code = ms.pipeline_code(g, M, 2)
    # ceil(L/I) = 2 overlapped copies, prologue of (2-1)*2 cycles that holds only S = gemm(Q, K[0])
    assert code["copies"] == 2 and code["prologue_cycles"] == 2
    assert [v for _, v, _ in code["prologue"]] == ["S"]
    # steady state: the new iteration's S next to the previous iteration's P, then its O (Fig. 1f)
    steady = {v: k for _, v, k in code["steady"]}
    assert steady == {"S": 0, "P": 1, "O": 1}
    table = ms.modular_rrt(g, M, 2)
    assert table[0] == {"TC": 1, "EXP": 1} and table[1] == {"TC": 1}


def test_recurrence_bound():
    g = ms.Loop({"U": 2})
    g.op("a", "U", 3)
    g.op("b", "U", 2)
    g.dep("a", "b")
    g.dep("b", "a", delta=1)     # cycle of total delay 5 over one iteration
    assert ms.rec_mii(g) == 5
    M, I, L = ms.schedule(g)
    assert I == 5 and ms.is_valid(g, M, I)


def test_cost_normalisation_keeps_ratios():
    C = [1000, 1000, 500, 250]
    Cn, F = ms.normalise_costs(C, 12)
    assert sum(Cn) <= 12 and Cn == [4, 4, 2, 1] and F == 0
    Cn, F = ms.normalise_costs([512, 790, 512], 10)
    assert sum(Cn) <= 10
    # ratios within 15 % of the originals at this coarse resolution
    assert abs(Cn[1] / Cn[0] - 790 / 512) < 0.25


def test_gfx950_attention_is_matrix_pipe_bound_with_three_stages():
    g, c, _ = ms.gfx950_attention(U=24)
    M, I, L = ms.schedule(g, max_len=4 * sum(c.values()))
    assert ms.is_valid(g, M, I)
    # both MFMA products of a tile back to back: the initiation interval is the matrix pipe's
    assert I == c["QK"] + c["PV"]
    # the softmax of a tile does not fit between its two products inside one interval:
    # the schedule spans three intervals (QK of tile j+1, softmax of j, PV of j-1 overlap)
    assert math.ceil(L / I) == 3
    assert ms.in_order_interval(g) >= 2 * I - 2


def test_memory_capacity_on_the_running_example():
    # Section 4.2 on Fig. 1: S lives until P has executed, P until O has, O is an accumulator updated in place
    g = ms.paper_toy()
    M, I = {"S": 0, "P": 2, "O": 3}, 2
    assert ms.live_ranges(g, M, I) == {"S": (0, 3), "P": (2, 4), "O": (3, 5)}
    # steady state, cycle 0: the new S, the previous iteration's S (P reads it now), that P (being written)
    # and O; cycle 1: S, P (O reads it now) and O
    use = ms.live_footprint(g, M, I, {"S": 1, "P": 1, "O": 1})
    assert use == [4, 3]
    assert ms.fits(g, M, I, {"S": 1, "P": 1, "O": 1}, capacity=4)
    assert not ms.fits(g, M, I, {"S": 1, "P": 1, "O": 1}, capacity=3)
    # the program-order loop peaks one lower: pipelining costs memory (the trade the paper's Section 6.3
    # finds decisive for the backward pass on Hopper)
    seq = {"S": 0, "P": 1, "O": 2}
    assert ms.live_footprint(g, seq, 3, {"S": 1, "P": 1, "O": 1}) == [2, 3, 2]


def _load_generator(name):
    import importlib.util
    import os
    import sys
    csrc = os.path.join(os.path.dirname(ms.__file__), "csrc")
    if csrc not in sys.path:
        sys.path.insert(0, csrc)          # the generators import asm_emit from their own directory
    path = os.path.join(csrc, name + ".py")
    spec = importlib.util.spec_from_file_location(name, path)
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_register_demand_matches_what_the_generators_allocate():
    # forward, D = 128: the three-stage schedule keeps two S blocks and two P blocks alive at times; with
    # the loop invariants that fits the 256 registers of a wave at two waves per SIMD
    g, c, _ = ms.gfx950_attention(U=24)
    M, I, L = ms.schedule(g, max_len=4 * sum(c.values()))
    ranges = ms.live_ranges(g, M, I)
    assert ranges["QK"][1] - ranges["QK"][0] > I       # S(j+1) is produced while S(j) is still being read
    assert ranges["SM"][1] - ranges["SM"][0] > I       # P(j) is produced while P(j-1) is still being read
    peak = max(ms.live_footprint(g, M, I, ms.GFX950_D128_REGS, ms.GFX950_D128_RESIDENT))
    gen = _load_generator("gen_attn_loop").Gen("d128")     # the 8-wave tiling: two waves per SIMD
    # the generator double-buffers S and P statically and allocates exactly what the model's values need
    assert gen.SBUF - gen.SA == 32 and gen.PB - gen.PA == 16
    static = 2 * 32 + 2 * 16 + 64 + ms.GFX950_D128_RESIDENT
    assert peak <= static <= 256 and abs(gen.NV - static) <= 8
    # the backward key-owner sweep: accumulators for dK and dV plus the owner's rows do not fit 256,
    # so it runs one wave per SIMD (512 registers, the accumulators in AGPRs)
    g, c, _ = ms.gfx950_backward_key_owner()
    M, I, L = ms.schedule(g, max_len=4 * sum(c.values()))
    peak_b = max(ms.live_footprint(g, M, I, ms.GFX950_BWD_REGS, ms.GFX950_BWD_RESIDENT))
    assert 256 < peak_b <= 512
    genb = _load_generator("gen_attn_bwd_loop").Gen(True, 128)
    assert abs((genb.NV + genb.NA) - (2 * 32 + 2 * 16 + 128 + ms.GFX950_BWD_RESIDENT)) <= 8


def test_slot_level_model_of_the_generated_loops():
    # Section 6.1: sub-tiled to single matrix instructions.  The generated streams issue one MFMA per slot, so
    # their initiation interval in slots is the number of MFMAs, which is the matrix pipe's resource bound;
    # whether a slot table is VALID (dependences, the 11-wait-state rule, LDS waits) is what
    # tests/test_generated_loops.py checks on the emitted text.  Here: the interval and the unit loads.
    gen = _load_generator("gen_attn_loop")
    wide, narrow = gen.Gen("d128a"), gen.Gen("d128")
    wide.generate()
    narrow.generate()
    mw, mn = ms.stream_mix(wide.lines), ms.stream_mix(narrow.lines)
    assert mw["mfma"] == wide.NM == 32 and mn["mfma"] == narrow.NM == 32
    # both tilings do the softmax of 32 scores per lane per 32 MFMAs; the wide one reads half the fragments
    assert mw["lds"] * 2 == mn["lds"] == 48 and abs(mw["valu"] - mn["valu"]) <= 4
    assert sum(mw.values()) == ms.GFX950_STREAM_INSTRS and abs(mw["valu"] - ms.GFX950_SOFTMAX_INSTRS) <= 2
    # one wave per SIMD: the wave's issue port is the binding unit when the chip is not power limited; the
    # model's matrix-pipe utilisation is the one measured on all-zero inputs (it was calibrated there) ...
    bw = ms.slot_level_bounds(mw, 1)
    assert bw["issue"] > bw["matrix"] and abs(bw["matrix_busy"] - ms.GFX950_UNTHROTTLED_BUSY) < 0.01
    # ... and with two such waves on a SIMD the matrix pipe becomes the binding unit: nothing the schedule
    # could still rearrange lowers the interval below one slot per MFMA
    bn = ms.slot_level_bounds(mn, 2)
    assert bn["matrix"] > bn["issue"] and bn["interval"] == 2 * 32 * ms.GFX950_MFMA_CYCLES
    # the counters of the headline run see the same mix: SQ_INSTS_VALU (which counts MFMAs) per SQ_INSTS_MFMA
    # = 4.64 including prologue and epilogue (profiles/all_configs.md)
    assert abs((mw["valu"] + mw["mfma"]) / mw["mfma"] - 4.64) < 0.1
    # sub-tiled tile-level graph (two query blocks): the interval stays the matrix-pipe bound; the schedule
    # shrinks from three overlapped copies to two (the softmax of block 0 can start while the scores of block
    # 1 are still being produced).  What finer instructions could still buy here is therefore registers (one
    # S / P buffer less), not throughput: I is already at its bound
    g, c, _ = ms.gfx950_attention_subtiled(U=16)
    M, I, L = ms.schedule(g, max_len=4 * sum(c.values()))
    assert I == sum(c[n] for n in c if n[:2] in ("QK", "PV"))
    g1, c1, _ = ms.gfx950_attention(U=16)
    M1, I1, L1 = ms.schedule(g1, max_len=4 * sum(c1.values()))
    print("sub-tiled: I=%d L=%d; tile level: I=%d L=%d" % (I, L, I1, L1))
    assert I == I1 and math.ceil(L / I) == 2 and math.ceil(L1 / I1) == 3


# ------------------------------------------------------------------ warp assignment (Section 4.3)
def _unrolled_ok(loop, M, I, A, ws):
    """The constraints of Sections 4.1-4.3 checked the way the paper writes them: on the unrolled
    schedule, instance (v, i) issuing at cycle M[v] + i*I.  Enough iterations are unrolled that one full
    interval [T0, T0 + I) sees every instance that can overlap it; capacity, registers and concurrency
    are checked there, dependences on every pair of instances.  Written independently of
    ms.is_valid_assignment (no modular arithmetic, no closed-form liveness)."""
    cyc = lambda v: max(1, len(loop.rrt[v]))
    max_delta = max([dl for _, _, _, dl in loop.edges] + [0])
    T0 = max(M.values()) + max(cyc(v) for v in M) + I * max_delta
    n_iter = (T0 + 2 * I) // I + 2 + max_delta
    start = {(v, i): M[v] + i * I for v in M for i in range(n_iter)}
    window = range(T0, T0 + I)
    # warp uniqueness / variable latency
    for v in M:
        if not (0 <= A[v] < ws.n_warps):
            return False
        if ws.variable_latency and ((v in ws.variable_latency) != (A[v] == 0)):
            return False
    # dependences, with the cross-warp transfer excluded cycle by cycle
    for u, v, d, delta in loop.edges:
        for i in range(n_iter - delta):
            t = start[(u, i)]
            if start[(v, i + delta)] < t + d:
                return False
            if A[u] != A[v]:
                for s_ in range(ws.spillcost.get(u, 0)):
                    if start[(v, i + delta)] == t + d + s_:
                        return False
    # functional-unit capacity, cycle by cycle
    for t in window:
        use = {}
        for (v, i), s0 in start.items():
            if s0 <= t < s0 + len(loop.rrt[v]):
                for unit, n in loop.rrt[v][t - s0].items():
                    use[unit] = use.get(unit, 0) + n
        if any(n > loop.capacity[unit] for unit, n in use.items()):
            return False
    # register limit per warp: a value is live from its issue until its last consumer has finished
    # (an accumulator updated in place hands over to its next instance when that one issues)
    if ws.reg_limit is not None:
        for w in range(ws.n_warps):
            for t in window:
                live = 0
                for (v, i), s0 in start.items():
                    if A[v] != w:
                        continue
                    end = s0 + cyc(v)
                    for a, b, d, delta in loop.edges:
                        if a == v:
                            sb = M[b] + (i + delta) * I
                            end = max(end, sb + (0 if b == v else cyc(b)))
                    if s0 <= t < end:
                        live += ws.regs.get(v, 0)
                if live > ws.reg_limit:
                    return False
    # concurrency: behind a blocking (or cross-warp) edge the consumer issues with its warp otherwise idle
    for u, v, _, _ in loop.edges:
        if (u, v) in ws.blocking or A[u] != A[v]:
            for (v2, i), t in start.items():
                if v2 != v or t not in window:
                    continue
                for (o, i2), s0 in start.items():
                    if o != v and A[o] == A[v] and t - (cyc(o) - 1) <= s0 <= t:
                        return False
    return True


def _brute_force_joint(loop, ws, max_len, max_interval):
    import itertools
    names = loop.order
    for I in range(1, max_interval + 1):
        best = None
        for starts in itertools.product(range(max_len), repeat=len(names)):
            M = dict(zip(names, starts))
            L = ms.length(loop, M)
            if L > max_len or (best is not None and L >= best):
                continue
            for warps in itertools.product(range(ws.n_warps), repeat=len(names)):
                if _unrolled_ok(loop, M, I, dict(zip(names, warps)), ws):
                    best = L
                    break
        if best is not None:
            return I, best
    return None


def _blocking_example():
    # Section 3.2's figure: an addition consumes a GEMM behind a blocking wait while an independent EXP
    # runs; all three on different functional units
    g = ms.Loop({"TC": 1, "EXP": 1, "ALU": 1})
    g.op("GEMM", "TC", 2)
    g.op("EXP", "EXP", 2)
    g.op("ADD", "ALU", 1)
    g.dep("GEMM", "ADD")
    return g


def test_blocking_synchronisation_pushes_work_to_another_warp_or_another_time():
    g = _blocking_example()
    blocking = [("GEMM", "ADD")]
    # no blocking edge: one warp sustains the tensor core's interval
    M, I, L, A = ms.joint_schedule(g, ms.Warps(1))
    assert I == 2 and len(set(A.values())) == 1
    # blocking wait, one warp: ADD may only issue while GEMM and EXP are not in flight -> another time,
    # and the interval grows
    M, I, L, A = ms.joint_schedule(g, ms.Warps(1, blocking=blocking))
    assert I == 3
    assert all((M["ADD"] - M[o]) % I >= ms.duration(g, o) for o in ("GEMM", "EXP"))
    # two warps: the consumer moves to the other warp and the interval is the tensor core's again
    M, I, L, A = ms.joint_schedule(g, ms.Warps(2, blocking=blocking))
    assert I == 2 and A["ADD"] != A["GEMM"] and A["ADD"] != A["EXP"]
    assert ms.is_valid_assignment(g, M, I, A, ms.Warps(2, blocking=blocking))


def test_joint_search_agrees_with_brute_force_on_the_unrolled_constraints():
    # small graphs, every (M, A) enumerated and checked with the literal, unrolled constraints
    cases = []
    g = _blocking_example()
    cases.append((g, ms.Warps(1, blocking=[("GEMM", "ADD")])))
    cases.append((g, ms.Warps(2, blocking=[("GEMM", "ADD")])))
    cases.append((g, ms.Warps(2, blocking=[("GEMM", "ADD")], spillcost={"GEMM": 2})))
    t = ms.paper_toy()
    cases.append((t, ms.Warps(2, blocking=[("S", "P"), ("P", "O")])))
    cases.append((t, ms.Warps(2, regs={"S": 2, "P": 2, "O": 2}, reg_limit=5, spillcost={"S": 1, "P": 1})))
    cases.append((t, ms.Warps(3, regs={"S": 2, "P": 2, "O": 2}, reg_limit=4, spillcost={"S": 1, "P": 1})))
    ld = ms.Loop({"TC": 1, "LSU": 1})
    ld.op("LOAD", "LSU", 1)
    ld.op("MMA", "TC", 2)
    ld.dep("LOAD", "MMA")
    ld.dep("MMA", "MMA", delta=1)
    cases.append((ld, ms.Warps(2, variable_latency=["LOAD"])))
    for loop, ws in cases:
        got = ms.joint_schedule(loop, ws, max_len=7, max_interval=7)
        want = _brute_force_joint(loop, ws, max_len=7, max_interval=7)
        assert (got is None) == (want is None)
        if got is not None:
            M, I, L, A = got
            assert (I, L) == want, (I, L, want)
            assert _unrolled_ok(loop, M, I, A, ws)


def test_variable_latency_operations_get_the_designated_warp_to_themselves():
    g = ms.Loop({"TC": 1, "LSU": 1, "EXP": 1})
    g.op("LOAD", "LSU", 1)
    g.op("MMA", "TC", 2)
    g.op("EXP", "EXP", 1)
    g.dep("LOAD", "MMA")
    g.dep("MMA", "EXP")
    ws = ms.Warps(3, variable_latency=["LOAD"], spillcost={"MMA": 2})
    M, I, L, A = ms.joint_schedule(g, ws)
    assert A["LOAD"] == 0 and A["MMA"] != 0 and A["EXP"] != 0
    assert A["MMA"] == A["EXP"]                  # a third warp would cost the transfer of MMA's result
    bad = dict(A, EXP=0)                          # a fixed-latency operation on W_vl is not allowed
    assert not ms.is_valid_assignment(g, M, I, bad, ws)
    # with a single warp there is no W_vl to give: unsatisfiable (Section 5.1 relaxes such problems)
    assert ms.joint_schedule(g, ms.Warps(1, variable_latency=["LOAD"]), max_interval=6) is None


def test_register_limit_forces_a_partition_and_the_transfer_is_paid():
    g = ms.paper_toy()
    regs = {"S": 100, "P": 100, "O": 100}
    # everything on one warp needs up to 400 registers at once (two S, P and O overlap, see above)
    one = ms.Warps(1, regs=regs, reg_limit=400)
    M, I, L, A = ms.joint_schedule(g, one)
    assert (I, L) == (2, 4)
    # 255 per warp: no single warp can hold it; spread over warps, every crossing edge pays the transfer
    ws = ms.Warps(3, regs=regs, reg_limit=255, spillcost={"S": 1, "P": 1})
    assert ms.joint_schedule(g, ms.Warps(1, regs=regs, reg_limit=255), max_interval=8) is None
    M, I, L, A = ms.joint_schedule(g, ws)
    assert len(set(A.values())) >= 2 and I == 2 and L >= 4
    assert ms.is_valid_assignment(g, M, I, A, ws) and _unrolled_ok(g, M, I, A, ws)
    for u, v, d, delta in g.edges:
        if A[u] != A[v]:
            assert M[v] + I * delta >= M[u] + d + ws.spillcost[u]


def test_gfx950_attention_needs_no_warp_specialisation():
    # The loop this library runs, with the measured gfx950 costs.  Its global->LDS loads are streaming
    # operations several tiles ahead (zero latency in the model, Section 5.3), MFMA results reach the VALU
    # through fixed-latency interlocks rather than blocking waits, and the three-stage schedule keeps every
    # wait satisfied before it is reached: no variable-latency operation, no blocking edge.
    g, c, _ = ms.gfx950_attention(U=12)
    regs = dict(ms.GFX950_D128_REGS)
    free = 256 - ms.GFX950_D128_RESIDENT
    plain = ms.schedule(g, max_len=4 * sum(c.values()))
    # handing S or P to another wavefront goes through LDS: a write and a read of the tile, about the cost
    # of the operand reads of one product in normalised cycles
    spill = {"QK": c["LDS_K"] + c["LDS_V"], "SM": c["LDS_K"] + c["LDS_V"], "LDS_K": 1, "LDS_V": 1}
    M, I, L, A = ms.joint_schedule(g, ms.Warps(2, regs=regs, reg_limit=free, spillcost=spill),
                                   max_len=plain[2] + 4, max_interval=plain[1] + 3)
    assert (I, L) == (plain[1], plain[2]) and I == c["QK"] + c["PV"]
    assert len(set(A.values())) == 1             # the joint optimum is the single-wavefront schedule
    assert max(ms.live_footprint(g, M, I, regs)) <= free
    # with fewer registers per wavefront (more wavefronts per SIMD) the loop no longer fits one of them:
    # the model first moves the second product and its accumulators to another wavefront and pays the
    # transfer of P, then has to give up the matrix pipe's interval as well
    M2, I2, L2, A2 = ms.joint_schedule(g, ms.Warps(2, regs=regs, reg_limit=100, spillcost=spill),
                                       max_len=plain[2] + 4, max_interval=plain[1] + 3)
    assert len(set(A2.values())) == 2 and A2["PV"] != A2["SM"] and I2 == I
    M3, I3, L3, A3 = ms.joint_schedule(g, ms.Warps(2, regs=regs, reg_limit=68, spillcost=spill),
                                       max_len=plain[2] + 4, max_interval=plain[1] + 3)
    assert len(set(A3.values())) == 2 and I3 > I


def test_stage_bounded_search_of_section_5_1():
    # Section 5.1 admits, at every interval, only schedules with as many overlapped copies as the best plain
    # schedule at that interval (joint_schedule(..., stages="plain")).
    # where the plain optimum already satisfies the joint system, the bounded search returns it
    t = ms.paper_toy()
    M, I, L, A = ms.joint_schedule(t, ms.Warps(1), stages="plain")
    assert (I, L) == (2, 4) and ms.length(t, M) == 4 and ms.is_valid_assignment(t, M, I, A, ms.Warps(1))
    # the blocking example: one warp cannot hold I = 2 at any length, so both searches move to I = 3;
    # two warps solve it at I = 2
    g = _blocking_example()
    one, two = ms.Warps(1, blocking=[("GEMM", "ADD")]), ms.Warps(2, blocking=[("GEMM", "ADD")])
    assert ms.joint_schedule(g, one, stages="plain")[1] == 3 == ms.joint_schedule(g, one)[1]
    assert ms.joint_schedule(g, two, stages="plain")[1] == 2 == ms.joint_schedule(g, two)[1]
    # where the two differ.  Every warp can hold one value at a time and each hand-over costs a cycle: S stays
    # live for three cycles, so I >= 3, and at I = 3 the schedule is S 0, P 2, O 4 (L = 5, two overlapped
    # copies).  The plain optimum at I = 3 has L = 3 (one copy), so the bounded search may not take L = 5
    # there, nor at I = 4; it settles at I = 5, where L = 5 is still one copy.  The unbounded search takes I = 3.
    regs = {"S": 100, "P": 100, "O": 100}
    ws = ms.Warps(3, regs=regs, reg_limit=150, spillcost={"S": 1, "P": 1})
    Mj, Ij, Lj, Aj = ms.joint_schedule(t, ws)
    Mp, Ip, Lp, Ap = ms.joint_schedule(t, ws, stages="plain")
    assert (Ij, Lj) == (3, 5) and (Ip, Lp) == (5, 5) and ms.length(t, Mp) == 5
    assert ms.is_valid_assignment(t, Mp, Ip, Ap, ws) and _unrolled_ok(t, Mp, Ip, Ap, ws)
    assert _unrolled_ok(t, Mj, Ij, Aj, ws)
    plain = ms.optimal_modulo_schedule(t, Ip, 12)
    assert math.ceil(Lp / Ip) == math.ceil(ms.length(t, plain) / Ip) == 1


# ------------------------------------------------------------------ liveness as the paper states it
def _dataflow_footprint(loop, M, I, footprint):
    """Section 4.2 written out: a straight-line program of overlapped copies of M, I cycles apart, T cycles
    long; live[v, i, t] from the backward dataflow constraints (Init, LiveProp-1/2, DeadProp-1/2); the
    Memory Capacity sum per cycle.  The paper's Q executes the steady state once (ceil(L/I) copies); here
    a few more copies are laid out, so that one interval in the middle has every neighbour it has in the
    running loop (in Q itself the first steady cycles lack the loop-carried values of the copies before
    them).  Returns the use in that interval.  Independent of ms.live_ranges: no closed form, only the
    propagation rules."""
    L = ms.length(loop, M)
    max_delta = max([dl for _, _, _, dl in loop.edges] + [0])
    k = math.ceil(L / I) + max_delta + 1                 # the interval [k*I, (k+1)*I) is looked at
    copies = k + math.ceil(L / I) + max_delta + 2
    T = (copies - 1) * I + L
    op = lambda v, i, t: 0 <= i < copies and t == M[v] + i * I
    users = {v: [(u, dl) for a, u, _, dl in loop.edges if a == v] for v in M}
    live = {}
    for v in M:
        for i in range(copies):
            # Init: only loop-carried results of the last copy are live at the last cycle
            live[(v, i, T)] = i == copies - 1 and any(dl > 0 for _, dl in users[v])
    for t in range(T, 0, -1):
        for v in M:
            for i in range(copies):
                if live[(v, i, t)]:
                    live[(v, i, t - 1)] = not op(v, i, t)                        # LiveProp-1 / LiveProp-2
                else:
                    live[(v, i, t - 1)] = any(op(u, i + dl, t) for u, dl in users[v])   # DeadProp-1 / -2
    return [sum(footprint.get(v, 0) for v in M for i in range(copies) if live[(v, i, t)])
            for t in range(k * I, (k + 1) * I)]


def test_closed_form_liveness_is_the_papers_dataflow():
    import random
    rnd = random.Random(5)
    t = ms.paper_toy()
    M, I = {"S": 0, "P": 2, "O": 3}, 2
    fp = {"S": 1, "P": 1, "O": 1}
    # the paper's rule: S is live from its issue until P issues, P until O issues, O one interval
    assert ms.live_ranges(t, M, I, release="issue") == {"S": (0, 2), "P": (2, 3), "O": (3, 5)}
    assert _dataflow_footprint(t, M, I, fp) == ms.live_footprint(t, M, I, fp, release="issue") == [3, 2]
    # holding operands until the consumer has finished (what the register budgets here use) costs one more
    assert ms.live_footprint(t, M, I, fp) == [4, 3]
    # random small loops and their optimal schedules
    checked = 0
    while checked < 60:
        n = rnd.randint(2, 4)
        g = ms.Loop({"A": 2, "B": 1})
        names = ["v%d" % k for k in range(n)]
        for v in names:
            g.op(v, rnd.choice(["A", "B"]), rnd.randint(1, 2))
        for a in range(n):
            for b in range(a + 1, n):
                if rnd.random() < 0.6:
                    g.dep(names[a], names[b])
        if rnd.random() < 0.7:
            g.dep(names[-1], names[-1], delta=1)
        if rnd.random() < 0.3:
            g.dep(names[-1], names[0], d=0, delta=2)
        M, I, L = ms.schedule(g, max_len=12)
        fp = {v: rnd.randint(1, 3) for v in names}
        assert _dataflow_footprint(g, M, I, fp) == ms.live_footprint(g, M, I, fp, release="issue"), (M, I, g.edges)
        checked += 1


def test_cost_normalisation_with_the_papers_objective_is_the_global_minimum_of_f():
    import itertools

    def brute(C, U):
        best = None
        for cand in itertools.product(range(U + 1), repeat=len(C)):
            if 1 <= sum(cand) <= U:
                F = max(abs(C[i] * cand[j] - C[j] * cand[i]) for i in range(len(C)) for j in range(len(C)))
                if best is None or (F, -sum(cand)) < best[0]:
                    best = ((F, -sum(cand)), list(cand), F)
        return best[1], best[2]

    for C, U in [([512, 790, 512], 10), ([1000, 1000, 500, 250], 12), ([512, 480, 512], 24), ([3, 7, 11], 9),
                 ([100, 101], 15), ([90, 512, 790, 115, 512], 12), ([5, 5, 9, 2], 14)]:
        assert ms.normalise_costs(C, U, objective="paper") == brute(C, U), (C, U)
    # exact ratios are found by both objectives when U allows them
    assert ms.normalise_costs([1000, 1000, 500, 250], 12, objective="paper") == ([4, 4, 2, 1], 0)
    # absolute F leans towards coarse solutions, the relative objective keeps the resolution
    assert ms.normalise_costs([100, 101], 15, objective="paper") == ([1, 1], 1)
    assert ms.normalise_costs([100, 101], 15) == ([7, 7], 7)
