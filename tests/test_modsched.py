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
    path = os.path.join(os.path.dirname(ms.__file__), "csrc", name + ".py")
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
    gen = _load_generator("gen_attn_loop").Gen(128)
    # the generator double-buffers S and P statically and allocates exactly what the model's values need
    assert gen.SB - gen.SA == 32 and gen.PB - gen.PA == 16
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
