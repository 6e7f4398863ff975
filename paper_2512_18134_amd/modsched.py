"""Small optimal modulo scheduler, in the vocabulary of the paper's Section 3.1.

Host-side model only (no GPU work): it checks the claim that the loop order the
hand-scheduled kernels use is what modulo scheduling yields for the measured
gfx950 costs, and reproduces the paper's running example.

  * A loop is a dependence graph G = (V, E).  Every instruction v has a resource
    reservation table RRT[v]: a list with one entry per cycle of its execution,
    each entry a dict {functional unit: instances occupied}.  The machine
    description D gives the capacity of every unit.
  * An edge (u, v, d, delta): v of iteration i issues at least d cycles after u of
    iteration i - delta.
  * A modulo schedule is (M, I): instruction v issues at cycles M[v], I + M[v], ...;
    it is valid iff M[v] + I*delta >= M[u] + d for every edge and the modular RRT
    (unit use at every cycle mod I) stays within D.
  * L = length of M (last busy cycle + 1).  The pipelined loop overlaps
    ceil(L/I) copies of M, I cycles apart: the first (ceil(L/I) - 1) * I cycles
    are the prologue, the next I the steady state, the rest the epilogue.

The search is exhaustive (smallest I first, then smallest L): graphs here have a
handful of tile-level instructions, which is the granularity the paper
schedules at.  Section 4.2's memory-capacity constraint and Section 4.3's
warp-assignment constraints (`Warps`, `joint_schedule`) extend it to the joint
problem the paper solves.  Costs are normalised first (Section 5.2): integers C' with
sum <= U whose pairwise ratios stay as close as possible to those of C.
"""
import itertools
import math


class Loop:
    def __init__(self, capacity):
        self.capacity = dict(capacity)   # machine description D
        self.rrt = {}                    # name -> list of {unit: count}
        self.edges = []                  # (u, v, d, delta)
        self.order = []

    def op(self, name, unit, cycles, count=1):
        """Instruction that occupies `count` instances of `unit` for `cycles` cycles."""
        assert unit in self.capacity and cycles >= 0
        self.rrt[name] = [{unit: count} for _ in range(cycles)]
        self.order.append(name)
        return name

    def dep(self, u, v, d=None, delta=0):
        """v needs u's result: by default d = execution time of u."""
        self.edges.append((u, v, len(self.rrt[u]) if d is None else d, delta))


def modular_rrt(loop, M, I):
    """Unit use in the steady state: table[cycle mod I][unit]."""
    table = [dict() for _ in range(I)]
    for v, start in M.items():
        for c, use in enumerate(loop.rrt[v]):
            row = table[(start + c) % I]
            for unit, n in use.items():
                row[unit] = row.get(unit, 0) + n
    return table


def is_valid(loop, M, I):
    for u, v, d, delta in loop.edges:
        if M[v] + I * delta < M[u] + d:
            return False
    for row in modular_rrt(loop, M, I):
        for unit, n in row.items():
            if n > loop.capacity[unit]:
                return False
    return True


def length(loop, M):
    return max(M[v] + max(1, len(loop.rrt[v])) for v in M)


def res_mii(loop):
    """Resource bound on I: total occupation of a unit / its capacity."""
    use = {}
    for v in loop.rrt:
        for row in loop.rrt[v]:
            for unit, n in row.items():
                use[unit] = use.get(unit, 0) + n
    return max([1] + [math.ceil(n / loop.capacity[u]) for u, n in use.items()])


def rec_mii(loop):
    """Recurrence bound on I: max over dependence cycles of ceil(sum d / sum delta) (small graphs: brute force)."""
    names = list(loop.rrt)
    best = 1
    adj = {}
    for u, v, d, delta in loop.edges:
        adj.setdefault(u, []).append((v, d, delta))
    def walk(start, node, dsum, delsum, seen):
        nonlocal best
        for v, d, delta in adj.get(node, []):
            if v == start:
                if delsum + delta > 0:
                    best = max(best, math.ceil((dsum + d) / (delsum + delta)))
            elif v not in seen:
                walk(start, v, dsum + d, delsum + delta, seen | {v})
    for s in names:
        walk(s, s, 0, 0, {s})
    return best


def optimal_modulo_schedule(loop, I, max_len):
    """Valid M with initiation interval I and the smallest length <= max_len, or None."""
    names = loop.order
    for L in range(1, max_len + 1):
        ranges = [range(0, L - max(1, len(loop.rrt[v])) + 1) for v in names]
        for starts in itertools.product(*ranges):
            M = dict(zip(names, starts))
            if length(loop, M) == L and is_valid(loop, M, I):
                return M
    return None


def schedule(loop, max_len=None):
    """Smallest I, then smallest L: returns (M, I, L)."""
    total = sum(max(1, len(r)) for r in loop.rrt.values())
    max_len = max_len or 2 * total
    I = max(res_mii(loop), rec_mii(loop))
    while True:
        M = optimal_modulo_schedule(loop, I, max_len)
        if M is not None:
            return M, I, length(loop, M)
        I += 1


def in_order_interval(loop):
    """Cycles per iteration when the loop body runs in program order without overlap."""
    t = 0
    finish = {}
    for v in loop.order:
        start = t
        for u, w, d, delta in loop.edges:
            if w == v and delta == 0 and u in finish:
                start = max(start, finish[u][0] + d)
        finish[v] = (start, start + max(1, len(loop.rrt[v])))
        t = start + max(1, len(loop.rrt[v]))
    return t


def pipeline_code(loop, M, I):
    """Prologue / steady state / epilogue as lists of (instruction, iteration offset), by issue cycle.

    Iteration offset k in the steady state means "the instance that belongs k iterations
    before the newest one in flight" (Fig. 1f: Sn is offset 0, P and O are offset 1).
    """
    L = length(loop, M)
    copies = math.ceil(L / I)
    stage = {v: M[v] // I for v in M}
    steady = sorted(((M[v] % I, v, stage[v]) for v in M))
    prologue = []
    for c in range(copies - 1):                     # copy c starts at cycle c*I
        for v in M:
            pass
    for cyc in range((copies - 1) * I):
        for v in loop.order:
            for c in range(copies):
                if c * I + M[v] == cyc:
                    prologue.append((cyc, v, c))
    return {"copies": copies, "prologue_cycles": (copies - 1) * I,
            "prologue": prologue, "steady": [(c, v, k) for c, v, k in steady]}


def normalise_costs(C, U, objective="relative"):
    """Section 5.2: integers C' with 1 <= sum(C') <= U and |C[i]C'[j] - C[j]C'[i]| <= F for all i, j.

    objective="paper" minimises F itself, as the section's ILP states (ties: the finer resolution).  F grows
    with the magnitude of C', so that objective leans towards coarse solutions ([100, 101] with U = 15 gives
    [1, 1], F = 1, rather than [7, 7], F = 7: the same ratios); objective="relative" (default) minimises
    F / sum(C'), the ratio error at the scale of the solution, which keeps the resolution U pays for.
    Returns (C', F).  Candidates: every scale of the largest entry, each other entry rounded down or up."""
    assert objective in ("relative", "paper")
    n = len(C)
    big = max(range(n), key=lambda i: C[i])
    best = None
    for top in range(1, U + 1):
        # candidates: round each entry to one of the two integers around its scaled value
        scaled = [C[i] * top / C[big] for i in range(n)]
        choices = [sorted({max(0, math.floor(s)), math.ceil(s)}) for s in scaled]
        for cand in itertools.product(*choices):
            if not (1 <= sum(cand) <= U):
                continue
            F = max(abs(C[i] * cand[j] - C[j] * cand[i]) for i in range(n) for j in range(n))
            key = (F / max(1, sum(cand)), -sum(cand)) if objective == "relative" else (F, -sum(cand))
            if best is None or key < best[0]:
                best = (key, list(cand), F)
    return best[1], best[2]


# ------------------------------------------------------------------ memory capacity (Section 4.2)
def duration(loop, v):
    return max(1, len(loop.rrt[v]))


def live_ranges(loop, M, I, release="finish"):
    """[start, end) of the result of one instance of every instruction, in the time of its own iteration.

    release="issue" is the paper's definition (Section 4.2: backward dataflow over the unrolled schedule --
    a result becomes live in the cycle its instruction issues and dies in the cycle its last user (u, delta)
    issues, M[u] + I*delta; a result nobody uses is never live).  For a fixed (M, I) those constraints have
    this closed form; tests check it against the dataflow written out.

    release="finish" (default, what the gfx950 register budgets use) keeps a result reserved until its last
    user has FINISHED, M[u] + I*delta + duration(u): a tile-level instruction here is a run of MFMAs or
    VALU operations that reads its operand registers throughout, so they cannot be handed on at its issue.
    A result nobody uses then dies when its own instruction finishes.

    Either way a loop-carried self edge (an accumulator updated in place: O += ...) hands its registers to
    the next instance when that instance issues."""
    assert release in ("issue", "finish")
    out = {}
    for v in M:
        end = M[v] + duration(loop, v) if release == "finish" else M[v]
        for u, w, d, delta in loop.edges:
            if u == v and w == v:
                end = max(end, M[v] + I * delta)
            elif u == v:
                end = max(end, M[w] + I * delta + (duration(loop, w) if release == "finish" else 0))
        out[v] = (M[v], end)
    return out


def live_footprint(loop, M, I, footprint, resident=0, release="finish"):
    """Steady-state memory use per cycle (mod I): sum over instructions of footprint x number of
    overlapped iterations whose instance is live at that cycle, plus `resident` (loop invariants)."""
    ranges = live_ranges(loop, M, I, release)
    use = [resident] * I
    for v, (a, b) in ranges.items():
        f = footprint.get(v, 0)
        if not f:
            continue
        for t in range(a, b):
            use[t % I] += f
    return use


def fits(loop, M, I, footprint, capacity, resident=0, release="finish"):
    """The paper's Memory Capacity constraint for one memory (here: the register file of a wave)."""
    return max(live_footprint(loop, M, I, footprint, resident, release)) <= capacity


# ------------------------------------------------------------------ warp assignment (Section 4.3)
class Warps:
    """The inputs of the paper's warp-assignment constraints, for one loop:

      n_warps           warps (wavefronts here) the instructions may be spread over
      variable_latency  instructions whose latency is not known statically; they all go to the designated
                        warp W_vl (index 0), and nothing else does.  With none, every warp is an ordinary one.
      regs, reg_limit   registers a result occupies while live (Section 4.2's liveness), and the budget of
                        one warp; a result lives in the registers of the warp that produced it
      spillcost         cycles to hand a result to another warp through shared memory (LDS): added to the
                        delay of every edge whose ends sit on different warps
      blocking          edges (u, v) whose consumer must block on synchronisation before it can read the
                        result; an edge that crosses warps is blocking as well (the transfer needs a wait)
    """

    def __init__(self, n_warps, reg_limit=None, regs=None, variable_latency=(), spillcost=None, blocking=()):
        self.n_warps = n_warps
        self.reg_limit = reg_limit
        self.regs = dict(regs or {})
        self.variable_latency = frozenset(variable_latency)
        self.spillcost = dict(spillcost or {})
        self.blocking = frozenset(blocking)
        self.w_vl = 0 if self.variable_latency else None


def warp_edges(loop, A, ws):
    """The loop's edges with the cross-warp transfer cost added (Cross-Warp Spills)."""
    return [(u, v, d + (ws.spillcost.get(u, 0) if A[u] != A[v] else 0), delta) for u, v, d, delta in loop.edges]


def is_valid_assignment(loop, M, I, A, ws):
    """(M, I) with the warp assignment A (instruction -> warp index) against the constraints of Sections
    4.1-4.3: dependences with cross-warp delays, modular resource use, warp uniqueness, the variable-latency
    warp, the register limit of every warp and the concurrency constraint."""
    if set(A) != set(loop.rrt) or any(not (0 <= w < ws.n_warps) for w in A.values()):
        return False
    for v in loop.rrt:
        if (v in ws.variable_latency) != (ws.w_vl is not None and A[v] == ws.w_vl):
            return False
    for u, v, d, delta in warp_edges(loop, A, ws):
        if M[v] + I * delta < M[u] + d:
            return False
    for row in modular_rrt(loop, M, I):
        for unit, n in row.items():
            if n > loop.capacity[unit]:
                return False
    if ws.reg_limit is not None:
        for w in range(ws.n_warps):
            mine = {v: ws.regs.get(v, 0) for v in loop.rrt if A[v] == w}
            if max(live_footprint(loop, M, I, mine)) > ws.reg_limit:
                return False
    # concurrency: when v issues behind a blocking edge, its warp has nothing else in flight
    for u, v, _, _ in loop.edges:
        if (u, v) in ws.blocking or A[u] != A[v]:
            for o in loop.rrt:
                if o != v and A[o] == A[v]:
                    if (M[v] - M[o]) % I < duration(loop, o) or duration(loop, o) >= I:
                        return False
    return True


def _assignments(loop, ws):
    """Warp assignments up to renaming of the ordinary warps (they are interchangeable)."""
    names = [v for v in loop.order if v not in ws.variable_latency]
    first = 0 if ws.w_vl is None else 1
    def rec(i, used, cur):
        if i == len(names):
            A = dict(cur)
            for v in ws.variable_latency:
                A[v] = ws.w_vl
            yield A
            return
        for w in range(first, min(used + 1, ws.n_warps - 1) + 1):
            cur[names[i]] = w
            yield from rec(i + 1, max(used, w + 1), cur)
        cur.pop(names[i], None)
    yield from rec(0, first, {})


def _search(loop, I, L, edges, accept, A=None, blocked=()):
    """Depth-first search for start times with schedule length exactly L.  Every instruction is placed no
    earlier than its already placed predecessors allow; a partial schedule is dropped as soon as it breaks
    a dependence, oversubscribes a unit in some cycle mod I, or (with a warp assignment A and the set
    `blocked` of instructions that issue behind a blocking wait) breaks the concurrency constraint;
    `accept(M)` decides a complete schedule."""
    names = loop.order
    dur = {v: duration(loop, v) for v in names}
    M = {}
    table = [dict() for _ in range(I)]

    def occupy(v, t, sign):
        ok = True
        for c, use in enumerate(loop.rrt[v]):
            row = table[(t + c) % I]
            for unit, n in use.items():
                row[unit] = row.get(unit, 0) + sign * n
                if row[unit] > loop.capacity[unit]:
                    ok = False
        return ok

    def concurrent_ok(v, t):
        if A is None:
            return True
        for o, to in M.items():
            if o == v or A[o] != A[v]:
                continue
            if v in blocked and ((t - to) % I < dur[o] or dur[o] >= I):
                return False
            if o in blocked and ((to - t) % I < dur[v] or dur[v] >= I):
                return False
        return True

    def rec(i):
        if i == len(names):
            return dict(M) if length(loop, M) == L and accept(M) else None
        v = names[i]
        lo = 0
        for a, b, d, delta in edges:
            if b == v and a in M and a != v:
                lo = max(lo, M[a] + d - I * delta)
            if a == v and b == v and I * delta < d:
                return None                      # a recurrence on v itself that I cannot satisfy
        for t in range(lo, L - dur[v] + 1):
            ok = True
            for a, b, d, delta in edges:
                if a == v and b in M and b != v and M[b] + I * delta < t + d:
                    ok = False
                    break
            if not ok or not concurrent_ok(v, t):
                continue
            M[v] = t
            if occupy(v, t, +1):
                got = rec(i + 1)
                if got is not None:
                    return got
            occupy(v, t, -1)
            del M[v]
        return None
    return rec(0)


def joint_schedule(loop, ws, max_len=None, max_interval=None, stages=None):
    """The joint problem of Section 4: the smallest I, then the smallest L, over modulo schedules AND warp
    assignments; among equals the assignment that uses the fewest warps.  Returns (M, I, L, A), or None when
    nothing fits up to max_interval.

    stages="plain" narrows the search the way Section 5.1 does: at an interval I only schedules that overlap
    no more copies of the loop body than the best plain modulo schedule at that I (warps ignored) are
    admitted, i.e. L <= I * ceil(L_plain(I) / I); intervals at which no plain schedule exists are skipped.
    The joint constraints contain the plain ones, so nothing shorter than L_plain(I) is lost; what is given
    up are deeper pipelines at a small I, in favour of the next interval.  The default (None) admits them."""
    assert stages in (None, "plain")
    total = sum(duration(loop, v) for v in loop.rrt)
    max_len = max_len or 2 * total + sum(ws.spillcost.values())
    max_interval = max_interval or max_len
    cands = sorted(_assignments(loop, ws), key=lambda A: len(set(A.values())))
    I = max(res_mii(loop), rec_mii(loop))
    while I <= max_interval:
        cap = max_len
        if stages == "plain":
            plain = optimal_modulo_schedule(loop, I, max_len + I)
            if plain is None:
                I += 1
                continue
            cap = I * math.ceil(length(loop, plain) / I)
        best = None
        for A in cands:
            edges = warp_edges(loop, A, ws)
            top = cap if best is None else best[2] - 1
            for L in range(1, top + 1):
                blocked = {v for u, v, _, _ in loop.edges if (u, v) in ws.blocking or A[u] != A[v]}
                M = _search(loop, I, L, edges, lambda M: is_valid_assignment(loop, M, I, A, ws), A, blocked)
                if M is not None:
                    best = (M, I, L, A)
                    break
        if best is not None:
            return best
        I += 1
    return None


# ------------------------------------------------------------------ the paper's running example
def paper_toy():
    """Fig. 1: S = gemm(Q,K) on the tensor core, P = exp(S) on the exp unit, O += gemm(P,V) on the
    tensor core; every instruction one cycle; O carries a dependence to the next iteration."""
    g = Loop({"TC": 1, "EXP": 1})
    g.op("S", "TC", 1)
    g.op("P", "EXP", 1)
    g.op("O", "TC", 1)
    g.dep("S", "P")
    g.dep("P", "O")
    g.dep("O", "O", delta=1)
    return g


# ------------------------------------------------------------------ the gfx950 loop
# Per-wave costs of one K/V tile at D = 128 (32 scores per lane), in matrix-pipe cycles.  Sources, all
# reproducible from the repository (profiles/attn_fwd_d128_config4.md gives the commands):
#   * an MFMA occupies the matrix pipe for 32 cycles (SQ_VALU_MFMA_BUSY_CYCLES / SQ_INSTS_MFMA), 16 MFMAs
#     per product;
#   * on all-zero inputs (chip not power limited) the one-wave-per-SIMD loop keeps the pipe busy 81.5 % of
#     the cycles while it issues GFX950_STREAM_INSTRS instructions per 32 MFMAs: the wave's issue port is
#     the binding unit there, at 32 * 32 / 0.815 / 194 = 6.5 cycles per instruction on average;
#   * the softmax of a tile is GFX950_SOFTMAX_INSTRS of those instructions, the LDS operand reads 16 + 32
#     (8 + 16 when a fragment feeds two MFMAs).
GFX950_MFMA_CYCLES = 32
GFX950_UNTHROTTLED_BUSY = 0.815
GFX950_STREAM_INSTRS = 194
GFX950_SOFTMAX_INSTRS = 114
GFX950_ISSUE_CYCLES = GFX950_MFMA_CYCLES * 32 / GFX950_UNTHROTTLED_BUSY / GFX950_STREAM_INSTRS
GFX950_D128 = {"QK": 16 * GFX950_MFMA_CYCLES, "SM": round(GFX950_SOFTMAX_INSTRS * GFX950_ISSUE_CYCLES),
               "PV": 16 * GFX950_MFMA_CYCLES, "LDS_K": round(16 * GFX950_ISSUE_CYCLES),
               "LDS_V": round(32 * GFX950_ISSUE_CYCLES)}


def gfx950_attention(costs=GFX950_D128, U=24):
    """Tile-level dependence graph of one wave of the attention loop on gfx950: the matrix pipe (MFMA),
    the VALU and the LDS port are separate units fed from one instruction stream; global->LDS loads are
    streaming operations (zero latency in the model, Section 5.3) and do not appear."""
    names = ["LDS_K", "QK", "SM", "LDS_V", "PV"]
    Cn, F = normalise_costs([costs[n] for n in names], U)
    c = dict(zip(names, Cn))
    g = Loop({"MFMA": 1, "VALU": 1, "LDS": 1})
    g.op("LDS_K", "LDS", c["LDS_K"])
    g.op("QK", "MFMA", c["QK"])
    g.op("SM", "VALU", c["SM"])
    g.op("LDS_V", "LDS", c["LDS_V"])
    g.op("PV", "MFMA", c["PV"])
    g.dep("LDS_K", "QK", d=1)       # fragments stream into the MFMAs: the first one must have arrived
    g.dep("QK", "SM")
    g.dep("SM", "PV")
    g.dep("LDS_V", "PV", d=1)
    g.dep("SM", "SM", delta=1)      # running max / row sum
    g.dep("PV", "PV", delta=1)      # accumulator O
    return g, c, F


def gfx950_attention_subtiled(costs=GFX950_D128, parts=2, U=24):
    """The same loop with every tile-level instruction cut into `parts` sub-tiles (Section 6.1: the paper
    sub-tiles to the size of one matrix instruction before scheduling; here one sub-tile is one 32-row query
    block of the one-wave-per-SIMD tiling, or one 32-key block of the two-wave one).  Sub-tile p of the
    softmax needs only sub-tile p of the scores, sub-tile p of the second product only sub-tile p of P."""
    unit = {"QK": "MFMA", "SM": "VALU", "PV": "MFMA"}
    names = [n + str(p) for p in range(parts) for n in ("QK", "SM", "PV")]
    Cn, F = normalise_costs([costs[n[:2]] / parts for n in names], U)
    c = dict(zip(names, Cn))
    g = Loop({"MFMA": 1, "VALU": 1})
    for n in names:
        g.op(n, unit[n[:2]], c[n])
    for p in range(parts):
        g.dep("QK%d" % p, "SM%d" % p)
        g.dep("SM%d" % p, "PV%d" % p)
        g.dep("SM%d" % p, "SM%d" % p, delta=1)      # row state
        g.dep("PV%d" % p, "PV%d" % p, delta=1)      # accumulator O
    return g, c, F


def stream_mix(lines, body=1):
    """Instruction mix of one steady-state iteration of a generated loop (the text between the labels of
    body `body` and the next one): {class: count} with classes mfma, valu (transcendentals included),
    lds, vmem, wait, salu (s_nop and barrier included)."""
    lines = [l.strip() for l in lines]
    i = next(k for k, l in enumerate(lines) if l.startswith("BODY%d_" % body))
    j = next(k for k, l in enumerate(lines) if l.startswith("BODY%d_" % (body + 1)))
    mix = {"mfma": 0, "valu": 0, "lds": 0, "vmem": 0, "wait": 0, "salu": 0}
    for l in lines[i + 1:j]:
        if l.endswith(":"):
            continue
        op = l.split()[0]
        key = ("mfma" if op.startswith("v_mfma") else "valu" if op.startswith("v_") else "lds" if op.startswith("ds_")
               else "vmem" if op.startswith("global_") else "wait" if op.startswith("s_waitcnt") else "salu")
        mix[key] += 1
    return mix


def slot_level_bounds(mix, waves_per_simd):
    """Lower bounds on the initiation interval of one iteration at the granularity of single instructions
    (cycles per SIMD): the matrix pipe needs GFX950_MFMA_CYCLES per MFMA of every wave on the SIMD; a wave's
    issue port needs GFX950_ISSUE_CYCLES per instruction of that wave (waves issue side by side).  The
    generated loops issue exactly one MFMA per slot, so their I in slots is mix['mfma']: the matrix-pipe bound."""
    matrix = mix["mfma"] * GFX950_MFMA_CYCLES * waves_per_simd
    issue = sum(mix.values()) * GFX950_ISSUE_CYCLES
    return {"matrix": matrix, "issue": issue, "interval": max(matrix, issue),
            "matrix_busy": matrix / max(matrix, issue)}


# Registers per lane of the values in that graph (D = 128, 32 query rows per wave, 64-key tile): the
# S block (two 32x32 fp32 accumulators), P packed to bf16, the O accumulators; the LDS fragments are
# counted per buffer (4 registers) over the time they wait for their MFMA.  Loop invariants: Q fragments
# (32), LDS/DMA addresses, masks, row state (~44 in the generated loop).
GFX950_D128_REGS = {"QK": 32, "SM": 16, "PV": 64}
GFX950_D128_RESIDENT = 32 + 16 + 44       # Q + fragment ring + addresses and state


def gfx950_backward_key_owner(U=24):
    """Tile-level graph of the key-owner backward sweep (one wave, 32 keys, 32-query tile): S and dP on the
    matrix pipe, the element-wise work on the VALU, the two contractions on the matrix pipe; dK/dV carry."""
    # measured per-wave costs in matrix-pipe cycles: 16 MFMAs for S+dP, 16 for the contractions, ~80 VALU ops
    names = ["SDP", "EW", "CON"]
    Cn, F = normalise_costs([512, 480, 512], U)
    c = dict(zip(names, Cn))
    g = Loop({"MFMA": 1, "VALU": 1})
    g.op("SDP", "MFMA", c["SDP"])
    g.op("EW", "VALU", c["EW"])
    g.op("CON", "MFMA", c["CON"])
    g.dep("SDP", "EW")
    g.dep("EW", "CON")
    g.dep("CON", "CON", delta=1)
    return g, c, F


# S and dP (16 + 16), P and dS packed (8 + 8), dK^T and dV^T accumulators (64 + 64); resident: the owner's
# K and V rows as B operands (64), LSE'/Delta of the tile (32), fragment ring (16), addresses and state (~56)
GFX950_BWD_REGS = {"SDP": 32, "EW": 16, "CON": 128}
GFX950_BWD_RESIDENT = 64 + 32 + 16 + 56


if __name__ == "__main__":
    g = paper_toy()
    M, I, L = schedule(g)
    print("paper toy: I=%d L=%d M=%s  in-order interval=%d" % (I, L, M, in_order_interval(g)))
    g, c, F = gfx950_attention()
    M, I, L = schedule(g, max_len=4 * sum(c.values()))
    print("gfx950 D=128 wave: normalised costs %s (F=%d)" % (c, F))
    print("  I=%d (MFMA-bound: %d)  L=%d  stages=%d  M=%s" % (I, c["QK"] + c["PV"], L, math.ceil(L / I), M))
    print("  in-order interval=%d  => pipelining gain %.2fx" % (in_order_interval(g), in_order_interval(g) / I))
    print("  registers live in the steady state: max %d of 256 (two waves per SIMD)" %
          max(live_footprint(g, M, I, GFX950_D128_REGS, GFX950_D128_RESIDENT)))
    g12, c12, _ = gfx950_attention(U=12)
    spill = {"QK": c12["LDS_K"] + c12["LDS_V"], "SM": c12["LDS_K"] + c12["LDS_V"], "LDS_K": 1, "LDS_V": 1}
    for limit in (256 - GFX950_D128_RESIDENT, 100, 68):
        Mj, Ij, Lj, Aj = joint_schedule(g12, Warps(2, regs=GFX950_D128_REGS, reg_limit=limit, spillcost=spill),
                                        max_len=17, max_interval=9)
        print("  joint problem, %3d free registers per wave: I=%d L=%d warps=%s" % (limit, Ij, Lj, Aj))
    g, c, F = gfx950_backward_key_owner()
    M, I, L = schedule(g, max_len=4 * sum(c.values()))
    print("gfx950 backward key-owner wave: I=%d L=%d stages=%d, registers max %d (one wave per SIMD: 512)" %
          (I, L, math.ceil(L / I), max(live_footprint(g, M, I, GFX950_BWD_REGS, GFX950_BWD_RESIDENT))))
