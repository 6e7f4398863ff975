"""Shared pieces of the loop generators (gen_attn_loop.py, gen_attn_bwd_loop.py).

A generated loop is ONE inline-asm statement whose operands are pinned to physical
registers.  The assembler inserts no wait states and no s_waitcnt, so everything the
hardware does not interlock is done here, by construction:

  * LDS reads return in order: `Emitter.lds_issue` / `Emitter.lds_wait` keep the list
    of reads in flight and compute every `s_waitcnt lgkmcnt(N)` by replaying it;
  * one MFMA stream per iteration (`Emitter.stream`): slot i = [wait for the operand
    of group i] the MFMAs of group i, the LDS reads of group i + PFD (a ring of NF
    fragment buffers), scalar extras, then this slot's share of the VALU program;
  * direct global->LDS loads: scalar write of m0, s_nop (a wait state is needed between the
    two), the load;
  * m0 is a reserved register that cannot be named as a clobber: `save_m0` /
    `restore_m0` bracket the statement.

`check_stream` (used by the tests) replays a finished instruction list and verifies
these rules on the text itself.
"""
import re


class Emitter:
    def __init__(self):
        self.lines = []
        self.outstanding = []     # ids of the LDS reads in flight, in issue order

    # ------------------------------------------------------------------ text
    def e(self, s):
        self.lines.append(s)

    def lab(self, name):
        return "%s%%=" % name     # unique per expansion of the asm statement

    @staticmethod
    def rg(cls, base, n=1):
        return "%s%d" % (cls, base) if n == 1 else "%s[%d:%d]" % (cls, base, base + n - 1)

    def vr(self, base, n=1):
        return self.rg("v", base, n)

    def ar(self, base, n=1):
        return self.rg("a", base, n)

    def sr(self, base, n=1):
        return self.rg("s", base, n)

    # ------------------------------------------------------------- LDS reads
    def lds_issue(self, ident, instrs):
        for ins in instrs:
            self.e(ins)
            self.outstanding.append(ident)

    def lds_wait(self, ident):
        """Wait until every read tagged `ident` has returned (reads return in order)."""
        hits = [p for p, x in enumerate(self.outstanding) if x == ident]
        if not hits:
            return
        last = hits[-1]
        self.e("s_waitcnt lgkmcnt(%d)" % (len(self.outstanding) - 1 - last))
        self.outstanding = self.outstanding[last + 1:]

    # ------------------------------------------------------------ MFMA stream
    def stream(self, groups, mfma_texts, frag_loads, NF, PFD, valu_by_slot, extra_by_slot, nxt_frag_loads,
               prefetched=None, wait_every=1, lds_by_slot=None):
        """Emit the slots of one iteration.

        groups: fragment groups in issue order; mfma_texts(g, buf) -> the MFMAs fed by group g's fragment
        (buffer buf); frag_loads(g, buf) -> the LDS reads that fill it; nxt_frag_loads(i, buf) -> reads of
        group i of the NEXT iteration (prefetched in the last PFD groups) or None when there is none.
        The reads of the first `prefetched` groups (default PFD) are already in flight (ids 0.. in
        self.outstanding); the rest up to PFD is issued first.  wait_every = W: one s_waitcnt per W groups,
        for the operands of all W (needs PFD >= W).  A slot is one MFMA; extras and VALU shares are keyed by
        slot number.  lds_by_slot: other LDS reads issued in a slot; they take their place in the in-order
        count but are never waited for by index (they must retire inside the iteration: a later wait of a
        fragment covers them).
        """
        n = len(groups)
        prefetched = PFD if prefetched is None else prefetched
        assert PFD >= wait_every and PFD < NF
        for i in range(prefetched, min(PFD, n)):
            self.lds_issue(i, frag_loads(groups[i], i % NF))
        slot = 0
        for i, g in enumerate(groups):
            if i % wait_every == 0:
                self.lds_wait(min(i + wait_every - 1, n - 1))
            texts = mfma_texts(g, i % NF)
            for t, text in enumerate(texts):
                self.e(text)
                if t == len(texts) - 1:
                    # the buffer of group i+PFD was last read by group i+PFD-NF <= i-1
                    j = i + PFD
                    if j < n:
                        self.lds_issue(j, frag_loads(groups[j], j % NF))
                    elif nxt_frag_loads is not None:
                        self.lds_issue(j - n + 1000, nxt_frag_loads(j - n, (j - n) % NF))
                for ins in extra_by_slot.get(slot, []):
                    self.e(ins)
                for ins in (lds_by_slot or {}).get(slot, []):
                    self.e(ins)
                    self.outstanding.append(-1)
                for ins in valu_by_slot.get(slot, []):
                    self.e(ins)
                slot += 1
        assert lds_by_slot is None or -1 not in self.outstanding, "auxiliary LDS reads must retire inside the iteration"
        # the next iteration's prefetches take its own numbering
        self.outstanding = [x - 1000 if x >= 0 else x for x in self.outstanding]
        assert nxt_frag_loads is None or all(0 <= x < PFD for x in self.outstanding), self.outstanding
        return slot

    # ------------------------------------------------------------------- m0
    def save_m0(self, sreg):
        self.e("s_mov_b32 s%d, m0" % sreg)

    def restore_m0(self, sreg):
        self.e("s_mov_b32 m0, s%d" % sreg)


def spread(ops, fixed_cost, n_slots, cost=lambda ins: 2.5 if ins.startswith("v_exp") else 1.0):
    """Deal the VALU program `ops` (kept in order) over n_slots slots so that every slot carries about
    the same issue cost, given the cost of what the slot holds already (fixed_cost[slot]: its MFMA,
    LDS reads, waits, scalar work).  Returns {slot: [ops]}."""
    total = sum(cost(o) for o in ops) + sum(fixed_cost.get(i, 0.0) for i in range(n_slots))
    out = {i: [] for i in range(n_slots)}
    k = 0
    done = 0.0
    for i in range(n_slots):
        target = total * (i + 1) / n_slots
        done += fixed_cost.get(i, 0.0)
        while k < len(ops) and (done + cost(ops[k]) / 2 <= target or i == n_slots - 1):
            out[i].append(ops[k])
            done += cost(ops[k])
            k += 1
    assert k == len(ops)
    return out


# ---------------------------------------------------------------------------------------------
# Checker: replays an instruction list (one fall-through path) and asserts the hazard rules.
# ---------------------------------------------------------------------------------------------
_RANGE = re.compile(r"\b([vas])\[(\d+):(\d+)\]|\b([vas])(\d+)\b")


def regs_of(operand):
    """Registers named by one operand: 'v[4:7]' -> {('v',4),...}; 'v12' -> {('v',12)}; '-v3' too."""
    out = set()
    for m in _RANGE.finditer(operand):
        if m.group(1):
            out.update((m.group(1), r) for r in range(int(m.group(2)), int(m.group(3)) + 1))
        else:
            out.add((m.group(4), int(m.group(5))))
    return out


def parse(ins):
    """(opcode, [destination registers], [source registers]) of one instruction line."""
    ins = ins.strip()
    op, _, rest = ins.partition(" ")
    ops = [x.strip() for x in rest.split(",")] if rest else []
    if op.startswith(("s_waitcnt", "s_nop", "s_barrier", "s_branch", "s_cbranch", "s_endpgm")) or ins.endswith(":"):
        return op, set(), set()
    if op.startswith("global_load_lds"):
        return op, set(), set().union(*[regs_of(o) for o in ops]) | {("m", 0)}
    if op.startswith(("s_cmp", "s_bitcmp", "v_cmpx")):
        return op, set(), set().union(*[regs_of(o) for o in ops]) if ops else set()
    if op.startswith("v_permlane32_swap"):
        both = regs_of(ops[0]) | regs_of(ops[1])
        return op, both, both
    dst = regs_of(ops[0]) if ops else set()
    if ops and ops[0] == "m0":
        dst = {("m", 0)}
    if ops and ops[0] == "vcc":
        dst = {("vcc", 0)}
    src = set()
    for o in ops[1:]:
        o = o.split(" offset:")[0]
        src |= regs_of(o)
        if o == "m0":
            src.add(("m", 0))
        if o == "vcc":
            src.add(("vcc", 0))
    return op, dst, src


def wait_states(ins):
    m = re.match(r"s_nop (\d+)", ins.strip())
    return int(m.group(1)) + 1 if m else 1


def check_stream(lines, mfma_to_valu=11, valu_to_mfma=2, trans_to_use=1, m0_to_dma=1, max_lgkm=15):
    """Replay `lines` (a fall-through instruction sequence: labels and not-taken branches are skipped)
    and raise AssertionError on a violated rule:

      * an LDS read's destination is not read before an s_waitcnt lgkmcnt that covers it;
      * an MFMA result is not read or overwritten by a VALU instruction sooner than `mfma_to_valu` wait
        states after the MFMA issued (every instruction counts one, s_nop N counts N+1);
      * a VALU result is not read by an MFMA sooner than `valu_to_mfma` wait states later;
      * a transcendental result is not used by the next `trans_to_use` instructions;
      * at least `m0_to_dma` wait states separate a scalar write of m0 from a direct global->LDS load;
      * no s_waitcnt lgkmcnt exceeds the counter's range.

    Returns the number of instructions checked.
    """
    pending = []                    # LDS reads in flight: sets of destination registers, issue order
    last_mfma_write = {}            # reg -> time of the MFMA that last wrote it
    last_valu_write = {}
    last_trans_write = {}
    last_m0_write = None
    t = 0
    n = 0
    for raw in lines:
        ins = raw.strip()
        if not ins or ins.endswith(":"):
            continue
        op, dst, src = parse(ins)
        n += 1
        if op == "s_waitcnt":
            m = re.search(r"lgkmcnt\((\d+)\)", ins)
            if m:
                k = int(m.group(1))
                assert k <= max_lgkm, ins
                if len(pending) > k:
                    pending = pending[len(pending) - k:] if k else []
            t += 1
            continue
        if op.startswith("ds_read"):
            for p in pending:      # LDS reads return in order: a later read into the same registers wins
                p -= dst
            for p in pending:
                assert not (p & src), "address register still in flight: %s" % ins
            pending.append(set(dst))
            t += 1
            continue
        touched = dst | src
        for p in pending:
            assert not (p & touched), "register used before its LDS read was waited for: %s" % ins
        is_mfma = op.startswith("v_mfma")
        is_valu = op.startswith("v_") and not is_mfma
        if is_valu:
            for r in touched:
                if r in last_mfma_write:
                    assert t - last_mfma_write[r] >= mfma_to_valu + 1, "MFMA result touched too early: %s" % ins
            for r in src:
                if r in last_trans_write:
                    assert t - last_trans_write[r] >= trans_to_use + 1, "transcendental result used too early: %s" % ins
        if is_mfma:
            for r in src:
                if r in last_valu_write:
                    assert t - last_valu_write[r] >= valu_to_mfma + 1, "VALU result read by MFMA too early: %s" % ins
        if op.startswith("global_load_lds"):
            assert last_m0_write is not None and t - last_m0_write >= m0_to_dma + 1, "no wait state after m0 write: %s" % ins
        if ("m", 0) in dst:
            last_m0_write = t
        for r in dst:
            if is_mfma:
                last_mfma_write[r] = t
                last_valu_write.pop(r, None)
            elif is_valu:
                last_valu_write[r] = t
                last_mfma_write.pop(r, None)
                if op in ("v_exp_f32", "v_log_f32", "v_rcp_f32", "v_rsq_f32", "v_sqrt_f32"):
                    last_trans_write[r] = t
                else:
                    last_trans_write.pop(r, None)
        t += wait_states(ins)
    return n


def walk(lines, take=(), loop_label=None, loop_visits=2, limit=200000):
    """One execution path through `lines` as a flat instruction list: conditional branches are taken the
    first time their target is in `take` (each entry of `take` is used once) and fall through otherwise;
    unconditional branches are followed, except that the path ends when `loop_label` would be entered for
    the (loop_visits+1)-th time.  Labels are dropped."""
    where = {}
    for i, l in enumerate(lines):
        l = l.strip()
        if l.endswith(":"):
            where[l[:-1]] = i
    take = list(take)
    out = []
    visits = 0
    pc = 0
    while pc < len(lines) and len(out) < limit:
        l = lines[pc].strip()
        if l.endswith(":"):
            if loop_label is not None and l[:-1] == loop_label:
                visits += 1
                if visits > loop_visits:
                    break
            pc += 1
            continue
        op, _, rest = l.partition(" ")
        if op == "s_branch":
            out.append(l)
            pc = where[rest.strip()]
            continue
        if op.startswith("s_cbranch"):
            out.append(l)
            tgt = rest.strip()
            if tgt in take:
                take.remove(tgt)
                pc = where[tgt]
            else:
                pc += 1
            continue
        out.append(l)
        pc += 1
    return out


def run_scalar(lines, sgprs, bn, tb, bases, limit=2000000):
    """Execute the scalar control flow of `lines` (labels, s_mov / s_add / s_addc / s_sub / s_min / s_lshl /
    s_and / s_cmp_ge / s_cmp_lt / s_cbranch_scc0/1 / s_branch; vector instructions are skipped, branches on
    vcc fall through) from the SGPR values in `sgprs` ({number: value}; unset registers read 0) and return the
    events of the run in order: ("barrier",) and ("load", which, tile, lds_address), where `bases` =
    {"k": (base register, pointer register), "v": (...)} names the scalar pairs the direct loads go through:
    a load through a base register takes its tile from the scalar operand of the v_add_u32 that started its
    address (rows = tile * bn + lane part), a load through a pointer register from pointer - base (tile * tb).
    Carries into the high word of a pointer are not modelled (addc adds its immediate only)."""
    where = {}
    for i, l in enumerate(lines):
        l = l.strip()
        if l.endswith(":"):
            where[l[:-1]] = i
    S = dict(sgprs)
    scc = 0
    m0 = 0
    vtile = {}
    events = []

    def val(tok):
        tok = tok.strip()
        if tok == "m0":
            return m0
        if re.fullmatch(r"s\d+", tok):
            return S.get(int(tok[1:]), 0)
        return int(tok, 0)

    pc = 0
    steps = 0
    while pc < len(lines):
        steps += 1
        assert steps < limit, "the scalar program does not end"
        l = lines[pc].strip()
        pc += 1
        if not l or l.endswith(":"):
            continue
        op, _, rest = l.partition(" ")
        ops = [x.strip() for x in rest.split(",")] if rest else []
        if op == "s_branch":
            pc = where[ops[0]]
        elif op in ("s_cbranch_scc1", "s_cbranch_scc0"):
            if scc == (1 if op.endswith("1") else 0):
                pc = where[ops[0]]
        elif op.startswith("s_cbranch"):
            pass
        elif op == "s_barrier":
            events.append(("barrier",))
        elif op in ("s_mov_b32", "s_add_u32", "s_add_i32", "s_addc_u32", "s_sub_i32", "s_min_i32", "s_lshl_b32",
                    "s_and_b32"):
            a = val(ops[1])
            b = val(ops[2]) if len(ops) > 2 else 0
            r = {"s_mov_b32": a, "s_add_u32": a + b, "s_add_i32": a + b, "s_addc_u32": a + b, "s_sub_i32": a - b,
                 "s_min_i32": min(a, b), "s_lshl_b32": a << b, "s_and_b32": a & b}[op]
            if op != "s_mov_b32":
                scc = int(r != 0) if op in ("s_lshl_b32", "s_and_b32", "s_min_i32") else 0
                if op == "s_min_i32":
                    scc = int(a < b)
            if ops[0] == "m0":
                m0 = r
            else:
                S[int(ops[0][1:])] = r
        elif op in ("s_cmp_ge_i32", "s_cmp_lt_i32"):
            a, b = val(ops[0]), val(ops[1])
            scc = int(a >= b) if op == "s_cmp_ge_i32" else int(a < b)
        elif op == "v_add_u32" and re.fullmatch(r"s\d+", ops[1]):
            vtile[ops[0]] = val(ops[1]) // bn
        elif op.startswith("global_load_lds"):
            reg = int(re.search(r"s\[(\d+):", ops[1]).group(1))
            which = [w for w, pair in bases.items() if reg in pair][0]
            base, ptr = bases[which]
            off = re.search(r"offset:(\d+)", l)
            lds = m0 + (int(off.group(1)) if off else 0)
            tile = vtile[ops[0]] if reg == base else (S.get(ptr, 0) - S.get(base, 0)) // tb
            events.append(("load", which, tile, lds))
        elif op.startswith("s_") and op not in ("s_waitcnt", "s_nop"):
            raise AssertionError("scalar instruction not modelled: " + l)
    return events
