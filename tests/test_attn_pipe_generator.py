"""Host-side checks of the generated block loop of the long-suffix attention kernel
(csrc/gen_attn_pipe.py -> csrc/lsp_attn_pipe_loop.inc).  The loop is hand-scheduled text, so
what a compiler would guarantee is checked here instead, on the CPU, by an independent walk
over the instruction stream:

  * the committed .inc is exactly what the generator emits;
  * every register an instruction touches has been waited for if an LDS read that writes it is
    still in flight (LDS reads complete in order; `s_waitcnt lgkmcnt(n)` leaves at most n
    outstanding), on the hot path walked twice around the unrolled ring and on every cold
    block entered from it;
  * no LDS read lands in a register that the asm statement pins for something else;
  * wait-count and offset fields fit their encodings, every branch target exists, and no
    instruction writes memory through the scalar cache or uses packed fp32 arithmetic.
"""
import importlib.util
import os
import re

import pytest

CSRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2603_05454_amd", "csrc")
VREG = re.compile(r"\bv\[(\d+):(\d+)\]|\bv(\d+)\b")


@pytest.fixture(scope="module")
def gen():
    spec = importlib.util.spec_from_file_location("gen_attn_pipe", os.path.join(CSRC, "gen_attn_pipe.py"))
    m = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(m)
    return m


@pytest.fixture(scope="module")
def lines(gen):
    return gen.generate()


def _vregs(text):
    out = set()
    for m in VREG.finditer(text):
        if m.group(3) is not None:
            out.add(int(m.group(3)))
        else:
            out.update(range(int(m.group(1)), int(m.group(2)) + 1))
    return out


def _split(line):
    mnem, _, rest = line.partition(" ")
    return mnem, rest


def test_committed_include_is_what_the_generator_emits(lines):
    with open(os.path.join(CSRC, "lsp_attn_pipe_loop.inc")) as f:
        text = f.read()
    have = re.findall(r'^    "(.*)\\n"$', text, flags=re.M)
    assert have == lines


def test_fields_fit_and_nothing_forbidden(lines):
    labels = {l[:-1] for l in lines if l.endswith(":")}
    for l in lines:
        mnem, rest = _split(l)
        assert not mnem.startswith(("s_store", "s_buffer_store", "s_atomic", "s_buffer_atomic", "s_dcache", "s_scratch_store")), l
        assert not mnem.startswith(("v_pk_add_f32", "v_pk_mul_f32", "v_pk_fma_f32")), l
        for n in re.findall(r"lgkmcnt\((\d+)\)", l):
            assert 0 <= int(n) <= 15, l
        for n in re.findall(r"vmcnt\((\d+)\)", l):
            assert 0 <= int(n) <= 63, l
        for n in re.findall(r"offset:(\d+)", l):
            assert 0 <= int(n) <= 65535, l
        if mnem.startswith(("s_cbranch", "s_branch")):
            assert rest.strip() in labels, l
        assert all(r < 256 for r in _vregs(l)), l


def test_lds_reads_only_land_in_scratch_registers(gen, lines):
    pinned = set(range(32, 64)) | set(range(152, 170)) | set(range(176, 240))      # Q fragments, addresses, m and l, O
    frag = set()
    for base in gen.KF + gen.VF:
        frag.update(range(base, base + 4))
    for l in lines:
        mnem, rest = _split(l)
        if mnem.startswith("ds_read"):
            dst = _vregs(rest.split(",")[0])
            assert dst and not (dst & pinned), l
            assert dst <= frag, l


def _walk(lines, start, pending, labels, follow_back_edge, max_steps):
    """Walk from `start` along the hot path (conditional branches not taken, s_branch followed
    when follow_back_edge says so); returns the list of (index, pending-at-that-point) for every
    conditional branch passed, and stops at an s_branch it does not follow or after max_steps."""
    pend = [set(p) for p in pending]
    seen_cond = []
    i, steps = start, 0
    while i < len(lines) and steps < max_steps:
        l = lines[i]
        steps += 1
        if l.endswith(":"):
            i += 1
            continue
        mnem, rest = _split(l)
        if mnem == "s_waitcnt":
            m = re.search(r"lgkmcnt\((\d+)\)", l)
            if m:
                n = int(m.group(1))
                pend = pend[len(pend) - n:] if n else []
            i += 1
            continue
        if mnem.startswith("s_cbranch"):
            seen_cond.append((i, rest.strip(), [set(p) for p in pend]))
            i += 1
            continue
        if mnem == "s_branch":
            if follow_back_edge(rest.strip()):
                i = labels[rest.strip()]
                continue
            return seen_cond, pend, i
        touched = _vregs(rest)
        inflight = set().union(*pend) if pend else set()
        assert not (touched & inflight), f"line {i}: '{l}' touches {sorted(touched & inflight)} while an LDS read into them is in flight"
        if mnem.startswith("ds_read"):
            pend.append(_vregs(rest.split(",")[0]))
            assert len(pend) <= 16, f"line {i}: more than 16 LDS reads outstanding"
        i += 1
    return seen_cond, pend, i


def test_every_lds_result_is_waited_for_before_use(lines):
    labels = {l[:-1]: k for k, l in enumerate(lines) if l.endswith(":")}
    loop = next(k for k in labels if k.startswith(".Lloop"))
    # prologue, then twice around the eight unrolled iterations
    conds, _, _ = _walk(lines, 0, [], labels, lambda t: t == loop, max_steps=len(lines) * 3)
    assert sum(1 for _, t, _ in conds if t.startswith(".Lexit")) >= 16
    # every cold block, entered with the in-flight reads of the branch that leads to it
    checked = 0
    for idx, target, pend in conds:
        if target.startswith(".Lexit"):
            continue
        sub, _, end = _walk(lines, labels[target], pend, labels, lambda t: False, max_steps=400)
        assert not sub, (target, "conditional branch inside a cold block")
        assert lines[end].startswith("s_branch"), target
        assert not any(lines[k].startswith("ds_read") for k in range(labels[target], end)), target
        checked += 1
    assert checked >= 16 + 6


def test_exit_drains_every_counter(lines):
    labels = {l[:-1]: k for k, l in enumerate(lines) if l.endswith(":")}
    ex = next(v for k, v in labels.items() if k.startswith(".Lexit"))
    assert lines[ex + 1] == "s_waitcnt vmcnt(0) lgkmcnt(0)"


def test_the_checker_sees_a_missing_wait(lines):
    """The walk above must fail when a wait is taken away: drop, one at a time, a sample of the
    lgkmcnt waits inside the loop and require an assertion for each."""
    labels = {l[:-1]: k for k, l in enumerate(lines) if l.endswith(":")}
    loop_label = next(k for k in labels if k.startswith(".Lloop"))
    waits = [k for k, l in enumerate(lines) if l.startswith("s_waitcnt lgkmcnt") and k > labels[loop_label]
             and k < next(v for kk, v in labels.items() if kk.startswith(".Lexit"))]
    assert len(waits) >= 16
    caught = 0
    for k in waits[::3]:
        broken = lines[:k] + ["s_nop 0"] + lines[k + 1:]
        try:
            _walk(broken, 0, [], labels, lambda t: t == loop_label, max_steps=len(lines) * 3)
        except AssertionError:
            caught += 1
    assert caught == len(waits[::3])


# ---- the loop of a wave without an active query (csrc/lsp_attn_pipe_idle_loop.inc) ----

def _sync_skeleton(lines):
    """What the waves of a workgroup must agree on, in order, up to the loop's exit label: the
    stage every load goes to (m0), the loads, the block counter and its exit test, the waits
    for loads and the barriers."""
    out = []
    for l in lines:
        if l == ".Lexit_%=:":
            break
        mnem, rest = _split(l)
        if (mnem.startswith("global_load_lds") or mnem == "s_barrier" or "vmcnt" in l or l.endswith(":") and ("loop" in l or "issue" in l)
                or mnem == "s_add_u32" and rest.startswith("m0") or "s72" in l or l == "s_cbranch_scc0 .Lexit_%="
                or mnem in ("s_cmp_eq_u32", "s_cselect_b32", "s_addc_u32") or mnem == "s_add_u32" and rest.startswith(("s66", "s68", "s71"))
                or mnem.startswith("s_cbranch_scc1")):
            out.append(l)
    return out


def test_idle_include_is_what_the_generator_emits(gen):
    with open(os.path.join(CSRC, "lsp_attn_pipe_idle_loop.inc")) as f:
        text = f.read()
    assert re.findall(r'^    "(.*)\\n"$', text, flags=re.M) == gen.generate_idle()


def test_idle_loop_keeps_the_loads_waits_and_barriers_of_the_full_loop(gen, lines):
    """A wave that runs the idle loop sits in the same workgroup as waves that run the full one:
    both must issue the same loads into the same stages and meet at the same barriers, block by
    block, or the ring protocol breaks (a stage overwritten while it is read, or a barrier that
    some wave never reaches)."""
    idle = gen.generate_idle()
    a, b = _sync_skeleton(lines), _sync_skeleton(idle)
    assert sum(l == "s_barrier" for l in a) == 1 + gen.NS // 2
    assert sum(l.startswith("global_load_lds") for l in a) == 2 * (gen.LA + gen.NS)
    assert a == b
    # after the exit label: every load of the wave has landed before it goes on, m0 is restored
    for stream in (lines, idle):
        tail = stream[stream.index(".Lexit_%=:"):]
        assert "vmcnt(0)" in tail[1] and any(l.startswith("s_mov_b32 m0") for l in tail[:4])
    # the same cold cache -> suffix switch blocks exist
    assert [l for l in idle if l.startswith(".Lswitch")] == [l for l in lines if l.startswith(".Lswitch")]
    # the comparison notices a barrier, a load or a wait that one side lacks, and a load sent to another stage
    for victim in ("s_barrier", "global_load_lds_dwordx4 v165, s[68:69]", "s_waitcnt vmcnt(4)"):
        k = [i for i, l in enumerate(idle) if l == victim][3]
        assert _sync_skeleton(idle[:k] + idle[k + 1:]) != a, victim
    k = [i for i, l in enumerate(idle) if l.startswith("s_add_u32 m0")][5]
    assert _sync_skeleton(idle[:k] + ["s_add_u32 m0, %[ldsk], 0"] + idle[k + 1:]) != a


def test_idle_loop_leaves_the_matrix_pipe_and_the_vector_alu_alone(gen):
    idle = gen.generate_idle()
    labels = {l[:-1] for l in idle if l.endswith(":")}
    for l in idle:
        mnem, rest = _split(l)
        assert not mnem.startswith(("v_mfma", "ds_", "v_exp", "v_fma", "v_max", "v_cvt", "v_dot")), l
        assert not mnem.startswith(("s_store", "s_buffer_store", "s_atomic", "s_buffer_atomic", "s_dcache", "s_scratch_store")), l
        if mnem.startswith("v_"):
            assert mnem == "v_mov_b32" and _vregs(l) <= {gen.KOFF, gen.VOFF, gen.KOFF_S, gen.VOFF_S}, l
        if mnem.startswith("global_load_lds"):
            assert _vregs(l) <= {gen.KOFF, gen.VOFF}, l
        for n in re.findall(r"vmcnt\((\d+)\)", l):
            assert 0 <= int(n) <= 63, l
        if mnem.startswith(("s_cbranch", "s_branch")):
            assert rest.strip() in labels, l


# ---- the ring protocol, by running the scalar skeleton of both loops on concrete block counts ----

def _run_skeleton(lines, nb, nc, NS, max_steps=200000):
    """Interpret the scalar instructions of a generated loop for a key stream of nc cache blocks
    followed by nb - nc suffix blocks (vector, matrix and LDS instructions are skipped, the
    rescale branch is never taken).  Returns the event list: ("load", which, stage, address),
    ("wait", loads allowed to stay outstanding), ("barrier",), ("done", blocks finished)."""
    labels = {l[:-1]: k for k, l in enumerate(lines) if l.endswith(":")}
    KC, VC, KS, VS, CSTEP, SSTEP, LDSK = 0x10000000, 0x20000000, 0x30000000, 0x40000000, 0x8000, 0x2000, 0x400
    sym = {"%[kc]": KC, "%[vc]": VC, "%[ks]": KS, "%[vs]": VS, "%[cstep]": CSTEP, "%[sstep]": SSTEP,
           "%[nc]": nc, "%[nb]": nb, "%[ldsk]": LDSK}
    reg = {"m0": 0}
    scc = 0
    M = 0xFFFFFFFF

    def val(x):
        x = x.strip()
        if x in sym:
            return sym[x]
        m = re.fullmatch(r"s\[(\d+):(\d+)\]", x)
        if m:
            return reg[f"s{m.group(1)}"] | (reg[f"s{m.group(2)}"] << 32)
        if x in reg or re.fullmatch(r"s\d+", x):
            return reg[x]
        return int(x, 0) & M

    def signed(v):
        return v - (1 << 32) if v & 0x80000000 else v

    ev, i, steps = [], 0, 0
    while i < len(lines):
        steps += 1
        assert steps < max_steps, "the loop does not end"
        l = lines[i]
        i += 1
        if l.endswith(":"):
            continue
        mnem, rest = _split(l)
        ops = [o.strip() for o in rest.split(",")] if rest else []
        if mnem == "s_mov_b32":
            reg[ops[0]] = val(ops[1]) & M
        elif mnem == "s_mov_b64":
            m = re.fullmatch(r"s\[(\d+):(\d+)\]", ops[0])
            v = val(ops[1])
            reg[f"s{m.group(1)}"], reg[f"s{m.group(2)}"] = v & M, v >> 32
        elif mnem == "s_add_u32":
            t = val(ops[1]) + val(ops[2])
            reg[ops[0]], scc = t & M, int(t > M)
        elif mnem == "s_addc_u32":
            t = val(ops[1]) + val(ops[2]) + scc
            reg[ops[0]], scc = t & M, int(t > M)
        elif mnem == "s_sub_u32":
            t = val(ops[1]) - val(ops[2])
            reg[ops[0]], scc = t & M, int(t < 0)
        elif mnem in ("s_cmp_lt_u32", "s_cmp_eq_u32", "s_cmp_lt_i32", "s_cmp_gt_i32"):
            a, b = val(ops[0]), val(ops[1])
            if mnem.endswith("i32"):
                a, b = signed(a), signed(b)
            scc = int({"lt": a < b, "eq": a == b, "gt": a > b}[mnem.split("_")[2]])
        elif mnem == "s_cselect_b32":
            reg[ops[0]] = (val(ops[1]) if scc else val(ops[2])) & M
        elif mnem in ("s_cbranch_scc0", "s_cbranch_scc1"):
            if scc == int(mnem[-1]):
                i = labels[rest.strip()]
        elif mnem == "s_cbranch_vccnz":
            pass
        elif mnem == "s_branch":
            i = labels[rest.strip()]
        elif mnem.startswith("global_load_lds"):
            off = reg["m0"] - LDSK
            ev.append(("load", "V" if off >= NS * 8192 else "K", (off % (NS * 8192)) // 8192, val(ops[1])))
        elif mnem == "s_waitcnt":
            m = re.search(r"vmcnt\((\d+)\)", l)
            if m:
                ev.append(("wait", int(m.group(1))))
        elif mnem == "s_barrier":
            ev.append(("barrier",))
        else:
            assert mnem.startswith(("v_", "ds_", "s_nop", "s_setprio")), l
    ev.append(("done", reg["s72"]))
    return ev, (KC, VC, KS, VS, CSTEP, SSTEP)


@pytest.mark.parametrize("which", ["full", "idle"])
def test_ring_protocol_on_concrete_streams(gen, lines, which):
    """For key streams of 1..40 blocks with the cache -> suffix switch at several places: block i is
    requested, K and V, into stage (i mod NS) from the address of that block, in order; beyond the last
    block the last one is requested again (so that the number of loads in flight stays what the waits
    assume), LA blocks ahead of the iteration as everywhere else; at the barrier that ends iteration j
    the wave has waited for its loads of every block up to j + 4 (those are read before the next
    barrier) - at the first barrier up to block 3; a stage is not requested again before a barrier has
    passed since the block it held was last read (V of block i is read in iteration i); and the loop
    ends after exactly nb blocks."""
    stream = lines if which == "full" else gen.generate_idle()
    NS, LA = gen.NS, gen.LA
    for nb in list(range(1, 41)):
        for nc in sorted({0, 1, nb // 2, nb - 1, nb}):
            ev, (KC, VC, KS, VS, CSTEP, SSTEP) = _run_skeleton(stream, nb, nc, NS)
            assert ev[-1] == ("done", nb), (nb, nc, ev[-1])
            loads = [e for e in ev if e[0] == "load"]
            assert len(loads) == 2 * (LA + nb), (nb, nc, len(loads))      # LA before the loop, one per iteration
            for i in range(LA + nb):
                b = min(i, nb - 1)
                k, v = loads[2 * i], loads[2 * i + 1]
                ka, va = (KC + b * CSTEP, VC + b * CSTEP) if b < nc else (KS + (b - nc) * SSTEP, VS + (b - nc) * SSTEP)
                assert k == ("load", "K", i % NS, ka) and v == ("load", "V", i % NS, va), (nb, nc, i, k, v)
            issued = landed = barriers = 0
            request_time = {}   # block -> number of barriers passed when it was requested
            for e in ev:
                if e[0] == "load":
                    if e[1] == "K":
                        request_time[issued // 2] = barriers
                    issued += 1
                elif e[0] == "wait":
                    landed = max(landed, issued - e[1])
                elif e[0] == "barrier":
                    j = -1 if barriers == 0 else 2 * barriers - 1      # the iteration this barrier ends
                    assert landed >= 2 * (j + 4 + 1), (nb, nc, "barrier", barriers, "landed", landed)
                    barriers += 1
            # barriers: one before the loop, then one after every odd iteration that is not the last
            assert barriers == 1 + sum(1 for j in range(1, nb, 2) if j + 1 < nb), (nb, nc, barriers)
            # block i (i >= NS) reuses the stage of block i - NS, last read in iteration i - NS; the barrier
            # that ends odd iteration j is number (j + 1) / 2 + 1 counted from 1
            for i in range(NS, LA + nb):
                if i - NS >= nb:
                    continue        # the stage held a repeat of the last block, which nobody reads
                jodd = (i - NS) | 1
                if jodd + 1 < nb:   # (that barrier exists; otherwise the loop has ended before the request)
                    assert request_time[i] >= (jodd + 1) // 2 + 1, (nb, nc, i, request_time[i])


def test_the_ring_check_sees_a_wait_that_is_too_lax(gen, lines):
    """Planted mistake (on the CPU, in a copy of the text): the wait before the barriers made laxer by
    one block must leave a needed block in flight."""
    def first_violation(stream, nb):
        ev, _ = _run_skeleton(stream, nb, 0, gen.NS)
        issued = landed = barriers = 0
        for e in ev:
            if e[0] == "load":
                issued += 1
            elif e[0] == "wait":
                landed = max(landed, issued - e[1])
            elif e[0] == "barrier":
                j = -1 if barriers == 0 else 2 * barriers - 1
                if landed < 2 * (j + 4 + 1):
                    return barriers
                barriers += 1
        return None

    assert all(first_violation(lines, nb) is None for nb in range(1, 30))
    lax = [("s_waitcnt vmcnt(6)" if l == "s_waitcnt vmcnt(4)" else l) for l in lines]
    assert all(first_violation(lax, nb) == 0 for nb in range(1, 30))


def test_wave_priority_is_back_to_default_wherever_the_statement_can_end(gen, lines):
    """The loop raises the wave's priority for the first half of every iteration.  Walking the hot
    path: the priority is 0 at every branch that can leave the loop (the exit test, and the cold
    blocks, which come back to where they left), 1 exactly from the first S instruction to the
    first O instruction of an iteration, and the loader-only loop never touches it."""
    assert not any(l.startswith("s_setprio") for l in gen.generate_idle())
    labels = {l[:-1]: k for k, l in enumerate(lines) if l.endswith(":")}
    start, end = labels[".Lloop_%="], labels[".Lexit_%="]
    prio, seen = 0, 0
    for l in lines[:start]:
        assert not l.startswith("s_setprio"), "the prologue runs at the default priority"
    for l in lines[start:end]:
        mnem, rest = _split(l)
        if mnem == "s_setprio":
            prio = int(rest)
            assert prio in (0, 1)
            seen += 1
        elif mnem.startswith("s_cbranch") or mnem == "s_barrier":
            assert prio == 0, l
        elif mnem.startswith("v_mfma"):
            writes_scores = _vregs(rest.split(",")[0]) <= set(range(0, 32))
            assert prio == (1 if writes_scores else 0), l
    assert seen == 2 * gen.NS and prio == 0
    for l in lines[end:]:
        assert not l.startswith("s_setprio"), "cold blocks and the exit leave the priority alone"
