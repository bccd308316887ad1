"""Static checks of the hand-scheduled descent loop of the N = 64 ring-sum kernel (csrc/cc_2opt_n64_loop.inc), on the
CPU: the committed text is what its generator writes, and the instruction stream keeps the wait states gfx950 asks for,
which the compiler's hazard recognizer does not look at inside an asm statement:
  - a DPP instruction reads a VGPR no sooner than two wait states after a VALU instruction wrote it;
  - v_cndmask reads VCC, and a VALU instruction reads an SGPR, no sooner than two wait states after a VALU instruction
    wrote it; v_readlane reads a VGPR no sooner than one wait state after a VALU instruction wrote it;
  - no register that an LDS instruction still has to write is read (or overwritten) before an s_waitcnt has covered
    it, and no more LDS instructions are in flight than the counter can count.
The loop is walked twice, so the checks also hold from the end of one sweep into the next."""
import importlib.util
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2105_14088_amd", "csrc")


def _generator():
    spec = importlib.util.spec_from_file_location("gen_2opt_n64_loop", os.path.join(CSRC, "gen_2opt_n64_loop.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def _instructions():
    text = open(os.path.join(CSRC, "cc_2opt_n64_loop.inc")).read()
    body = text.split("#define CC_N64_DESCENT_LOOP_ASM")[1].split("#define CC_N64_DESCENT_LOOP_CLOBBERS")[0]
    lines = re.findall(r'"(.*?)\\n\\t"', body)
    return [l for l in lines if not l.endswith(":")]


def _operands(ins):
    parts = ins.replace(",", " ").split()
    ops = []
    for tok in parts[1:]:
        if re.fullmatch(r"(v\d+|s\d+|vcc|m0|%\[\w+\]|s\[\d+:\d+\])", tok):
            ops.append(tok)
    return parts[0], ops


def _expand(reg):
    m = re.fullmatch(r"s\[(\d+):(\d+)\]", reg)
    return [f"s{i}" for i in range(int(m.group(1)), int(m.group(2)) + 1)] if m else [reg]


NO_DST = ("s_nop", "s_waitcnt", "s_branch", "s_cbranch", "s_cmp", "s_bitcmp")


def _dst_src(ins):
    op, ops = _operands(ins)
    if op.startswith(NO_DST):
        return op, [], [r for o in ops for r in _expand(o)]
    dst = _expand(ops[0]) if ops else []
    src = [r for o in ops[1:] for r in _expand(o)]
    if op.startswith("v_cndmask"):
        src.append("vcc")
    if op in ("v_writelane_b32",):                # writes one lane: the destination is also read
        src += dst
    return op, dst, src


def _wait_states(ins):
    return int(ins.split()[1]) + 1 if ins.startswith("s_nop") else 1


def test_committed_text_is_what_the_generator_writes():
    assert open(os.path.join(CSRC, "cc_2opt_n64_loop.inc")).read() == _generator().text()


def test_every_diagonal_is_gathered_and_scored_once():
    ins = _instructions()
    gathers = [i for i in ins if i.startswith("ds_read_b32 v1") and int(i.split()[1][1:-1]) in range(102, 133)]
    assert len(gathers) == 31 and len(set(gathers)) == 31
    scored = [i for i in ins if i.startswith("v_add_u32_dpp")]
    assert len(scored) == 31 and len({i.split()[2] for i in scored}) == 31


def test_wait_states_between_dependent_instructions():
    ins = _instructions()
    stream = ins + ins                            # two sweeps: the hazards across the loop's back edge as well
    problems = []
    for i, cur in enumerate(stream):
        op, dst, src = _dst_src(cur)
        need = {}                                 # register -> wait states required since a VALU write of it
        if "_dpp" in op:
            need[_operands(cur)[1][1]] = 2        # the DPP operand is the first source
        if op.startswith("v_cndmask"):
            need["vcc"] = 2
        if op == "v_readlane_b32":
            need[_operands(cur)[1][1]] = 1
        if op.startswith("v_"):
            for r in src:
                if re.fullmatch(r"s\d+", r):
                    need[r] = max(need.get(r, 0), 2)
        ws, j = 0, i - 1
        while j >= 0 and ws < 3 and need:
            pop, pdst, _ = _dst_src(stream[j])
            if pop.startswith("v_"):
                for r in pdst:
                    if r in need and ws < need[r]:
                        problems.append((cur, stream[j], ws))
            ws += _wait_states(stream[j])
            j -= 1
    assert not problems, problems[:5]


def test_lds_results_are_waited_for_and_the_counter_never_overflows():
    ins = _instructions()
    in_flight, most = [], 0
    for cur in ins + ins:
        op, dst, src = _dst_src(cur)
        if op == "s_waitcnt":
            n = int(re.search(r"lgkmcnt\((\d+)\)", cur).group(1))
            while len(in_flight) > n:
                in_flight.pop(0)                  # LDS instructions complete in order
            continue
        busy = {r for regs in in_flight for r in regs}
        assert not (busy & set(src)), f"{cur}: reads a register an LDS instruction has not written yet"
        if op.startswith("ds_"):
            assert not (busy & set(dst)), f"{cur}: destination still in flight"
            in_flight.append(dst)
            most = max(most, len(in_flight))
        else:
            assert not (busy & set(dst)), f"{cur}: overwrites a register an LDS instruction has not written yet"
        if op == "s_branch":
            assert not in_flight, "LDS instructions in flight across the back edge"
    assert 0 < most <= 15


def test_the_loop_is_bounded_and_has_one_back_edge():
    ins = _instructions()
    assert sum(i.startswith("s_branch LOOP_TOP") for i in ins) == 1
    assert "s_bitcmp1_b32 %[applied], 22" in ins and ins.count("s_cbranch_scc1 LOOP_DONE%=") == 1
    assert ins.count("s_cbranch_scc0 LOOP_DONE%=") == 1


def _emulated_descent(c, tour):
    """Runs the committed loop text in the wave64 interpreter: matrix c (64 x 64, symmetric, entries below 2^16),
    start order `tour`; returns (final order, final cost, applied moves)."""
    import numpy as np
    from wave64_emulator import Wave
    gen = _generator()
    lines = gen.loop()
    n, mbase = 64, 0x2000
    lds = np.zeros(mbase // 4 + n * n, dtype="<u4")
    lds[mbase // 4:] = (c.astype(np.int64) << 14).reshape(-1)
    lane = np.arange(n)
    t = np.asarray(tour, dtype=np.int64)
    fm = (c[t, np.roll(t, 1)].astype(np.int64)) << 14
    rank_a = (lane + n - 1) & (n - 1)
    w = Wave(lds.tobytes(), dict(gen.operands(lane, rank_a, mbase), t=t, fm=fm, cur=int(fm.sum() >> 14), applied=0))
    w.run(lines)
    return w.named["t"].astype(np.int64), w.named["cur"], w.named["applied"]


def test_emulated_loop_takes_the_oracles_descent():
    """What the loop computes, checked on the CPU: the committed text, run instruction by instruction in a wave64
    interpreter, ends every descent with the oracle's order, cost and move count (random matrices with few distinct
    values, so that many moves tie and the lowest-id rule decides; the 16-bit edge of the value range)."""
    import sys
    import numpy as np
    sys.path.insert(0, ROOT)
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    import oracle
    for case, hi in enumerate((3, 40, 65535, 1000)):
        rng = np.random.default_rng(100 + case)
        c = rng.integers(0 if hi > 3 else 1, hi + 1, size=(64, 64))
        c = np.triu(c, 1)
        c = (c + c.T).astype(np.int32)
        tours = np.stack([np.concatenate(([0], 1 + rng.permutation(63))) for _ in range(3)]).astype(np.int32)
        want_c, want_t, want_m = oracle.restarts(c, oracle.SUM, 0, 0, len(tours), init=tours)
        for r, tour in enumerate(tours):
            t, cost, applied = _emulated_descent(c, tour)
            assert np.array_equal(t, want_t[r]) and cost == want_c[r] and applied == want_m[r], (case, r)
