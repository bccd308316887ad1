"""Writes cc_2opt_n64_loop.inc: the descent loop of the N = 64 ring-sum kernel (32-bit keys) as one inline-asm text.

Run by hand after a change (python gen_2opt_n64_loop.py); the build only reads the committed .inc file, and a CPU test
checks that the two agree and that the text keeps the wait states the instruction set asks for.

Why assembly.  With 1024 restarts every SIMD holds exactly one wavefront, and a lone wavefront issues one instruction
about every 4.5 clocks whatever its kind, s_nop and s_waitcnt included.  The loop is therefore written so that
(a) a batch of LDS gathers is covered by ONE s_waitcnt; (b) the two wait states a DPP read needs after the write of
its source are filled with instructions of an older batch, not with s_nop; (c) the hop array travels with the order
through the applied move (a lane permute plus the winner's two new hops), so a sweep starts without an LDS round trip.

The sweep itself is the cyclic-diagonal sweep described in cc_2opt_n64.hip.  Per diagonal d = 2 .. 32:
    rotate   pk_d   = pk_(d-1) from the next lane          (partner word: -f[b] << 14 | rank(b) << 8 | 4 t[b])
    address  A_d    = (pk_d & 0xff) | row offset of t[a]
    gather   D_d    = LDS[A_d]                              (c[t[a]][t[a+d]] << 14)
    score    key    = D_d + pk_d + D_d of the previous lane (one add, one DPP add)
    keep     best   = min(best, key)                        (one v_min3 per two diagonals)

Registers.  v66 .. v96: partner word of diagonal d in v(64+d); v102 .. v132: gather address, then gathered entry, of
diagonal d in v(100+d); v142 .. v145 keys; v150 .. v158 per-sweep values; s40 .. s53 scalars of the move.
Operands (see cc_2opt_n64.hip): t, fm (f << 14), cur, applied are read and written; rank_bits, ra, id_base, id_flip,
lane, lane4, mbase, mask (0xff), himask (0xfffff000) are read.
"""
import os

ROL = 'wave_rol:1 row_mask:0xf bank_mask:0xf bound_ctrl:1'      # lane p <- lane p+1
ROR = 'wave_ror:1 row_mask:0xf bank_mask:0xf bound_ctrl:1'      # lane p <- lane p-1
DIAGONALS = list(range(2, 33))
BATCHES = (6, 6, 6, 6, 7)

ROWOFS, FNEXT, BEST, YBEST, KEY2, RED, T0, T1, T2 = ("v150", "v151", "v152", "v153", "v154", "v155", "v156", "v157",
                                                     "v158")
S_WIN, S_DWIN, S_MI, S_MJ, S_DIF, S_SUM, S_MJ1, S_FA, S_FB, S_X, S_Y, S_WL = ("s40", "s41", "s42", "s43", "s44", "s45",
                                                                              "s46", "s47", "s48", "s49", "s50", "s51")
S_HIT = "s[52:53]"
VGPR_CLOBBERS = list(range(66, 97)) + list(range(102, 133)) + list(range(142, 146)) + list(range(150, 159))
SGPR_CLOBBERS = list(range(40, 54))


def pk(d):
    return f"v{64 + d}"


def entry(d):
    return f"v{100 + d}"


def rotate(d):
    return f"v_mov_b32_dpp {pk(d)}, {pk(d - 1)} {ROL}"


def address(d):
    return f"v_and_or_b32 {entry(d)}, {pk(d)}, %[mask], {ROWOFS}"


def gather(d):
    return f"ds_read_b32 {entry(d)}, {entry(d)}"


def wait(n):
    return f"s_waitcnt lgkmcnt({n})"


class Scoring:
    """key = D + pk + D of the previous lane; two keys share one v_min3."""

    def __init__(self):
        self.pending, self.count = [], 0

    def one(self, d):
        k = f"v{142 + self.count % 4}"
        self.count += 1
        out = [f"v_add_u32 {k}, {pk(d)}, {entry(d)}", f"v_add_u32_dpp {k}, {entry(d)}, {k} {ROR}"]
        self.pending.append(k)
        if len(self.pending) == 2:
            out.append(f"v_min3_i32 {BEST}, {self.pending[0]}, {self.pending[1]}, {BEST}")
            self.pending = []
        return out

    def batch(self, ds):
        out = []
        for d in ds:
            out += self.one(d)
        return out

    def flush(self):
        out = [f"v_min_i32 {BEST}, {k}, {BEST}" for k in self.pending]
        self.pending = []
        return out


def sweep():
    """All diagonals.  pk(2) is already in its register.  The gathers of a batch go out in one burst; the address
    arithmetic of batch k+2 is interleaved with the scoring of batch k, whose instructions fill the wait states
    between two dependent rotates (the first two batches have nothing to interleave with and take s_nop)."""
    out, score = [], Scoring()
    batches, i = [], 0
    for n in BATCHES:
        batches.append(DIAGONALS[i:i + n])
        i += n
    assert i == len(DIAGONALS)

    def issue(ds, filler):
        s = []
        for d in ds:
            if d != DIAGONALS[0]:
                s.append(rotate(d))
                if filler:
                    s.append(filler.pop(0))
            s.append(address(d))
            s.append(filler.pop(0) if filler else "s_nop 0")
        if s[-1] == "s_nop 0":
            s.pop()
        s += filler
        s += [gather(d) for d in ds]
        return s

    out += issue(batches[0], [])
    out += issue(batches[1], [])
    for k, ds in enumerate(batches):
        in_flight = len(batches[k + 1]) if k + 1 < len(batches) else 0
        out.append(wait(in_flight))
        if k + 2 < len(batches):
            out += issue(batches[k + 2], score.batch(ds))
        else:
            out += score.batch(ds)
    out += score.flush()
    return out


def loop():
    out = ["LOOP_TOP%=:"]
    # partner words and row offsets of this sweep; the loop bound takes the place of two wait states
    out += [f"v_lshl_add_u32 {T0}, %[t], 2, %[rank_bits]",
            f"v_sub_u32 {T0}, {T0}, %[fm]",
            f"v_lshl_add_u32 {ROWOFS}, %[t], 8, %[mbase]",
            f"v_bfrev_b32 {BEST}, -2",
            f"v_mov_b32_dpp {T1}, {T0} {ROL}",
            # every move lowers an integer cost that starts below 64 * 2^16 = 2^22: never taken, it only bounds the loop
            "s_bitcmp1_b32 %[applied], 22",
            "s_cbranch_scc1 LOOP_DONE%=",
            f"v_mov_b32_dpp {pk(2)}, {T1} {ROL}"]
    out += sweep()
    # this lane's best candidate -> (value, move id); its new hop (t[a], t[b]) is fetched before the winner is known
    out += [f"v_sub_u32 {KEY2}, {BEST}, %[fm]",
            f"v_bfe_u32 {T0}, {KEY2}, 8, 6",
            f"v_cmp_lt_u32 vcc, {T0}, %[ra]",
            f"v_lshl_add_u32 {T1}, {T0}, 6, %[id_flip]",
            f"v_or_b32 {T2}, {T0}, %[id_base]",
            f"v_ashrrev_i32 {KEY2}, 2, {KEY2}",
            f"v_cndmask_b32 {T0}, {T2}, {T1}, vcc",
            f"v_and_or_b32 {KEY2}, {KEY2}, %[himask], {T0}",
            f"v_and_or_b32 {YBEST}, {BEST}, %[mask], {ROWOFS}",
            f"ds_read_b32 {YBEST}, {YBEST}",
            # minimum over the wave; lane 63 ends with it
            f"v_min_i32_dpp {RED}, {KEY2}, {KEY2} quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf",
            f"v_mov_b32_dpp {FNEXT}, %[fm] {ROL}",
            "s_nop 0",
            f"v_min_i32_dpp {RED}, {RED}, {RED} quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf",
            "s_nop 1",
            f"v_min_i32_dpp {RED}, {RED}, {RED} row_half_mirror row_mask:0xf bank_mask:0xf",
            "s_nop 1",
            f"v_min_i32_dpp {RED}, {RED}, {RED} row_mirror row_mask:0xf bank_mask:0xf",
            "s_nop 1",
            f"v_min_i32_dpp {RED}, {RED}, {RED} row_bcast:15 row_mask:0xa bank_mask:0xf",
            "s_nop 1",
            f"v_min_i32_dpp {RED}, {RED}, {RED} row_bcast:31 row_mask:0xc bank_mask:0xf",
            "s_nop 1",
            f"v_readlane_b32 {S_WIN}, {RED}, 63",
            f"s_ashr_i32 {S_DWIN}, {S_WIN}, 12",
            f"s_cmp_lt_i32 {S_DWIN}, 0",
            "s_cbranch_scc0 LOOP_DONE%=",
            # apply the move: reverse ranks mi .. mj of the order; the hops of the reversed piece go with it
            f"s_bfe_u32 {S_MI}, {S_WIN}, 0x60006",
            f"s_and_b32 {S_MJ}, {S_WIN}, 63",
            f"s_sub_i32 {S_DIF}, {S_MJ}, {S_MI}",
            f"s_add_i32 {S_SUM}, {S_MJ}, {S_MI}",
            f"s_lshl_b32 {S_SUM}, {S_SUM}, 2",
            f"v_subrev_u32 {T0}, {S_MI}, %[lane]",
            f"v_sub_u32 {T1}, {S_SUM}, %[lane4]",
            f"v_cmp_ge_u32 vcc, {S_DIF}, {T0}",
            f"s_add_i32 {S_MJ1}, {S_MJ}, 1",
            f"s_and_b32 {S_MJ1}, {S_MJ1}, 63",
            f"v_cndmask_b32 {T1}, %[lane4], {T1}, vcc",
            f"ds_bpermute_b32 %[t], {T1}, %[t]",
            f"ds_bpermute_b32 {T2}, {T1}, {FNEXT}",
            # while the permutes are in flight: the two new hops.  y = hop (t[mi], t[mj+1]) is the winning lane's
            # prefetched entry; x = hop (t[mi-1], t[mj]) follows from the move's value
            f"v_cmp_eq_u32_e64 {S_HIT}, {S_WIN}, {KEY2}",
            f"v_readlane_b32 {S_FA}, %[fm], {S_MI}",
            f"v_readlane_b32 {S_FB}, %[fm], {S_MJ1}",
            f"s_add_i32 %[cur], %[cur], {S_DWIN}",
            f"s_ff1_i32_b64 {S_WL}, {S_HIT}",
            f"s_lshl_b32 {S_X}, {S_DWIN}, 14",
            f"s_add_i32 {S_X}, {S_X}, {S_FA}",
            f"s_add_i32 {S_X}, {S_X}, {S_FB}",
            f"s_add_i32 %[applied], %[applied], 1",
            "s_waitcnt lgkmcnt(2)",
            f"v_readlane_b32 {S_Y}, {YBEST}, {S_WL}",
            f"s_sub_i32 {S_X}, {S_X}, {S_Y}",
            f"s_mov_b32 m0, {S_MI}",
            "s_waitcnt lgkmcnt(0)",
            f"v_cndmask_b32 %[fm], %[fm], {T2}, vcc",
            f"v_writelane_b32 %[fm], {S_X}, m0",
            f"s_mov_b32 m0, {S_MJ1}",
            "s_nop 0",
            f"v_writelane_b32 %[fm], {S_Y}, m0",
            "s_branch LOOP_TOP%=",
            "LOOP_DONE%=:"]
    return out


def operands(lane, rank_a, mbase):
    """The read-only operands of the asm statement as cc_2opt_n64.hip computes them (lane = 0 .. 63,
    rank_a = (lane - 1) mod 64, mbase = LDS byte offset of the matrix): for the CPU model of the loop in the tests."""
    return {"rank_bits": rank_a << 8, "ra": rank_a, "id_base": lane * 64, "id_flip": 64 + rank_a, "lane": lane,
            "lane4": lane << 2, "mbase": mbase, "mask": 0xff, "himask": 0xfffff000}


def text():
    lines = loop()
    out = ["// Generated by gen_2opt_n64_loop.py - do not edit by hand.  The descent loop of twoopt_sum_n64_kernel for matrices",
           "// with entries below 2^16 (32-bit keys); operands and register use are described in the generator.",
           "#define CC_N64_DESCENT_LOOP_ASM \\"]
    for i, l in enumerate(lines):
        out.append(f'    "{l}\\n\\t"' + (" \\" if i + 1 < len(lines) else ""))
    clob = ", ".join([f'"v{r}"' for r in VGPR_CLOBBERS] + [f'"s{r}"' for r in SGPR_CLOBBERS]
                     + ['"vcc"', '"scc"', '"m0"', '"memory"'])
    out += ["", f"#define CC_N64_DESCENT_LOOP_CLOBBERS {clob}", ""]
    return "\n".join(out)


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "cc_2opt_n64_loop.inc")
    with open(path, "w") as fh:
        fh.write(text())
    print(len(loop()), "lines ->", path)
