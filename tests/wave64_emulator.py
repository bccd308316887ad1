"""A small interpreter for the subset of the gfx9 wave64 instruction set that the hand-written descent loop of the
N = 64 ring-sum kernel uses (csrc/cc_2opt_n64_loop.inc): 64 lanes of 32-bit VGPRs, SGPRs, VCC, SCC, M0, an LDS image,
DPP lane selections, labels and branches.  It executes the committed loop text on the CPU, one instruction at a
time in program order (timing, wait states and s_waitcnt are the business of the static checks, not of this model),
so that what the loop computes can be compared with the oracle without a GPU.  CPU test infrastructure only."""
import re

import numpy as np

M32 = 0xffffffff
LANES = np.arange(64)


def _i32(x):
    return ((np.asarray(x, dtype=np.int64) & M32) ^ 0x80000000) - 0x80000000


def _dpp_source_lane(ctrl):
    """lane -> (source lane, valid) for one DPP control string."""
    m = re.search(r"quad_perm:\[(\d),(\d),(\d),(\d)\]", ctrl)
    if m:
        perm = np.array([int(g) for g in m.groups()])
        return (LANES & ~3) + perm[LANES & 3], np.ones(64, bool)
    if "wave_rol:1" in ctrl:
        return (LANES + 1) & 63, np.ones(64, bool)
    if "wave_ror:1" in ctrl:
        return (LANES - 1) & 63, np.ones(64, bool)
    if "row_half_mirror" in ctrl:
        return (LANES & ~7) + 7 - (LANES & 7), np.ones(64, bool)
    if "row_mirror" in ctrl:
        return (LANES & ~15) + 15 - (LANES & 15), np.ones(64, bool)
    m = re.search(r"row_bcast:(15|31)", ctrl)
    if m:
        if m.group(1) == "15":                       # lane 15 of every row to the whole next row
            return ((LANES & ~15) - 1) & 63, LANES >= 16
        return np.full(64, 31), LANES >= 32          # lane 31 to rows 2 and 3
    raise ValueError(f"unknown DPP control: {ctrl}")


def _row_enable(ctrl):
    m = re.search(r"row_mask:0x([0-9a-f])", ctrl)
    mask = int(m.group(1), 16) if m else 0xf
    return ((mask >> (LANES >> 4)) & 1).astype(bool)


class Wave:
    def __init__(self, lds_bytes, operands):
        """lds_bytes: numpy uint8 image of the LDS; operands: name -> int (scalar) or array of 64 (vector) for the
        %[name] operands of the asm statement."""
        self.lds = np.frombuffer(bytes(lds_bytes), dtype="<u4").copy()
        self.v, self.s = {}, {}
        self.named = {k: (np.asarray(x, dtype=np.int64) & M32) if np.ndim(x) else int(x) & M32 for k, x in operands.items()}
        self.vcc = np.zeros(64, bool)
        self.scc = False
        self.executed = 0

    # ---- operands
    def get(self, tok, vector=True):
        tok = tok.strip()
        if tok.startswith("%["):
            x = self.named[tok[2:-1]]
        elif re.fullmatch(r"v\d+", tok):
            x = self.v[tok]
        elif re.fullmatch(r"s\d+", tok) or tok == "m0":
            x = self.s[tok]
        elif re.fullmatch(r"s\[\d+:\d+\]", tok):
            x = self.s[tok]
        elif tok == "vcc":
            return self.vcc
        else:
            x = int(tok, 0) & M32
        if vector and not np.ndim(x):
            return np.full(64, x, dtype=np.int64)
        return x

    def put(self, tok, val, lanes=None):
        tok = tok.strip()
        if tok.startswith("%["):
            name = tok[2:-1]
            if np.ndim(self.named[name]):
                cur = self.named[name].copy()
                if lanes is None:
                    cur = np.asarray(val, dtype=np.int64) & M32
                else:
                    cur[lanes] = (np.asarray(val, dtype=np.int64) & M32)[lanes]
                self.named[name] = cur
            else:
                self.named[name] = int(val) & M32
        elif tok.startswith("v"):
            new = np.asarray(val, dtype=np.int64) & M32
            if lanes is None:
                self.v[tok] = new.copy()
            else:
                cur = self.v.get(tok, np.zeros(64, dtype=np.int64)).copy()
                cur[lanes] = new[lanes]
                self.v[tok] = cur
        else:
            self.s[tok] = int(val) & (M32 if not tok.startswith("s[") else 0xffffffffffffffff)

    # ---- execution
    def run(self, lines, limit=10_000_000):
        labels = {l[:-1]: i for i, l in enumerate(lines) if l.endswith(":")}
        pc = 0
        while pc < len(lines):
            ins = lines[pc]
            pc += 1
            if ins.endswith(":"):
                continue
            self.executed += 1
            if self.executed > limit:
                raise RuntimeError("instruction limit reached: the loop does not end")
            target = self.step(ins)
            if target is not None:
                pc = labels[target]

    def step(self, ins):
        op, _, rest = ins.partition(" ")
        ctrl = ""
        m = re.search(r"\s(quad_perm|wave_ro[lr]|row_half_mirror|row_mirror|row_bcast)", rest)
        if m:
            rest, ctrl = rest[:m.start()], rest[m.start():]
        a = [x.strip() for x in rest.split(",")] if rest.strip() else []
        g, gi = self.get, lambda t: _i32(self.get(t))
        if op in ("s_nop", "s_waitcnt"):
            return None
        if op == "s_branch":
            return a[0]
        if op == "s_cbranch_scc1":
            return a[0] if self.scc else None
        if op == "s_cbranch_scc0":
            return None if self.scc else a[0]
        if op.endswith("_dpp"):
            src_lane, valid = _dpp_source_lane(ctrl)
            enable = _row_enable(ctrl) & (valid | ("bound_ctrl:1" in ctrl))
            x = g(a[1])[src_lane]
            if "bound_ctrl:1" in ctrl:
                x = np.where(valid, x, 0)
            base = op[:-4]
            if base == "v_mov_b32":
                res = x
            elif base == "v_add_u32":
                res = x + g(a[2])
            elif base == "v_sub_u32":
                res = x - g(a[2])
            elif base == "v_min_i32":
                res = np.minimum(_i32(x), gi(a[2]))
            else:
                raise ValueError(ins)
            self.put(a[0], res, lanes=enable)
            return None
        sc = lambda t: int(self.get(t, vector=False))            # noqa: E731  scalar operand
        si = lambda t: int(_i32(sc(t)))                          # noqa: E731
        if op == "v_add_u32":
            self.put(a[0], g(a[1]) + g(a[2]))
        elif op == "v_sub_u32":
            self.put(a[0], g(a[1]) - g(a[2]))
        elif op == "v_subrev_u32":
            self.put(a[0], g(a[2]) - g(a[1]))
        elif op == "v_lshl_add_u32":
            self.put(a[0], (g(a[1]) << (sc(a[2]) & 31)) + g(a[3]))
        elif op == "v_lshl_or_b32":
            self.put(a[0], (g(a[1]) << (sc(a[2]) & 31)) | g(a[3]))
        elif op == "v_lshlrev_b32":
            self.put(a[0], g(a[2]) << (sc(a[1]) & 31))
        elif op == "v_and_or_b32":
            self.put(a[0], (g(a[1]) & g(a[2])) | g(a[3]))
        elif op == "v_or_b32":
            self.put(a[0], g(a[1]) | g(a[2]))
        elif op == "v_mov_b32":
            self.put(a[0], g(a[1]))
        elif op == "v_ashrrev_i32":
            self.put(a[0], gi(a[2]) >> (sc(a[1]) & 31))
        elif op == "v_bfe_u32":
            self.put(a[0], (g(a[1]) >> (sc(a[2]) & 31)) & ((1 << sc(a[3])) - 1))
        elif op == "v_bfrev_b32":
            x = sc(a[1])
            self.put(a[0], np.full(64, int(f"{x:032b}"[::-1], 2)))
        elif op == "v_min_i32":
            self.put(a[0], np.minimum(gi(a[1]), gi(a[2])))
        elif op == "v_min3_i32":
            self.put(a[0], np.minimum(np.minimum(gi(a[1]), gi(a[2])), gi(a[3])))
        elif op in ("v_cmp_lt_u32", "v_cmp_ge_u32", "v_cmp_eq_u32_e64"):
            x, y = g(a[1]), g(a[2])
            r = x < y if "lt" in op else x >= y if "ge" in op else x == y
            if a[0] == "vcc":
                self.vcc = r
            else:
                self.s[a[0]] = int(sum(1 << int(i) for i in LANES[r]))
        elif op == "v_cndmask_b32":
            self.put(a[0], np.where(self.vcc, g(a[2]), g(a[1])))
        elif op == "v_readlane_b32":
            self.put(a[0], int(g(a[1])[sc(a[2]) & 63]))
        elif op == "v_writelane_b32":
            lane = np.zeros(64, bool)
            lane[sc(a[2]) & 63] = True
            self.put(a[0], np.full(64, sc(a[1])), lanes=lane)
        elif op == "ds_read_b32":
            addr = g(a[1])
            assert not (addr & 3).any() and (addr // 4 < len(self.lds)).all(), f"{ins}: address outside the LDS image"
            self.put(a[0], self.lds[addr // 4].astype(np.int64))
        elif op == "ds_bpermute_b32":
            self.put(a[0], g(a[2])[(g(a[1]) >> 2) & 63])
        elif op == "s_mov_b32":
            self.put(a[0], sc(a[1]))
        elif op == "s_add_i32":
            self.put(a[0], sc(a[1]) + sc(a[2]))
        elif op == "s_sub_i32":
            self.put(a[0], sc(a[1]) - sc(a[2]))
        elif op == "s_and_b32":
            self.put(a[0], sc(a[1]) & sc(a[2]))
        elif op == "s_lshl_b32":
            self.put(a[0], sc(a[1]) << (sc(a[2]) & 31))
        elif op == "s_ashr_i32":
            self.put(a[0], si(a[1]) >> (sc(a[2]) & 31))
        elif op == "s_bfe_u32":
            spec = sc(a[2])
            self.put(a[0], (sc(a[1]) >> (spec & 31)) & ((1 << ((spec >> 16) & 0x7f)) - 1))
        elif op == "s_cmp_lt_i32":
            self.scc = si(a[0]) < si(a[1])
        elif op == "s_bitcmp1_b32":
            self.scc = bool((sc(a[0]) >> (sc(a[1]) & 31)) & 1)
        elif op == "s_ff1_i32_b64":
            x = sc(a[1])
            self.put(a[0], (x & -x).bit_length() - 1 if x else M32)
        else:
            raise ValueError(f"instruction not modelled: {ins}")
        return None
