"""Address-level emulator for this project's own gfx950 code objects (test infrastructure).

The code object is disassembled with llvm-objdump and run wave by wave: scalar, integer-vector, execution-mask,
cross-lane and accumulation-register instructions are emulated exactly, floating-point data is not (float results are
written as 0: no address may depend on them).  Every register starts with a value that makes any address built from it
invalid, as on the GPU, where a wave inherits whatever the previous one left.  Every LDS and global access of every
active lane is checked against the allocation it should fall in.  This sees what a source-level check cannot: what
the compiler did, e.g. spill code placed where the execution mask is empty (the value is lost, the reload returns the
register's old content, and an address built from it points anywhere).

check(hsaco, lds_bytes, B, grid, row_words, elt) -> list of problems (empty: every access in bounds).
exec_zero_windows(hsaco) -> vector instructions between the exit of a divergent loop (lanes leave at different
times: exec &= ~done; branch back while exec != 0) and the next write to exec: they run with an empty mask.
"""
import re, struct, subprocess
import numpy as np

OBJDUMP = "/opt/rocm/llvm/bin/llvm-objdump"

M32 = 0xFFFFFFFF
FLOAT_OPS = {"v_add_f64", "v_fmac_f64_e32", "v_mul_f64", "v_fma_f64", "v_fmac_f32_e32", "v_fma_f32", "v_mul_f32_e32", "v_add_f32_e32",
             "v_mul_f32_e64", "v_fmac_f64_e64", "v_add_f32_e64", "v_sub_f32_e32", "v_fmac_f32_e64"}


def load(hsaco):
    txt = subprocess.run([OBJDUMP, "-d", "--no-show-raw-insn", hsaco], capture_output=True, text=True).stdout
    prog, base = [], None
    for l in txt.split("\n"):
        m = re.match(r"\s+(\S.*?)\s*//\s*([0-9A-F]{12}):(.*)$", l)
        if not m: continue
        ins, addr, rest = m.group(1), int(m.group(2), 16), m.group(3)
        if base is None: base = addr
        t = re.search(r"<[^>]*\+0x([0-9a-f]+)>", rest)
        prog.append((addr, ins, base + int(t.group(1), 16) if t else None))
    return prog


class OOB(Exception):
    pass


class Emu:
    def __init__(self, prog, lds_size, kernarg, buffers):
        self.prog = prog; self.idx = {a: i for i, (a, _, _) in enumerate(prog)}
        self.lds_size = lds_size; self.kernarg = kernarg; self.buffers = buffers
        self.KA = 0x7000_0000_0000
        self.problems = []
        self.track = True
        self.trace = False; self.trace_log = []
        self.written = {}

    def run(self, wg_id, wave=0, max_steps=10_000_000):
        # registers hold whatever the previous wave left: a value that makes any address built from it invalid
        P = 0xDEADBEE0
        self.s = np.full(128, P, dtype=np.uint64)     # 32-bit values, kept in 64-bit cells
        self.v = np.full((512, 64), P, dtype=np.uint64)
        self.a = np.full((512, 64), P, dtype=np.uint64)
        self.vcc = 0; self.exec = (1 << 64) - 1; self.scc = 0; self.scratch = {}
        # "undefined" flags: a register lane (scalar register, LDS word, private-memory word) no instruction has written
        # with a defined value.  Only the registers the hardware initialises start defined.
        self.us = np.ones(128, dtype=bool); self.us[0:3] = False
        self.uv = np.ones((512, 64), dtype=bool); self.uv[0] = False
        self.ua = np.ones((512, 64), dtype=bool)
        self.uvcc = self.uexec = self.uscc = False
        self.ulds = np.ones(self.lds_size // 4 + 4, dtype=bool)
        self.uscratch = {}
        self.fexact = set()       # vector registers whose float value was computed exactly (cvt / rcp / mul chain of a division)
        self.s[0] = self.KA & M32; self.s[1] = self.KA >> 32; self.s[2] = wg_id
        self.v[0] = np.arange(64, dtype=np.uint64) + np.uint64(64 * wave)
        pc = 0; steps = 0
        while True:
            addr, ins, tgt = self.prog[pc]
            steps += 1
            if steps > max_steps: raise RuntimeError("step limit")
            op, _, rest = ins.partition(" ")
            if op == "s_endpgm": return steps
            nxt = pc + 1
            if self.track and ((op.startswith("s_cbranch_exec") and self.uexec) or (op.startswith("s_cbranch_vcc") and self.uvcc)
                               or (op.startswith("s_cbranch_scc") and self.uscc)):
                self.note(f"{addr:x}: {ins}: branch on a value derived from an undefined register or lane")
            if op in ("s_branch",): nxt = self.idx[tgt]
            elif op == "s_cbranch_execz": nxt = self.idx[tgt] if self.exec == 0 else nxt
            elif op == "s_cbranch_execnz": nxt = self.idx[tgt] if self.exec != 0 else nxt
            elif op == "s_cbranch_vccnz": nxt = self.idx[tgt] if self.vcc != 0 else nxt
            elif op == "s_cbranch_vccz": nxt = self.idx[tgt] if self.vcc == 0 else nxt
            elif op == "s_cbranch_scc0": nxt = self.idx[tgt] if self.scc == 0 else nxt
            elif op == "s_cbranch_scc1": nxt = self.idx[tgt] if self.scc == 1 else nxt
            elif op in ("s_waitcnt", "s_nop", "s_setprio", "s_barrier", "s_sleep"): pass
            else:
                self.jump = None
                if self.track: self.flow(addr, op, rest.strip())
                self.step(addr, op, rest.strip())
                if self.jump is not None: nxt = self.idx[self.jump]
            pc = nxt

    # ---- operands
    def split(self, rest):
        out, depth, cur = [], 0, ""
        for ch in rest:
            if ch == "[": depth += 1
            if ch == "]": depth -= 1
            if ch == "," and depth == 0: out.append(cur.strip()); cur = ""
            else: cur += ch
        if cur.strip(): out.append(cur.strip())
        return out

    def rng(self, tok):
        m = re.fullmatch(r"([sva])(\d+)", tok)
        if m: return m.group(1), int(m.group(2)), 1
        m = re.fullmatch(r"([sva])\[(\d+):(\d+)\]", tok)
        if m: return m.group(1), int(m.group(2)), int(m.group(3)) - int(m.group(2)) + 1
        return None

    def rd_s32(self, tok):            # scalar 32-bit source
        if tok == "vcc_lo": return self.vcc & M32
        if tok == "vcc_hi": return self.vcc >> 32
        if tok == "exec_lo": return self.exec & M32
        if tok == "exec_hi": return self.exec >> 32
        r = self.rng(tok)
        if r: assert r[0] == "s" and r[2] == 1, tok; return int(self.s[r[1]])
        return self.lit(tok) & M32

    def lit(self, tok):
        if re.fullmatch(r"-?\d+", tok): return int(tok)
        if re.fullmatch(r"0x[0-9a-fA-F]+", tok): return int(tok, 16)
        if re.fullmatch(r"-?\d+\.\d*(e[-+]?\d+)?", tok): return 0      # float inline constant: data only
        raise ValueError("literal " + tok)

    def rd_s64(self, tok):
        if tok == "vcc": return self.vcc
        if tok == "exec": return self.exec
        r = self.rng(tok)
        if r: assert r[0] == "s" and r[2] == 2, tok; return int(self.s[r[1]]) | (int(self.s[r[1] + 1]) << 32)
        v = self.lit(tok)
        return v & ((1 << 64) - 1)

    def wr_s64(self, tok, val):
        val &= (1 << 64) - 1
        if tok == "vcc": self.vcc = val; return
        if tok == "exec": self.exec = val; return
        r = self.rng(tok); assert r and r[0] == "s" and r[2] == 2, tok
        self.s[r[1]] = val & M32; self.s[r[1] + 1] = val >> 32

    def wr_s32(self, tok, val):
        if tok == "vcc_lo": self.vcc = (self.vcc & ~M32) | (val & M32); return
        if tok == "vcc_hi": self.vcc = (self.vcc & M32) | ((val & M32) << 32); return
        r = self.rng(tok); assert r and r[0] == "s" and r[2] == 1, tok
        self.s[r[1]] = val & M32

    def rd_v32(self, tok):            # per-lane 32-bit source (vector, scalar or literal) -> uint64[64]
        r = self.rng(tok)
        if r and r[0] == "v": assert r[2] == 1; return self.v[r[1]].copy()
        if r and r[0] == "a": assert r[2] == 1; return self.a[r[1]].copy()
        return np.full(64, self.rd_s32(tok), dtype=np.uint64)

    def rd_v64(self, tok):
        r = self.rng(tok)
        if r and r[0] in "va":
            assert r[2] == 2, tok
            f = self.v if r[0] == "v" else self.a
            return f[r[1]] | (f[r[1] + 1] << np.uint64(32))
        if r or tok in ("vcc", "exec"): return np.full(64, self.rd_s64(tok), dtype=np.uint64)
        return np.full(64, self.lit(tok) & ((1 << 64) - 1), dtype=np.uint64)

    def mask(self):
        return np.array([(self.exec >> i) & 1 for i in range(64)], dtype=bool)

    def wr_v(self, tok, vals, n=1, m=None):          # vals: uint64[64] (n == 1: low 32 bits; n == 2: 64 bits)
        self.fexact.discard(tok)
        r = self.rng(tok); assert r and r[0] in "va", tok
        f = self.v if r[0] == "v" else self.a
        m = self.mask() if m is None else m
        if n == 1: f[r[1]][m] = vals[m] & np.uint64(M32)
        else:
            assert r[2] == 2, tok
            f[r[1]][m] = vals[m] & np.uint64(M32); f[r[1] + 1][m] = vals[m] >> np.uint64(32)

    def wr_zero(self, tok):
        self.fexact.discard(tok)
        r = self.rng(tok); assert r and r[0] in "va", tok
        f = self.v if r[0] == "v" else self.a
        m = self.mask()
        for k in range(r[2]): f[r[1] + k][m] = 0

    def bits(self, arr):
        v = 0
        for i in range(64):
            if arr[i]: v |= 1 << i
        return v

    @staticmethod
    def s32(a):         # uint64 array holding 32-bit values -> signed int64
        a = a.astype(np.int64)
        return np.where(a >= (1 << 31), a - (1 << 32), a)

    # ---- memory checks
    def fetch(self, a, ndw):            # dwords at address a from a buffer that has contents; else None
        for t in self.buffers:
            if len(t) > 3 and t[3] is not None and t[0] <= a and a + 4 * ndw <= t[0] + t[1]:
                return struct.unpack_from("<%dI" % ndw, t[3], a - t[0])
        return None

    def check_global(self, addr_txt, ins, addrs, size, m):
        for lane in np.flatnonzero(m):
            a = int(addrs[lane])
            ok = any(t[0] <= a and a + size <= t[0] + t[1] for t in self.buffers)
            if not ok:
                near = min(self.buffers, key=lambda t: abs(t[0] - a))
                self.problems.append(f"{addr_txt:x}: {ins}: lane {lane} global address {a:#x} size {size} outside every buffer (nearest {near[2]} base {near[0]:#x} bytes {near[1]})")
                raise OOB()

    def mark_written(self, addrs, size, m):
        for lane in np.flatnonzero(m):
            a = int(addrs[lane])
            for t in self.buffers:
                if t[0] <= a < t[0] + t[1]:
                    self.written.setdefault(t[2], np.zeros(t[1], dtype=bool))[a - t[0]:a - t[0] + size] = True

    def unwritten(self, name):          # first byte of buffer `name` that no store has touched, or None
        for t in self.buffers:
            if t[2] == name:
                w = self.written.get(name, np.zeros(t[1], dtype=bool))
                gap = np.flatnonzero(~w)
                return int(gap[0]) if len(gap) else None
        raise KeyError(name)

    def check_lds(self, addr_txt, ins, addrs, size, m):
        for lane in np.flatnonzero(m):
            a = int(addrs[lane])
            if a + size > self.lds_size:
                self.problems.append(f"{addr_txt:x}: {ins}: lane {lane} LDS address {a} size {size} beyond {self.lds_size}")
                raise OOB()
            if a % min(size, 8):
                self.problems.append(f"{addr_txt:x}: {ins}: lane {lane} LDS address {a} misaligned for {size}")

    # ---- definedness of values (which lanes of which registers hold something an instruction computed)
    def note(self, text):
        if text not in self.problems: self.problems.append(text)

    def U(self, tok):                 # undefined flags of an operand, per lane
        tok = tok.strip().lstrip("-").strip("|")
        if tok == "vcc" or tok.startswith("vcc_"): return np.full(64, self.uvcc)
        if tok == "exec" or tok.startswith("exec_"): return np.full(64, self.uexec)
        r = self.rng(tok)
        if not r: return np.zeros(64, dtype=bool)
        if r[0] == "s": return np.full(64, bool(self.us[r[1]:r[1] + r[2]].any()))
        f = self.uv if r[0] == "v" else self.ua
        return f[r[1]:r[1] + r[2]].any(axis=0)

    def setU(self, tok, u, m=None):
        tok = tok.strip()
        if tok == "vcc" or tok.startswith("vcc_"): self.uvcc = bool(np.any(u)); return
        if tok == "exec": self.uexec = bool(np.any(u)); return
        r = self.rng(tok)
        if not r: return
        if r[0] == "s": self.us[r[1]:r[1] + r[2]] = bool(np.any(u)); return
        f = self.uv if r[0] == "v" else self.ua
        m = self.mask() if m is None else m
        for k in range(r[2]): f[r[1] + k][m] = u[m]

    def dpp_source(self, rest):
        i = np.arange(64)
        m = re.search(r"quad_perm:\[(\d),(\d),(\d),(\d)\]", rest)
        if m: q = np.array([int(t) for t in m.groups()]); return (i & ~3) | q[i & 3]
        if "row_mirror" in rest: return (i & ~15) | (15 - (i & 15))
        if "row_half_mirror" in rest: return (i & ~7) | (7 - (i & 7))
        raise NotImplementedError("dpp " + rest)

    def flow(self, addr, op, rest):
        o = self.split(re.sub(r"\s+(offset\d?:\S+|nt|sc0|sc1|quad_perm:\S+|row_\w+(:\S+)?|row_mask:\S+|bank_mask:\S+|bound_ctrl:\S+)", lambda mm: " \x00" + mm.group(1), rest).split("\x00")[0])
        mods = dict(re.findall(r"(offset\d?):(\S+)", rest))
        ins = op + " " + rest
        m = self.mask()
        anyu = lambda toks: np.logical_or.reduce([self.U(t) for t in toks]) if toks else np.zeros(64, dtype=bool)
        if op in ("buffer_wbl2", "buffer_inv"): return
        if op.startswith("s_"):
            if op in ("s_getpc_b64",): self.setU(o[0], False); return
            if op == "s_setpc_b64":
                if self.U(o[0]).any(): self.note(f"{addr:x}: {ins}: jump to an undefined address")
                return
            if op.startswith("s_load_dword"): self.setU(o[0], self.U(o[1]).any()); return
            if op.startswith(("s_cmp", "s_bitcmp")): self.uscc = bool(anyu(o).any()); return
            src = o[1:] + ([o[0]] if op in ("s_addk_i32", "s_mulk_i32", "s_bitset1_b32") else [])
            u = bool(anyu(src).any()) or (op in ("s_addc_u32", "s_subb_u32") and self.uscc)
            if op in ("buffer_wbl2", "buffer_inv"): return
            if op in ("s_cselect_b32", "s_cselect_b64"): self.setU(o[0], bool(anyu(o[1:]).any()) or self.uscc); return
            if op in ("s_and_saveexec_b64", "s_or_saveexec_b64", "s_andn2_saveexec_b64"):
                self.setU(o[0], self.uexec); self.uexec = self.uexec or u; self.uscc = self.uexec; return
            self.setU(o[0], u)
            if not op.startswith(("s_mov", "s_movk")): self.uscc = u
            return
        if op == "v_readlane_b32":
            r = self.rng(o[1]); lane = self.rd_s32(o[2]) & 63
            self.setU(o[0], bool((self.uv if r[0] == "v" else self.ua)[r[1]][lane]) or self.U(o[2]).any()); return
        if op == "v_readfirstlane_b32":
            r = self.rng(o[1]); lane = int(np.flatnonzero(m)[0]) if m.any() else 0
            self.setU(o[0], bool(self.uv[r[1]][lane]) or self.uexec); return
        if op == "v_writelane_b32":
            r = self.rng(o[0]); lane = self.rd_s32(o[2]) & 63
            self.uv[r[1]][lane] = bool(self.U(o[1]).any() or self.U(o[2]).any()); return
        if op.startswith("v_cmp_"):
            self.setU(o[0], bool(((self.U(o[1]) | self.U(o[2])) & m).any()) or self.uexec); return
        if op.startswith("v_cndmask_b32"):
            sel = self.vcc if op.endswith("e32") else self.rd_s64(o[3])
            selv = np.array([(sel >> i) & 1 for i in range(64)], dtype=bool)
            self.setU(o[0], np.where(selv, self.U(o[2]), self.U(o[1])) | self.U(o[3] if len(o) > 3 else "vcc")); return
        if op.endswith("_dpp"):
            src = self.dpp_source(rest)
            self.setU(o[0], self.U(o[1])[src] | (~m)[src]); return      # a lane that is switched off supplies nothing defined
        if op.startswith(("global_load", "global_store")):
            load_ = op.startswith("global_load")
            at, sa = (o[1], o[2]) if load_ else (o[0], o[2])
            ua = self.U(at) | (np.zeros(64, dtype=bool) if sa == "off" else self.U(sa))
            if (ua & m).any(): self.note(f"{addr:x}: {ins}: address built from an undefined register or lane (lane {int(np.flatnonzero(ua & m)[0])})")
            if load_: self.setU(o[0], np.zeros(64, dtype=bool))
            elif (self.U(o[1]) & m).any():
                self.note(f"{addr:x}: {ins}: stores a value derived from an undefined register or lane (lane {int(np.flatnonzero(self.U(o[1]) & m)[0])})")
            return
        if op.startswith(("ds_read", "ds_write")):
            rd = op.startswith("ds_read")
            at = o[1] if rd else o[0]
            if (self.U(at) & m).any(): self.note(f"{addr:x}: {ins}: LDS address built from an undefined register or lane"); return
            base = self.rd_v32(at)
            two = bool(re.search(r"2(st64)?_b(32|64)$", op))
            el = 8 if "b64" in op else 4 if "b32" in op else {"b96": 12, "b128": 16}[op.split("_")[-1]]
            unit = el * (64 if "st64" in op else 1)
            offs = [self.lit(mods.get(k, "0")) * unit for k in ("offset0", "offset1")] if two else [self.lit(mods.get("offset", "0"))]
            nd = el // 4
            if rd:
                r = self.rng(o[0]); f = self.uv if r[0] == "v" else self.ua
                for t, off in enumerate(offs):
                    w = ((base + np.uint64(off)) >> np.uint64(2)).astype(np.int64)
                    for k in range(nd):
                        idx = np.clip(w + k, 0, len(self.ulds) - 1)
                        f[r[1] + t * nd + k][m] = self.ulds[idx][m]
                        if self.trace and (self.ulds[idx] & m).any() and len(self.trace_log) < 40:
                            l_ = int(np.flatnonzero(self.ulds[idx] & m)[0])
                            self.trace_log.append(f"{addr:x}: {ins}: lane {l_} reads LDS word {int(idx[l_])} that holds nothing defined")
            else:
                datas = o[1:1 + len(offs)]
                for t, off in enumerate(offs):
                    r = self.rng(datas[t]); f = self.uv if r[0] == "v" else self.ua
                    w = ((base + np.uint64(off)) >> np.uint64(2)).astype(np.int64)
                    for k in range(nd):
                        idx = np.clip(w + k, 0, len(self.ulds) - 1)
                        self.ulds[idx[m]] = f[r[1] + k][m]
            return
        if op.startswith(("scratch_store", "scratch_load")):
            n = {"dword": 1, "dwordx2": 2, "dwordx3": 3, "dwordx4": 4}[op.split("_")[-1]]
            st = op.startswith("scratch_store")
            data, sa = (o[1], o[2]) if st else (o[0], o[2])
            base = self.lit(mods.get("offset", "0")) + (0 if sa == "off" else self.rd_s32(sa))
            r = self.rng(data); f = self.uv if r[0] == "v" else self.ua
            for k in range(n):
                cell = self.uscratch.setdefault(base + 4 * k, np.ones(64, dtype=bool))
                if st: cell[m] = f[r[1] + k][m]
                else: f[r[1] + k][m] = cell[m]
            return
        if op == "ds_bpermute_b32":
            src = ((self.rd_v32(o[1]) + np.uint64(self.lit(mods.get("offset", "0")))) >> np.uint64(2)).astype(np.int64) & 63
            self.setU(o[0], (self.U(o[2])[src] & m[src]) | self.U(o[1])); return
        if op in ("v_mad_u64_u32", "v_mad_i64_i32"):       # the low word of a * b + c does not depend on the high word of c
            r, c = self.rng(o[0]), self.rng(o[4])
            lo = self.U(o[2]) | self.U(o[3]) | (self.U(f"{c[0]}{c[1]}") if c else np.zeros(64, dtype=bool))
            hi = lo | self.U(o[4])
            self.setU(f"{r[0]}{r[1]}", lo); self.setU(f"{r[0]}{r[1] + 1}", hi); self.setU(o[1], bool((hi & m).any()))
            return
        # vector ALU: every listed source; accumulating forms also read their destination
        two_dest = "_co_" in op or op in ("v_mad_u64_u32", "v_mad_i64_i32")
        src = o[2:] if two_dest else o[1:]
        if re.match(r"v_(fmac|mac)_", op): src = src + [o[0]]
        u = anyu(src)
        if self.trace and (u & m).any() and len(self.trace_log) < 40:
            self.trace_log.append(f"{addr:x}: {ins}: active lane {int(np.flatnonzero(u & m)[0])} consumes an undefined value from " +
                                  ", ".join(t for t in src if (self.U(t) & m).any()))
        self.setU(o[0], u)
        if two_dest: self.setU(o[1], bool((u & m).any()))

    def step(self, addr, op, rest):
        o = self.split(re.sub(r"\s+(offset\d?:\S+|nt|sc0|sc1|quad_perm:\S+|row_\w+:\S+|row_mask:\S+|bank_mask:\S+|bound_ctrl:\S+|row_bcast:\d+|wave_\w+:\d+)", lambda mm: " \x00" + mm.group(1), rest).split("\x00")[0])
        mods = dict(re.findall(r"(offset\d?):(\S+)", rest))
        ins = op + " " + rest
        u64 = np.uint64
        # ---------------- SALU
        if op == "s_mov_b32": self.wr_s32(o[0], self.rd_s32(o[1]))
        elif op == "s_mov_b64": self.wr_s64(o[0], self.rd_s64(o[1]))
        elif op == "s_movk_i32": self.wr_s32(o[0], self.lit(o[1]) & M32 if self.lit(o[1]) < 0x8000 else (self.lit(o[1]) - 0x10000) & M32)
        elif op == "s_addk_i32":
            k = self.lit(o[1]); k = k - 0x10000 if k >= 0x8000 else k
            self.wr_s32(o[0], (self.rd_s32(o[0]) + k) & M32)
        elif op in ("s_add_u32", "s_add_i32"):
            t = self.rd_s32(o[1]) + self.rd_s32(o[2]); self.scc = t >> 32 if op == "s_add_u32" else self.scc; self.wr_s32(o[0], t)
        elif op == "s_addc_u32":
            t = self.rd_s32(o[1]) + self.rd_s32(o[2]) + self.scc; self.scc = t >> 32; self.wr_s32(o[0], t)
        elif op == "s_sub_u32" or op == "s_sub_i32":
            t = self.rd_s32(o[1]) - self.rd_s32(o[2]); self.scc = 1 if t < 0 else 0; self.wr_s32(o[0], t)
        elif op == "s_subb_u32":
            t = self.rd_s32(o[1]) - self.rd_s32(o[2]) - self.scc; self.scc = 1 if t < 0 else 0; self.wr_s32(o[0], t)
        elif op == "s_mul_i32": self.wr_s32(o[0], (self.rd_s32(o[1]) * self.rd_s32(o[2])) & M32)
        elif op in ("s_cselect_b32",): self.wr_s32(o[0], self.rd_s32(o[1]) if self.scc else self.rd_s32(o[2]))
        elif op in ("s_cselect_b64",): self.wr_s64(o[0], self.rd_s64(o[1]) if self.scc else self.rd_s64(o[2]))
        elif re.fullmatch(r"s_cmp_(eq|lg|gt|ge|lt|le)_(u32|i32|u64)", op):
            mm = re.fullmatch(r"s_cmp_(eq|lg|gt|ge|lt|le)_(u32|i32|u64)", op)
            if mm.group(2) == "u64": A, Bv = self.rd_s64(o[0]), self.rd_s64(o[1])
            else:
                A, Bv = self.rd_s32(o[0]), self.rd_s32(o[1])
                if mm.group(2) == "i32": A, Bv = (t - (1 << 32) if t >= (1 << 31) else t for t in (A, Bv))
            self.scc = int({"eq": A == Bv, "lg": A != Bv, "gt": A > Bv, "ge": A >= Bv, "lt": A < Bv, "le": A <= Bv}[mm.group(1)])
        elif op == "s_min_u32": A, Bv = self.rd_s32(o[1]), self.rd_s32(o[2]); self.wr_s32(o[0], min(A, Bv)); self.scc = int(A < Bv)
        elif op == "s_max_u32": A, Bv = self.rd_s32(o[1]), self.rd_s32(o[2]); self.wr_s32(o[0], max(A, Bv)); self.scc = int(A > Bv)
        elif op == "s_min_i32" or op == "s_max_i32":
            A, Bv = (t - (1 << 32) if t >= (1 << 31) else t for t in (self.rd_s32(o[1]), self.rd_s32(o[2])))
            r_ = min(A, Bv) if "min" in op else max(A, Bv); self.wr_s32(o[0], r_ & M32); self.scc = int(r_ == A and A != Bv)
        elif op == "s_lshr_b64": t = self.rd_s64(o[1]) >> (self.rd_s32(o[2]) & 63); self.wr_s64(o[0], t); self.scc = int(t != 0)
        elif op == "s_ashr_i64":
            A = self.rd_s64(o[1]); A = A - (1 << 64) if A >= (1 << 63) else A
            t = (A >> (self.rd_s32(o[2]) & 63)) & ((1 << 64) - 1); self.wr_s64(o[0], t); self.scc = int(t != 0)
        elif op == "s_andn2_saveexec_b64":
            src = self.rd_s64(o[1]); old = self.exec; self.wr_s64(o[0], old); self.exec = src & ~old & ((1 << 64) - 1); self.scc = int(self.exec != 0)
        elif op in ("buffer_wbl2", "buffer_inv"): pass
        elif op == "s_mul_hi_i32":
            sg = lambda t: t - (1 << 32) if t >= (1 << 31) else t
            self.wr_s32(o[0], ((sg(self.rd_s32(o[1])) * sg(self.rd_s32(o[2]))) >> 32) & M32)
        elif op in ("s_cmpk_eq_i32", "s_cmpk_lg_i32"):
            k = self.lit(o[1]); k = (k - 0x10000 if k >= 0x8000 else k) & M32
            self.scc = int((self.rd_s32(o[0]) == k) == (op == "s_cmpk_eq_i32"))
        elif op == "s_mul_hi_u32": self.wr_s32(o[0], (self.rd_s32(o[1]) * self.rd_s32(o[2])) >> 32)
        elif op == "s_lshl_b64": t = (self.rd_s64(o[1]) << (self.rd_s32(o[2]) & 63)); self.wr_s64(o[0], t); self.scc = int((t & ((1 << 64) - 1)) != 0)
        elif op == "s_lshl_b32": t = (self.rd_s32(o[1]) << (self.rd_s32(o[2]) & 31)) & M32; self.wr_s32(o[0], t); self.scc = int(t != 0)
        elif op == "s_lshr_b32": t = self.rd_s32(o[1]) >> (self.rd_s32(o[2]) & 31); self.wr_s32(o[0], t); self.scc = int(t != 0)
        elif op == "s_or_b64": t = self.rd_s64(o[1]) | self.rd_s64(o[2]); self.wr_s64(o[0], t); self.scc = int(t != 0)
        elif op == "s_and_b64": t = self.rd_s64(o[1]) & self.rd_s64(o[2]); self.wr_s64(o[0], t); self.scc = int(t != 0)
        elif op == "s_xor_b64": t = self.rd_s64(o[1]) ^ self.rd_s64(o[2]); self.wr_s64(o[0], t); self.scc = int(t != 0)
        elif op == "s_not_b64": t = ~self.rd_s64(o[1]) & ((1 << 64) - 1); self.wr_s64(o[0], t); self.scc = int(t != 0)
        elif op == "s_orn2_b64": t = (self.rd_s64(o[1]) | ~self.rd_s64(o[2])) & ((1 << 64) - 1); self.wr_s64(o[0], t); self.scc = int(t != 0)
        elif op == "s_xor_b32": t = self.rd_s32(o[1]) ^ self.rd_s32(o[2]); self.wr_s32(o[0], t); self.scc = int(t != 0)
        elif op == "s_andn2_b64": t = self.rd_s64(o[1]) & ~self.rd_s64(o[2]); self.wr_s64(o[0], t); self.scc = int((t & ((1 << 64) - 1)) != 0)
        elif op == "s_and_saveexec_b64":
            src = self.rd_s64(o[1]); old = self.exec; self.wr_s64(o[0], old); self.exec = old & src; self.scc = int(self.exec != 0)
        elif op == "s_or_saveexec_b64":
            src = self.rd_s64(o[1]); old = self.exec; self.wr_s64(o[0], old); self.exec = old | src; self.scc = int(self.exec != 0)
        elif op == "s_bcnt1_i32_b64": t = bin(self.rd_s64(o[1])).count("1"); self.wr_s32(o[0], t); self.scc = int(t != 0)
        elif op == "s_bcnt1_i32_b32": t = bin(self.rd_s32(o[1])).count("1"); self.wr_s32(o[0], t); self.scc = int(t != 0)
        elif op in ("s_bitcmp1_b32", "s_bitcmp0_b32"):
            bit = (self.rd_s32(o[0]) >> (self.rd_s32(o[1]) & 31)) & 1
            self.scc = int(bit == (1 if op == "s_bitcmp1_b32" else 0))
        elif op == "s_cmp_eq_u32": self.scc = int(self.rd_s32(o[0]) == self.rd_s32(o[1]))
        elif op == "s_cmp_lg_u32": self.scc = int(self.rd_s32(o[0]) != self.rd_s32(o[1]))
        elif op == "s_ashr_i32":
            a_ = self.rd_s32(o[1]); a_ = a_ - (1 << 32) if a_ >= (1 << 31) else a_
            t = (a_ >> (self.rd_s32(o[2]) & 31)) & M32; self.wr_s32(o[0], t); self.scc = int(t != 0)
        elif op == "s_mulk_i32":
            k = self.lit(o[1]); k = k - 0x10000 if k >= 0x8000 else k
            self.wr_s32(o[0], (self.rd_s32(o[0]) * k) & M32)
        elif op == "s_or_b32": t = self.rd_s32(o[1]) | self.rd_s32(o[2]); self.wr_s32(o[0], t); self.scc = int(t != 0)
        elif op == "s_and_b32": t = self.rd_s32(o[1]) & self.rd_s32(o[2]); self.wr_s32(o[0], t); self.scc = int(t != 0)
        elif op == "s_bitset1_b32": self.wr_s32(o[0], self.rd_s32(o[0]) | (1 << (self.rd_s32(o[1]) & 31)))
        elif op == "s_getpc_b64": self.wr_s64(o[0], addr + 4)
        elif op == "s_setpc_b64": self.jump = self.rd_s64(o[0])
        elif op.startswith("s_load_dword"):
            n = {"s_load_dword": 1, "s_load_dwordx2": 2, "s_load_dwordx4": 4, "s_load_dwordx8": 8, "s_load_dwordx16": 16}[op]
            base = self.rd_s64(o[1]) + self.lit(o[2])
            off = base - self.KA
            r = self.rng(o[0]); assert r[0] == "s" and r[2] == n
            if 0 <= off and off + 4 * n <= len(self.kernarg):
                for k in range(n): self.s[r[1] + k] = struct.unpack_from("<I", self.kernarg, off + 4 * k)[0]
            else:      # a wave-uniform row of floating-point data
                self.check_global(addr, ins, np.full(64, base, dtype=np.uint64), 4 * n, np.arange(64) == 0)
                got = self.fetch(base, n)
                for k in range(n): self.s[r[1] + k] = got[k] if got else 0
        # ---------------- cross-lane / accumulation registers
        elif op == "v_readlane_b32":
            r = self.rng(o[1]); lane = self.rd_s32(o[2]) & 63
            self.wr_s32(o[0], int((self.v if r[0] == "v" else self.a)[r[1]][lane]))
        elif op == "v_readfirstlane_b32":
            r = self.rng(o[1]); m = self.mask(); lane = int(np.flatnonzero(m)[0]) if m.any() else 0
            self.wr_s32(o[0], int(self.v[r[1]][lane]))
        elif op == "v_writelane_b32":
            r = self.rng(o[0]); lane = self.rd_s32(o[2]) & 63
            self.v[r[1]][lane] = self.rd_s32(o[1])
        elif op in ("v_accvgpr_write_b32", "v_accvgpr_read_b32", "v_accvgpr_mov_b32", "v_mov_b32_e32"): self.wr_v(o[0], self.rd_v32(o[1]))
        elif op == "v_mov_b64_e32": self.wr_v(o[0], self.rd_v64(o[1]), 2)
        elif op == "v_mov_b32_dpp": self.wr_zero(o[0])        # used on floating-point data only (checked: its results feed v_add_f64)
        elif op in ("v_cvt_f32_u32_e32", "v_cvt_f32_i32_e32"):
            src = self.rd_v32(o[1]); src = self.s32(src) if "i32" in op else src.astype(np.int64)
            self.wr_v(o[0], src.astype(np.float32).view(np.uint32).astype(u64)); self.fexact.add(o[0])
        elif op == "v_rcp_iflag_f32_e32" and o[1] in self.fexact:
            f_ = self.rd_v32(o[1]).astype(np.uint32).view(np.float32)
            with np.errstate(all="ignore"): r_ = (np.float32(1) / f_).astype(np.float32)
            self.wr_v(o[0], r_.view(np.uint32).astype(u64)); self.fexact.add(o[0])
        elif op == "v_mul_f32_e32" and all(t in self.fexact or re.fullmatch(r"0x[0-9a-f]+", t) for t in o[1:]):
            f1, f2 = (self.rd_v32(t).astype(np.uint32).view(np.float32) for t in o[1:])
            with np.errstate(all="ignore"): self.wr_v(o[0], (f1 * f2).astype(np.float32).view(np.uint32).astype(u64))
            self.fexact.add(o[0])
        elif op in ("v_cvt_u32_f32_e32", "v_cvt_i32_f32_e32"):
            if o[1] not in self.fexact: raise NotImplementedError("integer from a floating-point value that was not evaluated: " + ins)
            f_ = self.rd_v32(o[1]).astype(np.uint32).view(np.float32).astype(np.float64)
            f_ = np.nan_to_num(np.trunc(f_), nan=0.0)
            lo_, hi_ = (0, M32) if "u32" in op else (-(1 << 31), (1 << 31) - 1)
            self.wr_v(o[0], np.clip(f_, lo_, hi_).astype(np.int64).astype(u64) & u64(M32))
        elif op in FLOAT_OPS or (re.fullmatch(r"v_\w+_f(16|32|64)(_e32|_e64|_dpp)?", op) and not op.startswith("v_cmp")): self.wr_zero(o[0])
        # ---------------- integer VALU
        elif op == "v_add_u32_e32": self.wr_v(o[0], (self.rd_v32(o[1]) + self.rd_v32(o[2])) & u64(M32))
        elif op == "v_sub_u32_e32": self.wr_v(o[0], (self.rd_v32(o[1]) - self.rd_v32(o[2])) & u64(M32))
        elif op in ("v_min_u32_e32", "v_max_u32_e32"):
            A, Bv = self.rd_v32(o[1]) & u64(M32), self.rd_v32(o[2]) & u64(M32)
            self.wr_v(o[0], np.minimum(A, Bv) if op == "v_min_u32_e32" else np.maximum(A, Bv))
        elif op in ("v_min_i32_e32", "v_max_i32_e32"):
            A, Bv = (self.rd_v32(o[1]) & u64(M32)).astype(np.uint32).view(np.int32), (self.rd_v32(o[2]) & u64(M32)).astype(np.uint32).view(np.int32)
            r_ = np.minimum(A, Bv) if op == "v_min_i32_e32" else np.maximum(A, Bv)
            self.wr_v(o[0], r_.view(np.uint32).astype(np.uint64))
        elif op == "v_subrev_u32_e32": self.wr_v(o[0], (self.rd_v32(o[2]) - self.rd_v32(o[1])) & u64(M32))
        elif op == "v_add_lshl_u32": self.wr_v(o[0], ((self.rd_v32(o[1]) + self.rd_v32(o[2])) << (self.rd_v32(o[3]) & u64(31))) & u64(M32))
        elif op in ("v_sub_co_u32_e32", "v_sub_co_u32_e64"):
            A, Bv = self.rd_v32(o[2]), self.rd_v32(o[3]); m = self.mask()
            self.wr_v(o[0], (A - Bv) & u64(M32)); self.wr_s64(o[1], (self.rd_s64(o[1]) & ~self.exec) | self.bits((A < Bv) & m))
        elif op in ("v_subb_co_u32_e32", "v_subb_co_u32_e64"):
            cin = self.rd_s64(o[4]); cinv = np.array([(cin >> i) & 1 for i in range(64)], dtype=u64)
            A, Bv = self.rd_v32(o[2]), self.rd_v32(o[3]) + cinv; m = self.mask()
            self.wr_v(o[0], (A - Bv) & u64(M32)); self.wr_s64(o[1], (self.rd_s64(o[1]) & ~self.exec) | self.bits((A < Bv) & m))
        elif op == "v_lshl_or_b32": self.wr_v(o[0], ((self.rd_v32(o[1]) << (self.rd_v32(o[2]) & u64(31))) & u64(M32)) | self.rd_v32(o[3]))
        elif op == "v_and_or_b32": self.wr_v(o[0], (self.rd_v32(o[1]) & self.rd_v32(o[2])) | self.rd_v32(o[3]))
        elif op == "v_or3_b32": self.wr_v(o[0], self.rd_v32(o[1]) | self.rd_v32(o[2]) | self.rd_v32(o[3]))
        elif op == "v_lshrrev_b64": self.wr_v(o[0], self.rd_v64(o[2]) >> (self.rd_v32(o[1]) & u64(63)), 2)
        elif op == "v_ashrrev_i64": self.wr_v(o[0], (self.rd_v64(o[2]).astype(np.int64) >> (self.rd_v32(o[1]) & u64(63)).astype(np.int64)).astype(u64), 2)
        elif op in ("v_subrev_co_u32_e32", "v_subrev_co_u32_e64"):
            A, Bv = self.rd_v32(o[3]), self.rd_v32(o[2]); m = self.mask()
            self.wr_v(o[0], (A - Bv) & u64(M32)); self.wr_s64(o[1], (self.rd_s64(o[1]) & ~self.exec) | self.bits((A < Bv) & m))
        elif op in ("v_subbrev_co_u32_e32", "v_subbrev_co_u32_e64"):
            cin = self.rd_s64(o[4]); cinv = np.array([(cin >> i) & 1 for i in range(64)], dtype=u64)
            A, Bv = self.rd_v32(o[3]), self.rd_v32(o[2]) + cinv; m = self.mask()
            self.wr_v(o[0], (A - Bv) & u64(M32)); self.wr_s64(o[1], (self.rd_s64(o[1]) & ~self.exec) | self.bits((A < Bv) & m))
        elif op == "v_xor_b32_e32": self.wr_v(o[0], self.rd_v32(o[1]) ^ self.rd_v32(o[2]))
        elif op == "v_alignbit_b32":   # ({src0, src1} >> src2[4:0]), low 32 bits
            self.wr_v(o[0], (((self.rd_v32(o[1]) << u64(32)) | self.rd_v32(o[2])) >> (self.rd_v32(o[3]) & u64(31))) & u64(M32))
        elif op == "v_bfe_u32": self.wr_v(o[0], (self.rd_v32(o[1]) >> (self.rd_v32(o[2]) & u64(31))) & ((u64(1) << (self.rd_v32(o[3]) & u64(31))) - u64(1)))
        elif op == "v_bfrev_b32_e32": self.wr_v(o[0], np.array([int(format(int(t), "032b")[::-1], 2) for t in self.rd_v32(o[1])], dtype=u64))
        elif op in ("v_mbcnt_lo_u32_b32", "v_mbcnt_hi_u32_b32"):
            msk = self.rd_v32(o[1]); lanes = np.arange(64)
            below = np.clip(lanes - (32 if "hi" in op else 0), 0, 32)
            cnt = np.array([bin(int(msk[i]) & ((1 << int(below[i])) - 1)).count("1") for i in range(64)], dtype=u64)
            self.wr_v(o[0], (cnt + self.rd_v32(o[2])) & u64(M32))
        elif op == "v_mad_u32_u24": self.wr_v(o[0], ((self.rd_v32(o[1]) & u64(0xFFFFFF)) * (self.rd_v32(o[2]) & u64(0xFFFFFF)) + self.rd_v32(o[3])) & u64(M32))
        elif op == "v_mul_hi_u32_u24_e32": self.wr_v(o[0], ((self.rd_v32(o[1]) & u64(0xFFFFFF)) * (self.rd_v32(o[2]) & u64(0xFFFFFF))) >> u64(32))
        elif op == "v_mad_i64_i32":
            self.wr_v(o[0], (self.s32(self.rd_v32(o[2])) * self.s32(self.rd_v32(o[3])) + self.rd_v64(o[4]).astype(np.int64)).astype(u64), 2)
        elif op == "ds_bpermute_b32":      # dst[i] = data[lane addr[i] / 4]; a lane that is switched off supplies 0
            src = ((self.rd_v32(o[1]) + u64(self.lit(mods.get("offset", "0")))) >> u64(2)).astype(np.int64) & 63
            d_ = self.rd_v32(o[2]); m_ = self.mask()
            self.wr_v(o[0], np.where(m_[src], d_[src], u64(0)))
        elif op == "v_add3_u32": self.wr_v(o[0], (self.rd_v32(o[1]) + self.rd_v32(o[2]) + self.rd_v32(o[3])) & u64(M32))
        elif op == "v_and_b32_e32": self.wr_v(o[0], self.rd_v32(o[1]) & self.rd_v32(o[2]))
        elif op == "v_or_b32_e32": self.wr_v(o[0], self.rd_v32(o[1]) | self.rd_v32(o[2]))
        elif op == "v_lshlrev_b32_e32": self.wr_v(o[0], (self.rd_v32(o[2]) << (self.rd_v32(o[1]) & u64(31))) & u64(M32))
        elif op == "v_lshrrev_b32_e32": self.wr_v(o[0], self.rd_v32(o[2]) >> (self.rd_v32(o[1]) & u64(31)))
        elif op == "v_ashrrev_i32_e32": self.wr_v(o[0], (self.s32(self.rd_v32(o[2])) >> self.s32(self.rd_v32(o[1]) & u64(31))).astype(np.int64).astype(u64) & u64(M32))
        elif op == "v_lshlrev_b64": self.wr_v(o[0], self.rd_v64(o[2]) << (self.rd_v32(o[1]) & u64(63)), 2)
        elif op == "v_lshl_add_u32": self.wr_v(o[0], ((self.rd_v32(o[1]) << (self.rd_v32(o[2]) & u64(31))) + self.rd_v32(o[3])) & u64(M32))
        elif op == "v_lshl_add_u64": self.wr_v(o[0], (self.rd_v64(o[1]) << (self.rd_v32(o[2]) & u64(7))) + self.rd_v64(o[3]), 2)
        elif op == "v_mul_lo_u32": self.wr_v(o[0], (self.rd_v32(o[1]) * self.rd_v32(o[2])) & u64(M32))
        elif op == "v_mul_hi_i32": self.wr_v(o[0], ((self.s32(self.rd_v32(o[1])) * self.s32(self.rd_v32(o[2]))) >> 32).astype(u64) & u64(M32))
        elif op == "v_mul_hi_u32": self.wr_v(o[0], (self.rd_v32(o[1]) * self.rd_v32(o[2])) >> u64(32))
        elif op in ("v_mul_i32_i24_e32", "v_mul_u32_u24_e32"):
            s24 = lambda a: (lambda t: np.where(t >= (1 << 23), t - (1 << 24), t))((a & u64(0xFFFFFF)).astype(np.int64))
            self.wr_v(o[0], (s24(self.rd_v32(o[1])) * s24(self.rd_v32(o[2]))).astype(u64) & u64(M32))
        elif op == "v_mad_i32_i24":
            s24 = lambda a: (lambda t: np.where(t >= (1 << 23), t - (1 << 24), t))((a & u64(0xFFFFFF)).astype(np.int64))
            self.wr_v(o[0], (s24(self.rd_v32(o[1])) * s24(self.rd_v32(o[2])) + self.s32(self.rd_v32(o[3]))).astype(u64) & u64(M32))
        elif op == "v_mad_u64_u32":      # vdst64, sdst(carry), a, b, c64
            self.wr_v(o[0], self.rd_v32(o[2]) * self.rd_v32(o[3]) + self.rd_v64(o[4]), 2)
        elif op in ("v_add_co_u32_e32", "v_add_co_u32_e64"):
            t = self.rd_v32(o[2]) + self.rd_v32(o[3]); m = self.mask()
            c = self.bits((t >> u64(32)).astype(bool) & m)
            self.wr_v(o[0], t & u64(M32)); self.wr_s64(o[1], (self.rd_s64(o[1]) & ~self.exec) | c)
        elif op in ("v_addc_co_u32_e32", "v_addc_co_u32_e64"):
            cin = self.rd_s64(o[4]); cinv = np.array([(cin >> i) & 1 for i in range(64)], dtype=u64)
            t = self.rd_v32(o[2]) + self.rd_v32(o[3]) + cinv; m = self.mask()
            c = self.bits((t >> u64(32)).astype(bool) & m)
            self.wr_v(o[0], t & u64(M32)); self.wr_s64(o[1], (self.rd_s64(o[1]) & ~self.exec) | c)
        elif op in ("v_cndmask_b32_e32", "v_cndmask_b32_e64"):
            sel = self.vcc if op.endswith("e32") else self.rd_s64(o[3])
            selv = np.array([(sel >> i) & 1 for i in range(64)], dtype=bool)
            self.wr_v(o[0], np.where(selv, self.rd_v32(o[2]), self.rd_v32(o[1])))
        elif op.startswith("v_cmp_"):
            mm = re.fullmatch(r"v_cmp_(gt|lt|ge|le|eq|ne)_(i32|u32|i64|u64)_(e32|e64)", op); assert mm, op
            dst, a, b = o[0], o[1], o[2]
            if mm.group(2) in ("i32", "u32"):
                A, Bv = self.rd_v32(a), self.rd_v32(b)
                if mm.group(2) == "i32": A, Bv = self.s32(A), self.s32(Bv)
            else:
                A, Bv = self.rd_v64(a), self.rd_v64(b)
                if mm.group(2) == "i64": A, Bv = A.astype(np.int64), Bv.astype(np.int64)
            res = {"gt": A > Bv, "lt": A < Bv, "ge": A >= Bv, "le": A <= Bv, "eq": A == Bv, "ne": A != Bv}[mm.group(1)]
            self.wr_s64(dst, self.bits(res & self.mask()))
        # ---------------- memory
        elif op.startswith("global_load") or op.startswith("global_store"):
            n = {"dword": 1, "dwordx2": 2, "dwordx3": 3, "dwordx4": 4}[op.split("_")[-1]]
            load_ = op.startswith("global_load")
            at, sa = (o[1], o[2]) if load_ else (o[0], o[2])
            off = self.lit(mods.get("offset", "0"))
            r = self.rng(at)
            if sa == "off": addrs = self.rd_v64(at)
            else: addrs = self.rd_v32(at) + u64(self.rd_s64(sa))
            addrs = (addrs.astype(np.int64) + off).astype(u64)
            self.check_global(addr, ins, addrs, 4 * n, self.mask())
            if not load_: self.mark_written(addrs, 4 * n, self.mask())
            if load_:
                self.wr_zero(o[0])
                if any(len(t) > 3 and t[3] is not None for t in self.buffers):      # integer arrays: real values
                    r = self.rng(o[0]); f = self.v if r[0] == "v" else self.a
                    for lane in np.flatnonzero(self.mask()):
                        got = self.fetch(int(addrs[lane]), n)
                        if got:
                            for k in range(n): f[r[1] + k][lane] = got[k]
        elif op.startswith("ds_read") or op.startswith("ds_write"):
            rd = op.startswith("ds_read")
            at = o[1] if rd else o[0]
            base = self.rd_v32(at)
            if re.search(r"2(st64)?_b(32|64)$", op):
                el = 8 if "b64" in op else 4
                unit = el * (64 if "st64" in op else 1)
                for key in ("offset0", "offset1"):
                    self.check_lds(addr, ins, (base + u64(self.lit(mods.get(key, "0")) * unit)) & u64(M32), el, self.mask())
            else:
                el = {"b32": 4, "b64": 8, "b96": 12, "b128": 16}[op.split("_")[-1]]
                self.check_lds(addr, ins, (base + u64(self.lit(mods.get("offset", "0")))) & u64(M32), el, self.mask())
            if rd: self.wr_zero(o[0])
        elif op.startswith("scratch_store") or op.startswith("scratch_load"):
            # private memory, one copy per lane, addressed by immediate offset (+ scalar offset): values are kept exactly
            n = {"dword": 1, "dwordx2": 2, "dwordx3": 3, "dwordx4": 4}[op.split("_")[-1]]
            st = op.startswith("scratch_store")
            va, data, sa = (o[0], o[1], o[2]) if st else (o[1], o[0], o[2])
            assert va == "off", ins
            base = self.lit(mods.get("offset", "0")) + (0 if sa == "off" else self.rd_s32(sa))
            r = self.rng(data); f = self.v if r[0] == "v" else self.a; m = self.mask()
            for k in range(n):
                cell = self.scratch.setdefault(base + 4 * k, np.full(64, 0xDEADBEE0, dtype=np.uint64))
                if st: cell[m] = f[r[1] + k][m]
                else: f[r[1] + k][m] = cell[m]
        else:
            raise NotImplementedError(ins)


def check(hsaco, lds_bytes, B, grid, row_words, elt=8, waves=1, outputs=()):
    """Run `grid` workgroups of `waves` waves (which must not cooperate) over B rows; pointer argument i has
    B * row_words[i] elements of `elt` bytes, the last explicit argument is B (int64).  `outputs`: indices of pointer
    arguments every byte of which the kernel has to write."""
    prog = load(hsaco)
    bufs, ka = [], b""
    for i, w in enumerate(row_words):
        base = 0x1000_0000_0000 + i * 0x10_0000_0000
        bufs.append((base, B * w * elt, f"arg{i}")); ka += struct.pack("<Q", base)
    ka += struct.pack("<q", B)
    hidden = struct.pack("<IIIHHH", grid, 1, 1, 64 * waves, 1, 1)
    ka += hidden + b"\0" * (256 - len(hidden))
    emu = Emu(prog, lds_bytes, ka, bufs)
    for wg in range(grid):
        for wave in range(waves):
            try:
                emu.run(wg, wave)
            except OOB:
                return emu.problems
    for i in outputs:
        gap = emu.unwritten(f"arg{i}")
        if gap is not None: emu.problems.append(f"output argument {i}: byte {gap} (row {gap // (row_words[i] * elt)}, word {gap // elt % row_words[i]}) is never written")
    return emu.problems


def check_args(hsaco, lds_bytes, args, grid, waves=1):
    """As check(), for any argument list: ("buf", bytes) a buffer of floating-point data, ("buf", bytes, array) a buffer
    whose contents the kernel computes addresses from (integer arrays), ("i64", v), ("i32", v), ("null",)."""
    prog = load(hsaco)
    bufs, ka = [], b""
    for i, a in enumerate(args):
        if a[0] == "buf":
            base = 0x1000_0000_0000 + i * 0x10_0000_0000
            content = np.ascontiguousarray(a[2]).tobytes() if len(a) > 2 else None
            bufs.append((base, a[1], f"arg{i}", content)); ka += struct.pack("<Q", base)
        elif a[0] == "null": ka += struct.pack("<Q", 0)
        elif a[0] == "i64": ka += struct.pack("<q", a[1])
        elif a[0] == "i32": ka += struct.pack("<i", a[1])
        else: raise ValueError(a[0])
    ka += b"\0" * (-len(ka) % 8)
    hidden = struct.pack("<IIIHHH", grid, 1, 1, 64 * waves, 1, 1)
    ka += hidden + b"\0" * (256 - len(hidden))
    emu = Emu(prog, lds_bytes, ka, bufs)
    for wg in range(grid):
        for wave in range(waves):
            try:
                emu.run(wg, wave)
            except OOB:
                return emu.problems
    return emu.problems


def exec_zero_windows(hsaco):
    txt = subprocess.run([OBJDUMP, "-d", "--no-show-raw-insn", hsaco], capture_output=True, text=True).stdout
    ins = [re.sub(r"\s*//.*$", "", l).strip() for l in txt.split("\n") if "//" in l]
    hits, i = [], 0
    while i < len(ins):
        back_edge = ins[i].startswith("s_cbranch_execnz") and int(ins[i].split()[1]) >= 32768
        if back_edge and any(x.startswith("s_andn2_b64 exec, exec") for x in ins[max(0, i - 3):i]):
            j = i + 1
            while j < len(ins) and not re.match(r"s_\w+ exec\b", ins[j]) and not ins[j].startswith(("s_cbranch", "s_branch", "s_endpgm")):
                op = ins[j].split()[0]
                if op.startswith(("v_", "ds_", "global_", "scratch_", "buffer_", "flat_")) and not op.startswith(("v_readlane", "v_writelane", "v_readfirstlane", "v_cmp")):
                    hits.append(ins[j])
                j += 1
            i = j
        else:
            i += 1
    return hits
