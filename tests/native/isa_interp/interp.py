"""An interpreter for the machine code of this repository's decode kernels, as text (what
`hipcc -S` writes for gfx950): runs the workgroups of a recorded launch instruction by instruction,
64 lanes at a time, three waves of a workgroup in turn from barrier to barrier, and

  * checks every global load, store and atomic against the launch's buffers (an access outside
    all of them ends the run with the instruction, lane and address),
  * checks LDS accesses for alignment and counts those outside the workgroup's allocation,
  * compares every buffer afterwards with what the host build of the same source left.

It exists because a kernel can be right as source and wrong as compiled: the host build
(tests/native/kernel_cpu) runs the kernels' source under the sanitizers, this runs what the GPU
would run.  Waves run one after the other between barriers, which is the interleaving least
kind to a missing synchronisation.  Only the instructions the decode kernels use are known; an
unknown one stops the run by name.  Registers start poisoned, LDS starts as garbage.

usage: interp.py <kernel.s> <launch.bin> [after.bin] [--wg=first:last] [--hist=file]
  kernel.s    one kernel's text, from its label to .end_amdhsa_kernel
  launch.bin  a launch recorded by tests/native/kernel_cpu (L3CPU_RECORD)
  after.bin   the buffers after the host build's run
  --hist      writes, per instruction, how many times a wave executed it
Test infrastructure (tests/test_kernel_machine_code.py)."""
import re
import struct
import sys

import numpy as np

U32 = np.uint32
U64 = np.uint64
LANES = 64
VCC, EXEC = 106, 126
np.seterr(over="ignore")


class Fault(Exception):
    pass


def parse_int(t):
    t = t.strip()
    if t.startswith("0x") or t.startswith("-0x"):
        return int(t, 16)
    return int(t)


class Memory:
    def __init__(self):
        self.regions = []   # (base, bytearray, name)

    def add(self, base, data, name):
        self.regions.append((base, bytearray(data), name))

    def find(self, addr, n):
        for base, data, name in self.regions:
            if base <= addr and addr + n <= base + len(data):
                return data, addr - base
        return None, None

    def load(self, addr, n, what):
        data, off = self.find(addr, n)
        if data is None:
            raise Fault("%s: load of %d bytes at 0x%x outside every buffer" % (what, n, addr))
        return bytes(data[off:off + n])

    def store(self, addr, b, what):
        data, off = self.find(addr, len(b))
        if data is None:
            raise Fault("%s: store of %d bytes at 0x%x outside every buffer" % (what, len(b), addr))
        data[off:off + len(b)] = b


class Inst:
    __slots__ = ("op", "args", "mods", "line", "text")


def parse_kernel(path):
    insts, labels = [], {}
    lds_size = 0
    for ln, raw in enumerate(open(path), 1):
        line = raw.split(";")[0].strip()
        m = re.match(r"\.amdhsa_group_segment_fixed_size (\d+)", line)
        if m:
            lds_size = int(m.group(1))
        if not line or line.startswith("."):
            if re.match(r"^\.LBB\S+:$", line):
                labels[line[:-1]] = len(insts)
            continue
        if line.endswith(":"):
            labels[line[:-1]] = len(insts)
            continue
        parts = line.split(None, 1)
        ins = Inst()
        ins.op = parts[0]
        rest = parts[1] if len(parts) > 1 else ""
        ins.line, ins.text = ln, line
        # split operands on commas outside brackets
        ops, depth, cur = [], 0, ""
        for ch in rest:
            if ch == "[":
                depth += 1
            if ch == "]":
                depth -= 1
            if ch == "," and depth == 0:
                ops.append(cur.strip())
                cur = ""
            else:
                cur += ch
        if cur.strip():
            ops.append(cur.strip())
        mods = {}
        if ops:
            # modifiers trail the last operand, separated by spaces
            last = ops[-1]
            toks = re.findall(r"[A-Za-z_0-9]+:\[[^\]]*\]|[A-Za-z_0-9]+:[^\s]+|\S+", last)
            keep = []
            for t in toks:
                if ":" in t and not re.match(r"^[vs]\[", t):
                    k, v = t.split(":", 1)
                    mods[k] = v
                elif t in ("nt", "clamp", "glc", "slc", "off") and keep:
                    mods[t] = True
                else:
                    keep.append(t)
            ops[-1] = " ".join(keep)
            if ops[-1] == "":
                ops.pop()
        # 'off' as an address operand
        ins.args = ops
        ins.mods = mods
        insts.append(ins)
    return insts, labels, lds_size


class Wave:
    def __init__(self, wid):
        self.s = np.zeros(128, dtype=U32)
        self.v = np.zeros((256, LANES), dtype=U32)
        self.scc = 0
        self.pc = 0
        self.done = False
        self.at_barrier = False
        self.id = wid

    def exec_mask(self):
        e = int(self.s[EXEC]) | (int(self.s[EXEC + 1]) << 32)
        return np.array([(e >> i) & 1 for i in range(LANES)], dtype=bool)


class Emu:
    def __init__(self, insts, labels, lds_size, mem):
        self.insts, self.labels, self.mem = insts, labels, mem
        self.lds = bytearray(lds_size)
        self.lds_oob = 0
        self.count = 0
        self.executed = {}      # instruction index -> times a wave executed it

    # ---- operand access -------------------------------------------------
    def sreg_index(self, t):
        if t == "vcc" or t == "vcc_lo":
            return VCC
        if t == "vcc_hi":
            return VCC + 1
        if t == "exec" or t == "exec_lo":
            return EXEC
        if t == "exec_hi":
            return EXEC + 1
        m = re.match(r"^s(\d+)$", t)
        if m:
            return int(m.group(1))
        m = re.match(r"^s\[(\d+):(\d+)\]$", t)
        if m:
            return int(m.group(1))
        return None

    def rs(self, w, t):
        """scalar 32-bit source"""
        i = self.sreg_index(t)
        if i is not None:
            return int(w.s[i])
        if t == "scc":
            return w.scc
        return self.literal(t)

    def literal(self, t):
        if re.match(r"^-?\d+\.\d+$", t):
            return int(np.array([float(t)], dtype=np.float32).view(U32)[0])
        return parse_int(t) & 0xFFFFFFFF

    def rs64(self, w, t):
        i = self.sreg_index(t)
        if i is not None:
            return int(w.s[i]) | (int(w.s[i + 1]) << 32)
        v = parse_int(t)
        return v & 0xFFFFFFFFFFFFFFFF

    def ws(self, w, t, val):
        w.s[self.sreg_index(t)] = U32(val & 0xFFFFFFFF)

    def ws64(self, w, t, val):
        i = self.sreg_index(t)
        w.s[i] = U32(val & 0xFFFFFFFF)
        w.s[i + 1] = U32((val >> 32) & 0xFFFFFFFF)

    def vreg(self, t):
        m = re.match(r"^v(\d+)$", t)
        if m:
            return int(m.group(1)), 1
        m = re.match(r"^v\[(\d+):(\d+)\]$", t)
        if m:
            return int(m.group(1)), int(m.group(2)) - int(m.group(1)) + 1
        return None, 0

    def rv(self, w, t):
        """vector 32-bit source (scalars and literals are broadcast)"""
        r, n = self.vreg(t)
        if r is not None:
            return w.v[r].copy()
        return np.full(LANES, self.rs(w, t), dtype=U32)

    def rv64(self, w, t):
        r, n = self.vreg(t)
        if r is not None:
            return w.v[r].astype(U64) | (w.v[r + 1].astype(U64) << U64(32))
        return np.full(LANES, self.rs64(w, t), dtype=U64)

    def wv(self, w, t, val, mask=None):
        r, n = self.vreg(t)
        m = w.exec_mask() if mask is None else mask
        w.v[r][m] = val.astype(U32)[m]

    def wv64(self, w, t, val):
        r, n = self.vreg(t)
        m = w.exec_mask()
        w.v[r][m] = (val & U64(0xFFFFFFFF)).astype(U32)[m]
        w.v[r + 1][m] = (val >> U64(32)).astype(U32)[m]

    def mask_to_int(self, b, w):
        m = w.exec_mask() & b
        return sum(1 << i for i in range(LANES) if m[i])

    def int_to_mask(self, x):
        return np.array([(x >> i) & 1 for i in range(LANES)], dtype=bool)

    # ---- LDS ---------------------------------------------------------------
    def lds_read(self, addr, n):
        if addr < 0 or addr + n > len(self.lds):
            self.lds_oob += 1
            return bytes(n)
        return bytes(self.lds[addr:addr + n])

    def lds_write(self, addr, b):
        if addr < 0 or addr + len(b) > len(self.lds):
            self.lds_oob += 1
            return
        self.lds[addr:addr + len(b)] = b

    # ---- one instruction ------------------------------------------------------
    def step(self, w):
        ins = self.insts[w.pc]
        w.pc += 1
        self.count += 1
        self.executed[w.pc - 1] = self.executed.get(w.pc - 1, 0) + 1
        op, a, mods = ins.op, ins.args, ins.mods
        base = op
        for suf in ("_e32", "_e64", "_dpp", "_sdwa"):
            if base.endswith(suf):
                base = base[:-len(suf)]
        f = getattr(self, "i_" + base, None)
        if f is None:
            raise NotImplementedError("%s (line %d: %s)" % (op, ins.line, ins.text))
        f(w, ins, a, mods)

    # scalar ----------------------------------------------------------------
    def i_s_waitcnt(self, w, ins, a, m): pass
    def i_s_nop(self, w, ins, a, m): pass
    def i_s_setprio(self, w, ins, a, m): pass
    def i_s_endpgm(self, w, ins, a, m): w.done = True
    def i_s_barrier(self, w, ins, a, m): w.at_barrier = True

    def i_s_mov_b32(self, w, ins, a, m): self.ws(w, a[0], self.rs(w, a[1]))
    def i_s_mov_b64(self, w, ins, a, m): self.ws64(w, a[0], self.rs64(w, a[1]) if self.sreg_index(a[1]) is not None else (parse_int(a[1]) & 0xFFFFFFFFFFFFFFFF))
    def i_s_movk_i32(self, w, ins, a, m): self.ws(w, a[0], parse_int(a[1]) & 0xFFFFFFFF if parse_int(a[1]) >= 0 else parse_int(a[1]) & 0xFFFFFFFF)
    def i_s_addk_i32(self, w, ins, a, m):
        k = parse_int(a[1]) & 0xFFFF
        k = k - 0x10000 if k & 0x8000 else k
        x = self.rs(w, a[0])
        r = (x + k) & 0xFFFFFFFF
        sx, sk, sr = x >> 31, int(k < 0), r >> 31
        w.scc = int(sx == sk and sr != sx)
        self.ws(w, a[0], r)

    def i_s_mulk_i32(self, w, ins, a, m): self.ws(w, a[0], (self.rs(w, a[0]) * parse_int(a[1])) & 0xFFFFFFFF)

    def i_s_add_i32(self, w, ins, a, m):
        x, y = self.rs(w, a[1]), self.rs(w, a[2])
        r = (x + y) & 0xFFFFFFFF
        sx, sy, sr = x >> 31, y >> 31, r >> 31
        w.scc = int(sx == sy and sr != sx)
        self.ws(w, a[0], r)

    def i_s_sub_i32(self, w, ins, a, m):
        x, y = self.rs(w, a[1]), self.rs(w, a[2])
        r = (x - y) & 0xFFFFFFFF
        sx, sy, sr = x >> 31, y >> 31, r >> 31
        w.scc = int(sx != sy and sr != sx)
        self.ws(w, a[0], r)

    def i_s_add_u32(self, w, ins, a, m):
        r = self.rs(w, a[1]) + self.rs(w, a[2])
        w.scc = int(r > 0xFFFFFFFF)
        self.ws(w, a[0], r)

    def i_s_addc_u32(self, w, ins, a, m):
        r = self.rs(w, a[1]) + self.rs(w, a[2]) + w.scc
        w.scc = int(r > 0xFFFFFFFF)
        self.ws(w, a[0], r)

    def i_s_mul_i32(self, w, ins, a, m): self.ws(w, a[0], (self.rs(w, a[1]) * self.rs(w, a[2])) & 0xFFFFFFFF)
    def i_s_mul_hi_u32(self, w, ins, a, m): self.ws(w, a[0], (self.rs(w, a[1]) * self.rs(w, a[2])) >> 32)

    def i_s_min_u32(self, w, ins, a, m):
        x, y = self.rs(w, a[1]), self.rs(w, a[2])
        w.scc = int(x < y)
        self.ws(w, a[0], min(x, y))

    def _slogic(self, w, a, fn, bits):
        if bits == 64:
            r = fn(self.rs64(w, a[1]), self.rs64(w, a[2])) & 0xFFFFFFFFFFFFFFFF
            self.ws64(w, a[0], r)
        else:
            r = fn(self.rs(w, a[1]), self.rs(w, a[2])) & 0xFFFFFFFF
            self.ws(w, a[0], r)
        w.scc = int(r != 0)

    def i_s_and_b64(self, w, ins, a, m): self._slogic(w, a, lambda x, y: x & y, 64)
    def i_s_or_b64(self, w, ins, a, m): self._slogic(w, a, lambda x, y: x | y, 64)
    def i_s_xor_b64(self, w, ins, a, m): self._slogic(w, a, lambda x, y: x ^ y, 64)
    def i_s_andn2_b64(self, w, ins, a, m): self._slogic(w, a, lambda x, y: x & ~y, 64)
    def i_s_orn2_b64(self, w, ins, a, m): self._slogic(w, a, lambda x, y: x | ~y, 64)
    def i_s_and_b32(self, w, ins, a, m): self._slogic(w, a, lambda x, y: x & y, 32)
    def i_s_or_b32(self, w, ins, a, m): self._slogic(w, a, lambda x, y: x | y, 32)
    def i_s_lshr_b32(self, w, ins, a, m): self._slogic(w, a, lambda x, y: x >> (y & 31), 32)
    def i_s_lshl_b32(self, w, ins, a, m): self._slogic(w, a, lambda x, y: x << (y & 31), 32)

    def i_s_ashr_i32(self, w, ins, a, m):
        x = self.rs(w, a[1])
        x = x - (1 << 32) if x >> 31 else x
        r = (x >> (self.rs(w, a[2]) & 31)) & 0xFFFFFFFF
        self.ws(w, a[0], r)
        w.scc = int(r != 0)

    def i_s_sub_u32(self, w, ins, a, m):
        x, y = self.rs(w, a[1]), self.rs(w, a[2])
        w.scc = int(y > x)
        self.ws(w, a[0], (x - y) & 0xFFFFFFFF)

    def i_s_subb_u32(self, w, ins, a, m):
        x, y = self.rs(w, a[1]), self.rs(w, a[2]) + w.scc
        w.scc = int(y > x)
        self.ws(w, a[0], (x - y) & 0xFFFFFFFF)

    def i_s_lshr_b64(self, w, ins, a, m):
        r = self.rs64(w, a[1]) >> (self.rs(w, a[2]) & 63)
        self.ws64(w, a[0], r)
        w.scc = int(r != 0)

    def i_s_xor_b32(self, w, ins, a, m): self._slogic(w, a, lambda x, y: x ^ y, 32)
    def i_s_andn2_b32(self, w, ins, a, m): self._slogic(w, a, lambda x, y: x & ~y, 32)
    def i_s_not_b64(self, w, ins, a, m):
        r = ~self.rs64(w, a[1]) & 0xFFFFFFFFFFFFFFFF
        self.ws64(w, a[0], r)
        w.scc = int(r != 0)
    def i_s_max_u32(self, w, ins, a, m):
        x, y = self.rs(w, a[1]), self.rs(w, a[2])
        w.scc = int(x > y)
        self.ws(w, a[0], max(x, y))
    def i_s_max_i32(self, w, ins, a, m):
        x, y = self.rs(w, a[1]), self.rs(w, a[2])
        sx = x - (1 << 32) if x >> 31 else x
        sy = y - (1 << 32) if y >> 31 else y
        w.scc = int(sx > sy)
        self.ws(w, a[0], x if sx > sy else y)
    def i_s_min_i32(self, w, ins, a, m):
        x, y = self.rs(w, a[1]), self.rs(w, a[2])
        sx = x - (1 << 32) if x >> 31 else x
        sy = y - (1 << 32) if y >> 31 else y
        w.scc = int(sx < sy)
        self.ws(w, a[0], x if sx < sy else y)

    def i_s_brev_b32(self, w, ins, a, m):
        self.ws(w, a[0], int("{:032b}".format(self.rs(w, a[1]))[::-1], 2))

    def i_s_bcnt1_i32_b64(self, w, ins, a, m):
        r = bin(self.rs64(w, a[1])).count("1")
        self.ws(w, a[0], r)
        w.scc = int(r != 0)

    def i_s_bfe_u32(self, w, ins, a, m):
        x, y = self.rs(w, a[1]), self.rs(w, a[2])
        width = (y >> 16) & 0x7F
        r = (x >> (y & 31)) & ((1 << width) - 1) & 0xFFFFFFFF
        self.ws(w, a[0], r)
        w.scc = int(r != 0)

    def i_s_lshl_b64(self, w, ins, a, m):
        r = (self.rs64(w, a[1]) << (self.rs(w, a[2]) & 63)) & 0xFFFFFFFFFFFFFFFF
        self.ws64(w, a[0], r)
        w.scc = int(r != 0)

    def i_s_and_saveexec_b64(self, w, ins, a, m):
        old = self.rs64(w, "exec")
        new = old & self.rs64(w, a[1])
        self.ws64(w, a[0], old)
        self.ws64(w, "exec", new)
        w.scc = int(new != 0)

    def i_s_or_saveexec_b64(self, w, ins, a, m):
        old = self.rs64(w, "exec")
        new = old | self.rs64(w, a[1])
        self.ws64(w, a[0], old)
        self.ws64(w, "exec", new)
        w.scc = int(new != 0)

    def i_s_xor_saveexec_b64(self, w, ins, a, m):
        old = self.rs64(w, "exec")
        new = old ^ self.rs64(w, a[1])
        self.ws64(w, a[0], old)
        self.ws64(w, "exec", new)
        w.scc = int(new != 0)

    def i_s_andn2_saveexec_b64(self, w, ins, a, m):
        old = self.rs64(w, "exec")
        new = self.rs64(w, a[1]) & ~old & 0xFFFFFFFFFFFFFFFF
        self.ws64(w, a[0], old)
        self.ws64(w, "exec", new)
        w.scc = int(new != 0)

    def i_s_cselect_b32(self, w, ins, a, m): self.ws(w, a[0], self.rs(w, a[1]) if w.scc else self.rs(w, a[2]))
    def i_s_cselect_b64(self, w, ins, a, m): self.ws64(w, a[0], self.rs64(w, a[1]) if w.scc else self.rs64(w, a[2]))

    def i_s_ff1_i32_b64(self, w, ins, a, m):
        x = self.rs64(w, a[1])
        self.ws(w, a[0], 0xFFFFFFFF if x == 0 else (x & -x).bit_length() - 1)

    def _scmp(self, w, a, fn, signed=False):
        x, y = self.rs(w, a[0]), self.rs(w, a[1])
        if signed:
            x = x - (1 << 32) if x >> 31 else x
            y = y - (1 << 32) if y >> 31 else y
        w.scc = int(fn(x, y))

    def i_s_cmp_ge_u32(self, w, ins, a, m): self._scmp(w, a, lambda x, y: x >= y)
    def i_s_cmp_lt_u32(self, w, ins, a, m): self._scmp(w, a, lambda x, y: x < y)
    def i_s_cmp_le_u32(self, w, ins, a, m): self._scmp(w, a, lambda x, y: x <= y)
    def i_s_cmp_gt_u32(self, w, ins, a, m): self._scmp(w, a, lambda x, y: x > y)
    def i_s_cmp_eq_u32(self, w, ins, a, m): self._scmp(w, a, lambda x, y: x == y)
    def i_s_cmp_lg_u32(self, w, ins, a, m): self._scmp(w, a, lambda x, y: x != y)
    def i_s_cmp_gt_i32(self, w, ins, a, m): self._scmp(w, a, lambda x, y: x > y, True)
    def i_s_cmp_lt_i32(self, w, ins, a, m): self._scmp(w, a, lambda x, y: x < y, True)
    def i_s_cmp_ge_i32(self, w, ins, a, m): self._scmp(w, a, lambda x, y: x >= y, True)
    def i_s_cmp_le_i32(self, w, ins, a, m): self._scmp(w, a, lambda x, y: x <= y, True)
    def i_s_cmp_eq_i32(self, w, ins, a, m): self._scmp(w, a, lambda x, y: x == y, True)
    def i_s_cmp_lg_i32(self, w, ins, a, m): self._scmp(w, a, lambda x, y: x != y, True)
    def i_s_cmpk_lt_u32(self, w, ins, a, m): w.scc = int(self.rs(w, a[0]) < (parse_int(a[1]) & 0xFFFF))
    def i_s_bitcmp1_b32(self, w, ins, a, m): w.scc = (self.rs(w, a[0]) >> (self.rs(w, a[1]) & 31)) & 1
    def i_s_bitcmp0_b32(self, w, ins, a, m): w.scc = 1 - ((self.rs(w, a[0]) >> (self.rs(w, a[1]) & 31)) & 1)
    def i_s_cmp_eq_u64(self, w, ins, a, m): w.scc = int(self.rs64(w, a[0]) == self.rs64(w, a[1]))
    def i_s_cmp_lg_u64(self, w, ins, a, m): w.scc = int(self.rs64(w, a[0]) != self.rs64(w, a[1]))

    def _branch(self, w, a, cond):
        if cond:
            w.pc = self.labels[a[0]]

    def i_s_branch(self, w, ins, a, m): self._branch(w, a, True)
    def i_s_cbranch_scc0(self, w, ins, a, m): self._branch(w, a, w.scc == 0)
    def i_s_cbranch_scc1(self, w, ins, a, m): self._branch(w, a, w.scc == 1)
    def i_s_cbranch_vccz(self, w, ins, a, m): self._branch(w, a, self.rs64(w, "vcc") == 0)
    def i_s_cbranch_vccnz(self, w, ins, a, m): self._branch(w, a, self.rs64(w, "vcc") != 0)
    def i_s_cbranch_execz(self, w, ins, a, m): self._branch(w, a, self.rs64(w, "exec") == 0)
    def i_s_cbranch_execnz(self, w, ins, a, m): self._branch(w, a, self.rs64(w, "exec") != 0)

    def _sload(self, w, ins, a, n):
        addr = self.rs64(w, a[1]) + parse_int(a[2])
        b = self.mem.load(addr, 4 * n, "line %d %s" % (ins.line, ins.text))
        i = self.sreg_index(a[0])
        for k in range(n):
            w.s[i + k] = U32(struct.unpack_from("<I", b, 4 * k)[0])

    def i_s_load_dword(self, w, ins, a, m): self._sload(w, ins, a, 1)
    def i_s_load_dwordx2(self, w, ins, a, m): self._sload(w, ins, a, 2)
    def i_s_load_dwordx4(self, w, ins, a, m): self._sload(w, ins, a, 4)
    def i_s_load_dwordx8(self, w, ins, a, m): self._sload(w, ins, a, 8)

    # vector ALU -----------------------------------------------------------------
    def i_v_mov_b32(self, w, ins, a, m):
        src = self.rv(w, a[1])
        if ins.op.endswith("_dpp"):
            src = self.dpp(w, src, m)
            if src is None:
                return
            val, valid = src
            mask = w.exec_mask()
            if m.get("bound_ctrl") in ("1", "0") or "bound_ctrl" in m:
                val = np.where(valid, val, U32(0))
                self.wv(w, a[0], val, mask)
            else:
                self.wv(w, a[0], val, mask & valid)
            return
        self.wv(w, a[0], src)

    def dpp(self, w, src, m):
        out = np.zeros(LANES, dtype=U32)
        valid = np.zeros(LANES, dtype=bool)
        ex = w.exec_mask()
        if "wave_shr" in m:     # lane i <- lane i-1
            out[1:] = src[:-1]
            valid[1:] = ex[:-1]
        elif "wave_shl" in m:   # lane i <- lane i+1
            out[:-1] = src[1:]
            valid[:-1] = ex[1:]
        else:
            raise NotImplementedError("dpp control %r" % m)
        if m.get("row_mask", "0xf") != "0xf" or m.get("bank_mask", "0xf") != "0xf":
            raise NotImplementedError("dpp masks")
        return out, valid

    def i_v_mov_b64(self, w, ins, a, m): self.wv64(w, a[0], self.rv64(w, a[1]))
    def i_v_add_u32(self, w, ins, a, m): self.wv(w, a[0], self.rv(w, a[1]) + self.rv(w, a[2]))
    def i_v_sub_u32(self, w, ins, a, m): self.wv(w, a[0], self.rv(w, a[1]) - self.rv(w, a[2]))
    def i_v_subrev_u32(self, w, ins, a, m): self.wv(w, a[0], self.rv(w, a[2]) - self.rv(w, a[1]))
    def i_v_and_b32(self, w, ins, a, m): self.wv(w, a[0], self.rv(w, a[1]) & self.rv(w, a[2]))
    def i_v_or_b32(self, w, ins, a, m): self.wv(w, a[0], self.rv(w, a[1]) | self.rv(w, a[2]))
    def i_v_xor_b32(self, w, ins, a, m): self.wv(w, a[0], self.rv(w, a[1]) ^ self.rv(w, a[2]))
    def i_v_max_u32(self, w, ins, a, m): self.wv(w, a[0], np.maximum(self.rv(w, a[1]), self.rv(w, a[2])))
    def i_v_min_u32(self, w, ins, a, m): self.wv(w, a[0], np.minimum(self.rv(w, a[1]), self.rv(w, a[2])))
    def i_v_min3_u32(self, w, ins, a, m):
        self.wv(w, a[0], np.minimum(np.minimum(self.rv(w, a[1]), self.rv(w, a[2])), self.rv(w, a[3])))
    def i_v_max3_u32(self, w, ins, a, m):
        self.wv(w, a[0], np.maximum(np.maximum(self.rv(w, a[1]), self.rv(w, a[2])), self.rv(w, a[3])))
    def i_v_add3_u32(self, w, ins, a, m): self.wv(w, a[0], self.rv(w, a[1]) + self.rv(w, a[2]) + self.rv(w, a[3]))
    def _sdwa_sel(self, x, sel):
        if sel in (None, "DWORD"):
            return x
        if sel.startswith("BYTE_"):
            return (x >> U32(8 * int(sel[5:]))) & U32(0xFF)
        if sel.startswith("WORD_"):
            return (x >> U32(16 * int(sel[5:]))) & U32(0xFFFF)
        raise NotImplementedError(sel)

    def i_v_lshlrev_b32(self, w, ins, a, m):
        x, y = self.rv(w, a[1]), self.rv(w, a[2])
        if ins.op.endswith("_sdwa"):
            if m.get("dst_sel", "DWORD") != "DWORD":
                raise NotImplementedError("sdwa dst_sel")
            x, y = self._sdwa_sel(x, m.get("src0_sel")), self._sdwa_sel(y, m.get("src1_sel"))
        self.wv(w, a[0], y << (x & U32(31)))
    def i_v_ashrrev_i32(self, w, ins, a, m):
        self.wv(w, a[0], (self.rv(w, a[2]).view(np.int32) >> (self.rv(w, a[1]) & U32(31)).astype(np.int32)).view(U32))

    def i_v_lshlrev_b64(self, w, ins, a, m):
        self.wv64(w, a[0], self.rv64(w, a[2]) << (self.rv(w, a[1]).astype(U64) & U64(63)))

    def i_v_sub_co_u32(self, w, ins, a, m): raise NotImplementedError("carry ops")

    def i_v_lshrrev_b32(self, w, ins, a, m): self.wv(w, a[0], self.rv(w, a[2]) >> (self.rv(w, a[1]) & U32(31)))
    def i_v_lshl_add_u32(self, w, ins, a, m): self.wv(w, a[0], (self.rv(w, a[1]) << (self.rv(w, a[2]) & U32(31))) + self.rv(w, a[3]))
    def i_v_add_lshl_u32(self, w, ins, a, m): self.wv(w, a[0], (self.rv(w, a[1]) + self.rv(w, a[2])) << (self.rv(w, a[3]) & U32(31)))
    def i_v_lshl_or_b32(self, w, ins, a, m): self.wv(w, a[0], (self.rv(w, a[1]) << (self.rv(w, a[2]) & U32(31))) | self.rv(w, a[3]))
    def i_v_xad_u32(self, w, ins, a, m): self.wv(w, a[0], (self.rv(w, a[1]) ^ self.rv(w, a[2])) + self.rv(w, a[3]))
    def i_v_or3_b32(self, w, ins, a, m): self.wv(w, a[0], self.rv(w, a[1]) | self.rv(w, a[2]) | self.rv(w, a[3]))
    def i_v_not_b32(self, w, ins, a, m): self.wv(w, a[0], ~self.rv(w, a[1]))
    def i_v_sub_nc_u32(self, w, ins, a, m): self.wv(w, a[0], self.rv(w, a[1]) - self.rv(w, a[2]))
    def i_v_and_or_b32(self, w, ins, a, m): self.wv(w, a[0], (self.rv(w, a[1]) & self.rv(w, a[2])) | self.rv(w, a[3]))

    def i_v_lshl_add_u64(self, w, ins, a, m):
        self.wv64(w, a[0], (self.rv64(w, a[1]) << (self.rv(w, a[2]).astype(U64) & U64(7))) + self.rv64(w, a[3]))

    def i_v_bfe_u32(self, w, ins, a, m):
        x, off, wd = self.rv(w, a[1]), self.rv(w, a[2]) & U32(31), self.rv(w, a[3]) & U32(31)
        mask = ((U64(1) << wd.astype(U64)) - U64(1)).astype(U32)
        self.wv(w, a[0], np.where(wd == 0, U32(0), (x >> off) & mask))

    def i_v_alignbit_b32(self, w, ins, a, m):
        both = (self.rv(w, a[1]).astype(U64) << U64(32)) | self.rv(w, a[2]).astype(U64)
        self.wv(w, a[0], (both >> (self.rv(w, a[3]) & U32(31)).astype(U64)).astype(U32))

    def i_v_bitop3_b32(self, w, ins, a, m):
        x, y, z = self.rv(w, a[1]), self.rv(w, a[2]), self.rv(w, a[3])
        table = parse_int(m["bitop3"])
        out = np.zeros(LANES, dtype=U32)
        for k in range(8):
            if table >> k & 1:
                out |= (x if k & 4 else ~x) & (y if k & 2 else ~y) & (z if k & 1 else ~z)
        self.wv(w, a[0], out)

    def i_v_mad_u32_u24(self, w, ins, a, m):
        self.wv(w, a[0], ((self.rv(w, a[1]) & U32(0xFFFFFF)).astype(U64) * (self.rv(w, a[2]) & U32(0xFFFFFF)).astype(U64)).astype(U32) + self.rv(w, a[3]))

    def i_v_mul_u32_u24(self, w, ins, a, m):
        self.wv(w, a[0], ((self.rv(w, a[1]) & U32(0xFFFFFF)).astype(U64) * (self.rv(w, a[2]) & U32(0xFFFFFF)).astype(U64)).astype(U32))

    def i_v_mul_i32_i24(self, w, ins, a, m):
        def sx(x):
            x = (x & U32(0xFFFFFF)).astype(np.int64)
            return np.where(x & 0x800000, x - 0x1000000, x)
        self.wv(w, a[0], (sx(self.rv(w, a[1])) * sx(self.rv(w, a[2]))).astype(np.int64).astype(U64).astype(U32))

    def i_v_mad_i32_i24(self, w, ins, a, m):
        def sx(x):
            x = (x & U32(0xFFFFFF)).astype(np.int64)
            return np.where(x & 0x800000, x - 0x1000000, x)
        self.wv(w, a[0], ((sx(self.rv(w, a[1])) * sx(self.rv(w, a[2]))).astype(U64) + self.rv(w, a[3]).astype(U64)).astype(U32))

    def i_v_perm_b32(self, w, ins, a, m):
        s0, s1, sel = self.rv(w, a[1]), self.rv(w, a[2]), self.rv(w, a[3])
        both = (s0.astype(U64) << U64(32)) | s1.astype(U64)
        out = np.zeros(LANES, dtype=U32)
        for i in range(4):
            sb = (sel >> U32(8 * i)) & U32(0xFF)
            byte = np.where(sb < 8, (both >> (sb.astype(U64) & U64(7)) * U64(8)).astype(U32) & U32(0xFF),
                            np.where(sb == 12, U32(0), U32(0xFF)))
            if ((sb >= 8) & (sb < 12)).any():
                raise NotImplementedError("v_perm sign selectors")
            out |= byte.astype(U32) << U32(8 * i)
        self.wv(w, a[0], out)

    def i_v_mad_u64_u32(self, w, ins, a, m):
        # v_mad_u64_u32 vdst[2], sdst(carry), src0, src1, src2[2]
        prod = self.rv(w, a[2]).astype(object) * self.rv(w, a[3]).astype(object) + self.rv64(w, a[4]).astype(object)
        lo = np.array([int(x) & 0xFFFFFFFFFFFFFFFF for x in prod], dtype=U64)
        self.wv64(w, a[0], lo)
        self.ws64(w, a[1], self.mask_to_int(np.array([int(x) >> 64 != 0 for x in prod]), w))

    def i_v_mul_lo_u32(self, w, ins, a, m):
        self.wv(w, a[0], (self.rv(w, a[1]).astype(U64) * self.rv(w, a[2]).astype(U64)).astype(U32))

    def i_v_mul_hi_u32(self, w, ins, a, m):
        self.wv(w, a[0], ((self.rv(w, a[1]).astype(U64) * self.rv(w, a[2]).astype(U64)) >> U64(32)).astype(U32))

    def i_v_mul_f32(self, w, ins, a, m):
        self.wv(w, a[0], (self.rv(w, a[1]).view(np.float32) * self.rv(w, a[2]).view(np.float32)).astype(np.float32).view(U32))

    def i_v_rcp_iflag_f32(self, w, ins, a, m):
        with np.errstate(divide="ignore"):
            self.wv(w, a[0], (np.float32(1.0) / self.rv(w, a[1]).view(np.float32)).astype(np.float32).view(U32))

    def i_v_cvt_f32_u32(self, w, ins, a, m): self.wv(w, a[0], self.rv(w, a[1]).astype(np.float32).view(U32))

    def i_v_cvt_u32_f32(self, w, ins, a, m):
        f = self.rv(w, a[1]).view(np.float32).astype(np.float64)
        f = np.where(np.isnan(f), 0.0, np.clip(np.trunc(f), 0.0, 4294967295.0))
        self.wv(w, a[0], f.astype(U64).astype(U32))

    def _cmp(self, w, ins, a, fn, signed=False):
        if ins.op.endswith("_e64"):
            dst, x, y = a[0], self.rv(w, a[1]), self.rv(w, a[2])
        else:
            dst, x, y = "vcc", self.rv(w, a[1]), self.rv(w, a[2])
        if signed:
            x, y = x.view(np.int32), y.view(np.int32)
        self.ws64(w, dst, self.mask_to_int(fn(x, y), w))

    def i_v_cmp_lt_u32(self, w, ins, a, m): self._cmp(w, ins, a, lambda x, y: x < y)
    def i_v_cmp_le_u32(self, w, ins, a, m): self._cmp(w, ins, a, lambda x, y: x <= y)
    def i_v_cmp_gt_u32(self, w, ins, a, m): self._cmp(w, ins, a, lambda x, y: x > y)
    def i_v_cmp_ge_u32(self, w, ins, a, m): self._cmp(w, ins, a, lambda x, y: x >= y)
    def i_v_cmp_eq_u32(self, w, ins, a, m): self._cmp(w, ins, a, lambda x, y: x == y)
    def i_v_cmp_ne_u32(self, w, ins, a, m): self._cmp(w, ins, a, lambda x, y: x != y)
    def i_v_cmp_lt_i32(self, w, ins, a, m): self._cmp(w, ins, a, lambda x, y: x < y, True)
    def i_v_cmp_gt_i32(self, w, ins, a, m): self._cmp(w, ins, a, lambda x, y: x > y, True)
    def i_v_cmp_le_i32(self, w, ins, a, m): self._cmp(w, ins, a, lambda x, y: x <= y, True)
    def i_v_cmp_ge_i32(self, w, ins, a, m): self._cmp(w, ins, a, lambda x, y: x >= y, True)
    def i_v_cmp_eq_i32(self, w, ins, a, m): self._cmp(w, ins, a, lambda x, y: x == y, True)
    def i_v_cmp_ne_i32(self, w, ins, a, m): self._cmp(w, ins, a, lambda x, y: x != y, True)

    def i_v_cndmask_b32(self, w, ins, a, m):
        sel = self.int_to_mask(self.rs64(w, a[3] if len(a) > 3 else "vcc"))
        self.wv(w, a[0], np.where(sel, self.rv(w, a[2]), self.rv(w, a[1])))

    def i_v_readfirstlane_b32(self, w, ins, a, m):
        ex = w.exec_mask()
        r, _ = self.vreg(a[1])
        lane = int(np.argmax(ex)) if ex.any() else 0
        self.ws(w, a[0], int(w.v[r][lane]))

    def i_v_readlane_b32(self, w, ins, a, m):
        r, _ = self.vreg(a[1])
        self.ws(w, a[0], int(w.v[r][self.rs(w, a[2]) & 63]))

    def i_v_mbcnt_lo_u32_b32(self, w, ins, a, m):
        mask = self.rs(w, a[1])
        out = np.array([bin(mask & ((1 << min(i, 32)) - 1)).count("1") for i in range(LANES)], dtype=U32)
        self.wv(w, a[0], out + self.rv(w, a[2]))

    def i_v_mbcnt_hi_u32_b32(self, w, ins, a, m):
        mask = self.rs(w, a[1])
        out = np.array([bin(mask & ((1 << max(i - 32, 0)) - 1)).count("1") for i in range(LANES)], dtype=U32)
        self.wv(w, a[0], out + self.rv(w, a[2]))

    # packed 16-bit ----------------------------------------------------------------
    def _halves(self, x):
        return x & U32(0xFFFF), x >> U32(16)

    def _opsel(self, m, n):
        hi = [1] * n
        lo = [0] * n
        if "op_sel_hi" in m:
            hi = [int(t) for t in m["op_sel_hi"].strip("[]").split(",")]
        if "op_sel" in m:
            lo = [int(t) for t in m["op_sel"].strip("[]").split(",")]
        return lo, hi

    def _pk(self, w, ins, a, m, fn, nsrc):
        lo_sel, hi_sel = self._opsel(m, nsrc)
        srcs = [self._halves(self.rv(w, a[1 + k])) for k in range(nsrc)]
        lo_in = [srcs[k][lo_sel[k]] for k in range(nsrc)]
        hi_in = [srcs[k][hi_sel[k]] for k in range(nsrc)]
        lo = fn(*lo_in) & U32(0xFFFF)
        hi = fn(*hi_in) & U32(0xFFFF)
        self.wv(w, a[0], lo | (hi << U32(16)))

    def i_v_pk_mad_i16(self, w, ins, a, m): self._pk(w, ins, a, m, lambda x, y, z: x * y + z, 3)
    def i_v_pk_mad_u16(self, w, ins, a, m): self._pk(w, ins, a, m, lambda x, y, z: x * y + z, 3)
    def i_v_pk_sub_i16(self, w, ins, a, m): self._pk(w, ins, a, m, lambda x, y: x - y, 2)
    def i_v_pk_add_u16(self, w, ins, a, m): self._pk(w, ins, a, m, lambda x, y: x + y, 2)
    def i_v_pk_min_u16(self, w, ins, a, m): self._pk(w, ins, a, m, lambda x, y: np.minimum(x, y), 2)
    def i_v_pk_max_u16(self, w, ins, a, m): self._pk(w, ins, a, m, lambda x, y: np.maximum(x, y), 2)
    def i_v_pk_lshrrev_b16(self, w, ins, a, m): self._pk(w, ins, a, m, lambda s, x: x >> (s & U32(15)), 2)

    def i_v_pk_ashrrev_i16(self, w, ins, a, m):
        def sar(s, x):
            sx = np.where(x & U32(0x8000), x | U32(0xFFFF0000), x).view(np.int32)
            return (sx >> (s & U32(15)).astype(np.int32)).view(U32)
        self._pk(w, ins, a, m, sar, 2)

    # LDS --------------------------------------------------------------------------------
    def _lanes(self, w):
        return [i for i in range(LANES) if w.exec_mask()[i]]

    def i_ds_read2_b32(self, w, ins, a, m):
        r, _ = self.vreg(a[0])
        addr = self.rv(w, a[1])
        o0, o1 = 4 * parse_int(m.get("offset0", "0")), 4 * parse_int(m.get("offset1", "0"))
        for i in self._lanes(w):
            w.v[r][i] = struct.unpack("<I", self.lds_read(int(addr[i]) + o0, 4))[0]
            w.v[r + 1][i] = struct.unpack("<I", self.lds_read(int(addr[i]) + o1, 4))[0]

    def i_ds_read2st64_b32(self, w, ins, a, m):
        r, _ = self.vreg(a[0])
        addr = self.rv(w, a[1])
        o0, o1 = 256 * parse_int(m.get("offset0", "0")), 256 * parse_int(m.get("offset1", "0"))
        for i in self._lanes(w):
            w.v[r][i] = struct.unpack("<I", self.lds_read(int(addr[i]) + o0, 4))[0]
            w.v[r + 1][i] = struct.unpack("<I", self.lds_read(int(addr[i]) + o1, 4))[0]

    def i_ds_write2_b32(self, w, ins, a, m):
        addr = self.rv(w, a[0])
        v0, v1 = self.rv(w, a[1]), self.rv(w, a[2])
        o0, o1 = 4 * parse_int(m.get("offset0", "0")), 4 * parse_int(m.get("offset1", "0"))
        for i in self._lanes(w):
            self.lds_write(int(addr[i]) + o0, struct.pack("<I", int(v0[i])))
            self.lds_write(int(addr[i]) + o1, struct.pack("<I", int(v1[i])))

    def _ds_read(self, w, a, m, n, align):
        r, _ = self.vreg(a[0])
        addr = self.rv(w, a[1])
        off = parse_int(m.get("offset", "0"))
        for i in self._lanes(w):
            ad = int(addr[i]) + off
            if ad % align:
                raise Fault("misaligned LDS read of %d bytes at %d" % (4 * n, ad))
            b = self.lds_read(ad, 4 * n)
            for k in range(n):
                w.v[r + k][i] = struct.unpack_from("<I", b, 4 * k)[0]

    def i_ds_read_b32(self, w, ins, a, m): self._ds_read(w, a, m, 1, 4)
    def i_ds_read_b64(self, w, ins, a, m): self._ds_read(w, a, m, 2, 8)
    def i_ds_read_b96(self, w, ins, a, m): self._ds_read(w, a, m, 3, 4)
    def i_ds_read_b128(self, w, ins, a, m): self._ds_read(w, a, m, 4, 16)

    def _ds_write(self, w, a, m, n, align):
        addr = self.rv(w, a[0])
        r, _ = self.vreg(a[1])
        off = parse_int(m.get("offset", "0"))
        for i in self._lanes(w):
            ad = int(addr[i]) + off
            if ad % align:
                raise Fault("misaligned LDS write of %d bytes at %d" % (4 * n, ad))
            self.lds_write(ad, b"".join(struct.pack("<I", int(w.v[r + k][i])) for k in range(n)))

    def i_ds_write_b32(self, w, ins, a, m): self._ds_write(w, a, m, 1, 4)
    def i_ds_write_b64(self, w, ins, a, m): self._ds_write(w, a, m, 2, 8)
    def i_ds_write_b128(self, w, ins, a, m): self._ds_write(w, a, m, 4, 16)

    def i_ds_write_b16(self, w, ins, a, m):
        addr, val = self.rv(w, a[0]), self.rv(w, a[1])
        off = parse_int(m.get("offset", "0"))
        for i in self._lanes(w):
            self.lds_write(int(addr[i]) + off, struct.pack("<H", int(val[i]) & 0xFFFF))

    def i_ds_read_u16(self, w, ins, a, m):
        r, _ = self.vreg(a[0])
        addr = self.rv(w, a[1])
        off = parse_int(m.get("offset", "0"))
        for i in self._lanes(w):
            w.v[r][i] = struct.unpack("<H", self.lds_read(int(addr[i]) + off, 2))[0]

    def i_ds_read_u8(self, w, ins, a, m):
        r, _ = self.vreg(a[0])
        addr = self.rv(w, a[1])
        off = parse_int(m.get("offset", "0"))
        for i in self._lanes(w):
            w.v[r][i] = self.lds_read(int(addr[i]) + off, 1)[0]

    def i_ds_write_b8(self, w, ins, a, m):
        addr, val = self.rv(w, a[0]), self.rv(w, a[1])
        off = parse_int(m.get("offset", "0"))
        for i in self._lanes(w):
            self.lds_write(int(addr[i]) + off, bytes([int(val[i]) & 0xFF]))

    def i_ds_write_b8_d16_hi(self, w, ins, a, m):
        addr, val = self.rv(w, a[0]), self.rv(w, a[1])
        off = parse_int(m.get("offset", "0"))
        for i in self._lanes(w):
            self.lds_write(int(addr[i]) + off, bytes([(int(val[i]) >> 16) & 0xFF]))

    # global -----------------------------------------------------------------------------
    def _gaddr(self, w, a_addr, a_s, m):
        off = parse_int(m.get("offset", "0"))
        if a_s is not None and a_s != "off":
            return self.rs64(w, a_s) + self.rv(w, a_addr).astype(object) + off, off
        return self.rv64(w, a_addr).astype(object) + off, off

    def _gload(self, w, ins, a, m, n):
        r, _ = self.vreg(a[0])
        saddr = a[2] if len(a) > 2 else ("off" if m.get("off") else None)
        addr, _ = self._gaddr(w, a[1], saddr, m)
        for i in self._lanes(w):
            b = self.mem.load(int(addr[i]), 4 * n, "line %d lane %d wave %d: %s" % (ins.line, i, w.id, ins.text))
            for k in range(n):
                w.v[r + k][i] = struct.unpack_from("<I", b, 4 * k)[0]

    def _gload_small(self, w, ins, a, m, nbytes):
        r, _ = self.vreg(a[0])
        saddr = a[2] if len(a) > 2 else None
        addr, _ = self._gaddr(w, a[1], saddr, m)
        for i in self._lanes(w):
            b = self.mem.load(int(addr[i]), nbytes, "line %d lane %d wave %d: %s" % (ins.line, i, w.id, ins.text))
            w.v[r][i] = int.from_bytes(b, "little")

    def i_flat_load_ushort(self, w, ins, a, m): self._gload_small(w, ins, a, m, 2)
    def i_global_load_ushort(self, w, ins, a, m): self._gload_small(w, ins, a, m, 2)
    def i_global_load_ubyte(self, w, ins, a, m): self._gload_small(w, ins, a, m, 1)
    def i_global_load_dword(self, w, ins, a, m): self._gload(w, ins, a, m, 1)
    def i_global_load_dwordx2(self, w, ins, a, m): self._gload(w, ins, a, m, 2)
    def i_global_load_dwordx4(self, w, ins, a, m): self._gload(w, ins, a, m, 4)

    def _gstore(self, w, ins, a, m, nbytes, hi=False):
        saddr = a[2] if len(a) > 2 else ("off" if m.get("off") else None)
        addr, _ = self._gaddr(w, a[0], saddr, m)
        r, _ = self.vreg(a[1])
        for i in self._lanes(w):
            if nbytes >= 4:
                b = b"".join(struct.pack("<I", int(w.v[r + k][i])) for k in range(nbytes // 4))
            else:
                v = int(w.v[r][i])
                if hi:
                    v >>= 16
                b = struct.pack("<I", v)[:nbytes]
            self.mem.store(int(addr[i]), b, "line %d lane %d wave %d: %s" % (ins.line, i, w.id, ins.text))

    def i_global_store_dword(self, w, ins, a, m): self._gstore(w, ins, a, m, 4)
    def i_global_store_dwordx2(self, w, ins, a, m): self._gstore(w, ins, a, m, 8)
    def i_global_store_dwordx3(self, w, ins, a, m): self._gstore(w, ins, a, m, 12)
    def i_global_store_dwordx4(self, w, ins, a, m): self._gstore(w, ins, a, m, 16)
    def i_global_store_short(self, w, ins, a, m): self._gstore(w, ins, a, m, 2)
    def i_global_store_byte(self, w, ins, a, m): self._gstore(w, ins, a, m, 1)
    def i_global_store_byte_d16_hi(self, w, ins, a, m): self._gstore(w, ins, a, m, 1, True)
    def i_global_store_short_d16_hi(self, w, ins, a, m): self._gstore(w, ins, a, m, 2, True)

    def i_global_atomic_or(self, w, ins, a, m):
        saddr = a[2] if len(a) > 2 else None
        addr, _ = self._gaddr(w, a[0], saddr, m)
        val = self.rv(w, a[1])
        for i in self._lanes(w):
            old = struct.unpack("<I", self.mem.load(int(addr[i]), 4, ins.text))[0]
            self.mem.store(int(addr[i]), struct.pack("<I", old | int(val[i])), ins.text)

    # ---- a workgroup --------------------------------------------------------------------
    def run_workgroup(self, wg_id, kernarg_addr, waves=3, limit=5_000_000):
        ws = []
        for k in range(waves):
            w = Wave(k)
            w.s[0] = U32(kernarg_addr & 0xFFFFFFFF)
            w.s[1] = U32(kernarg_addr >> 32)
            w.s[2] = U32(wg_id)
            w.s[EXEC] = U32(0xFFFFFFFF)
            w.s[EXEC + 1] = U32(0xFFFFFFFF)
            w.v[0] = np.arange(LANES, dtype=U32) + U32(64 * k)
            # poison what the kernel must not depend on
            w.v[1:] = U32(0xDEADBEEF)
            w.s[3:100] = U32(0xBAD0BAD0)
            ws.append(w)
        steps = 0
        while not all(w.done for w in ws):
            progressed = False
            for w in ws:
                while not w.done and not w.at_barrier:
                    self.step(w)
                    steps += 1
                    progressed = True
                    if steps > limit:
                        raise Fault("workgroup %d: instruction limit reached" % wg_id)
            live = [w for w in ws if not w.done]
            if live and all(w.at_barrier for w in live):
                for w in live:
                    w.at_barrier = False
                progressed = True
            if not progressed:
                raise Fault("workgroup %d: no wave can proceed" % wg_id)
        return steps


def read_regions(f):
    (count,) = struct.unpack("<Q", f.read(8))
    out = []
    for _ in range(count):
        addr, n = struct.unpack("<QQ", f.read(16))
        out.append((addr, f.read(n)))
    return out


def main():
    args = [a for a in sys.argv[1:] if not a.startswith("--")]
    opts = dict(a[2:].split("=", 1) for a in sys.argv[1:] if a.startswith("--") and "=" in a)
    insts, labels, lds_size = parse_kernel(args[0])
    f = open(args[1], "rb")
    n, mode, kind, grid, block, _ = struct.unpack("<6i", f.read(24))
    (kn,) = struct.unpack("<Q", f.read(8))
    kernarg = bytearray(f.read(kn))
    regions = read_regions(f)
    # hidden arguments behind the explicit ones (8-byte aligned): block counts, group sizes
    hidden = (kn + 7) // 8 * 8
    kernarg += bytes(hidden - kn)
    kernarg += struct.pack("<3I3H", grid, 1, 1, block, 1, 1) + bytes(256)
    mem = Memory()
    KA = 0x7F0000000000
    mem.add(KA, kernarg, "kernarg")
    for addr, data in regions:
        mem.add(addr, data, "buffer")
    lo, hi = 0, grid
    if "wg" in opts:
        lo, hi = [int(t) for t in opts["wg"].split(":")]
    print("kernel for N=%d mode=%d kind=%d: grid %d, block %d, %d instructions, LDS %d, hidden args at %d" %
          (n, mode, kind, grid, block, len(insts), lds_size, hidden), flush=True)
    emu = Emu(insts, labels, lds_size, mem)
    total = 0
    for wg in range(lo, hi):
        emu.lds[:] = bytes([0xCD]) * len(emu.lds)      # garbage from the previous tenant
        try:
            total += emu.run_workgroup(wg, KA, waves=block // 64)
        except Fault as e:
            print("FAULT in workgroup %d: %s" % (wg, e), flush=True)
            return 1
        if (wg - lo) % 20 == 0:
            print("workgroup %d done, %d instructions so far, LDS accesses out of range: %d" % (wg, total, emu.lds_oob), flush=True)
    print("all workgroups done: %d wave instructions, LDS accesses out of range: %d" % (total, emu.lds_oob))
    if "hist" in opts:      # how often each instruction ran: where a kernel's instructions go
        with open(opts["hist"], "w") as hf:
            for k, ins in enumerate(insts):
                hf.write("%9d  %5d  %s\n" % (emu.executed.get(k, 0), ins.line, ins.text))
    if emu.lds_oob:
        return 1
    if len(args) > 2:
        after = dict(read_regions(open(args[2], "rb")))
        bad = 0
        for base, data, name in mem.regions[1:]:
            want = after.get(base)
            if want is None or (lo, hi) != (0, grid):
                continue
            if bytes(data) != want:
                k = next(i for i in range(len(want)) if data[i] != want[i])
                print("buffer at 0x%x differs from the host build's at byte %d of %d" % (base, k, len(want)))
                bad += 1
        print("buffers that differ from the host build's: %d of %d" % (bad, len(after)))
        return 1 if bad else 0
    return 0


if __name__ == "__main__":
    sys.exit(main())
