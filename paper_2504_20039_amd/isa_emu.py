"""A small emulator of the address arithmetic of one wave of a compiled gfx950 kernel (assembly text from hipcc -S), for the
build-time check of the kernels that issue hand-written loads with their own s_waitcnt accounting (check_isa.py).

It executes scalar ALU instructions exactly, the vector-ALU subset used for addressing for all 64 lanes, SGPR spills through
v_writelane / v_readlane, scratch spills, and follows branches.  Everything that holds DATA (loaded values, MFMA results,
floating-point compares) is unknown (None).  Every memory instruction and wait is reported through a callback together with
the emulator's state, so that the caller can check addresses against the buffers and the waits against in-order
completion.  It knows the instructions these kernels compile to, no more: an instruction it does not know raises.
"""
import re
import numpy as np

M32 = 0xFFFFFFFF


def s32(x):
    x &= M32
    return x - (1 << 32) if x & 0x80000000 else x


class Poison(Exception):
    pass


class Emu:
    def __init__(self, lines, kernarg: bytes, wg_id, tid_base, on_vmem, on_insn=None, max_steps=3_000_000):
        self.ins, self.labels = [], {}
        for l in lines:
            t = l.split(';')[0].strip()
            if not t:
                continue
            m = re.match(r'^(\.?\w+):$', t)
            if m:
                self.labels[m.group(1)] = len(self.ins)
                continue
            if t.startswith('.') or t.startswith(';'):
                continue
            self.ins.append(t)
        self.s = {}            # scalar registers: name -> int or None
        self.v = {}            # vector registers: index -> np.uint32[64] or None
        self.a = {}
        self.scc = 0
        self.kernarg = kernarg
        self.KBASE = 0x7000_0000_0000
        self.s['s0'], self.s['s1'] = self.KBASE & M32, self.KBASE >> 32
        self.s['s2'] = wg_id
        self.set64('exec', (1 << 64) - 1)
        self.set64('vcc', 0)
        self.s['m0'] = 0
        self.v[0] = (np.arange(64, dtype=np.uint32) + np.uint32(tid_base))
        self.scratch = {}
        self.on_vmem = on_vmem          # (emu, op, operands, text) at every memory instruction, wait and barrier
        self.on_insn = on_insn          # the same before every instruction, or None
        self.pc = 0
        self.steps = 0
        self.max_steps = max_steps
        self.trace_unknown = {}

    # ---- register access
    def get64(self, name):
        if name in ('vcc', 'exec'):
            lo, hi = self.s.get(name + '_lo'), self.s.get(name + '_hi')
        else:
            m = re.match(r's\[(\d+):(\d+)\]', name)
            lo, hi = self.s.get('s%d' % int(m.group(1))), self.s.get('s%d' % (int(m.group(1)) + 1))
        if lo is None or hi is None:
            return None
        return lo | (hi << 32)

    def set64(self, name, val):
        lo = None if val is None else val & M32
        hi = None if val is None else (val >> 32) & M32
        if name in ('vcc', 'exec'):
            self.s[name + '_lo'], self.s[name + '_hi'] = lo, hi
        else:
            m = re.match(r's\[(\d+):(\d+)\]', name)
            self.s['s%d' % int(m.group(1))], self.s['s%d' % (int(m.group(1)) + 1)] = lo, hi

    def sval(self, tok):
        """32-bit scalar source operand"""
        tok = tok.strip().split()[0]
        if re.match(r'^s\d+$', tok) or tok in ('m0', 'vcc_lo', 'vcc_hi', 'exec_lo', 'exec_hi'):
            return self.s.get(tok)
        if tok == 'scc':
            return self.scc
        if tok == 'off':
            return 0
        if re.match(r'^-?\d+$', tok):
            return int(tok) & M32
        if re.match(r'^-?0x[0-9a-fA-F]+$', tok):
            return int(tok, 16) & M32
        if re.match(r'^-?\d+\.\d*$', tok):
            return int(np.float32(float(tok)).view(np.uint32))
        raise ValueError('scalar operand ' + tok)

    def sval64(self, tok):
        tok = tok.strip()
        if tok in ('vcc', 'exec') or tok.startswith('s['):
            return self.get64(tok)
        v = self.sval(tok)
        if v is None:
            return None
        return v if not (v & 0x80000000 and re.match(r'^-', tok)) else v | (M32 << 32)

    def vsrc(self, tok):
        """vector source operand -> np.uint32[64] or None"""
        tok = tok.strip().split()[0]
        m = re.match(r'^v(\d+)$', tok)
        if m:
            return self.v.get(int(m.group(1)))
        x = self.sval(tok)
        return None if x is None else np.full(64, x, dtype=np.uint32)

    def vset(self, tok, val):
        m = re.match(r'^v(\d+)$', tok.strip().split()[0])
        i = int(m.group(1))
        if val is None:
            self.v[i] = None
            return
        ex = self.get64('exec')
        if ex is None or ex == (1 << 64) - 1 or self.v.get(i) is None:
            self.v[i] = val.astype(np.uint32)          # (a partial write over poison is treated as a full one)
        else:
            mask = np.array([(ex >> k) & 1 for k in range(64)], dtype=bool)
            out = self.v[i].copy()
            out[mask] = val.astype(np.uint32)[mask]
            self.v[i] = out

    def vrange(self, tok):
        tok = tok.strip().split()[0]
        m = re.match(r'^([va])\[(\d+):(\d+)\]$', tok)
        if m:
            return m.group(1), list(range(int(m.group(2)), int(m.group(3)) + 1))
        m = re.match(r'^([va])(\d+)$', tok)
        return m.group(1), [int(m.group(2))]

    def poison_dst(self, tok):
        f, rs = self.vrange(tok)
        for r in rs:
            (self.v if f == 'v' else self.a)[r] = None

    # ---- execution
    def run(self):
        while True:
            if self.pc >= len(self.ins):
                raise RuntimeError('ran off the end')
            self.steps += 1
            if self.steps > self.max_steps:
                raise RuntimeError('step limit')
            t = self.ins[self.pc]
            self.pc += 1
            op, _, rest = t.partition(' ')
            ops = [x.strip() for x in self.split_ops(rest)]
            if op == 's_endpgm':
                return
            if self.on_insn is not None:
                self.on_insn(self, op, ops, t)
            h = getattr(self, 'i_' + op, None)
            if h is not None:
                h(ops, t)
            elif op.startswith('v_mfma'):
                self.poison_dst(ops[0])
            elif op.startswith('v_cmp') or op.startswith('v_cmpx'):
                self.cmp(op, ops)
            elif op.startswith('v_'):
                self.trace_unknown[op] = self.trace_unknown.get(op, 0) + 1
                if re.match(r'^[va](\d+|\[)', ops[0]):
                    self.poison_dst(ops[0])
                elif ops[0].startswith('s[') or ops[0] == 'vcc':
                    self.set64(ops[0], None)
                elif ops[0].startswith('s'):
                    self.s[ops[0]] = None
            elif op.startswith('s_waitcnt') or op in ('s_nop', 's_barrier', 's_setprio', 's_sleep'):
                self.on_vmem(self, op, ops, t)
            else:
                raise RuntimeError('unhandled instruction: ' + t)

    @staticmethod
    def split_ops(rest):
        out, depth, cur = [], 0, ''
        for ch in rest:
            if ch == '[':
                depth += 1
            if ch == ']':
                depth -= 1
            if ch == ',' and depth == 0:
                out.append(cur)
                cur = ''
            else:
                cur += ch
        if cur.strip():
            out.append(cur)
        return out

    # ---- scalar ALU
    def bin32(self, ops, f, scc=None):
        a, b = self.sval(ops[1]), self.sval(ops[2])
        if a is None or b is None:
            self.s[ops[0]] = None
            if scc is not None:
                self.scc = None
            return
        r = f(a, b)
        self.s[ops[0]] = r & M32
        if scc is not None:
            self.scc = scc(a, b, r)

    def i_s_mov_b32(self, o, t): self.s[o[0]] = self.sval(o[1])
    def i_s_movk_i32(self, o, t): self.s[o[0]] = self.sval(o[1]) if not re.match(r'^0x', o[1]) else (s32(int(o[1], 16) << 16) >> 16) & M32
    def i_s_mov_b64(self, o, t): self.set64(o[0], self.sval64(o[1]))
    def i_s_add_i32(self, o, t): self.bin32(o, lambda a, b: a + b, lambda a, b, r: int(s32(a) + s32(b) != s32(r & M32)))
    def i_s_add_u32(self, o, t): self.bin32(o, lambda a, b: a + b, lambda a, b, r: int(r > M32))
    def i_s_sub_i32(self, o, t): self.bin32(o, lambda a, b: a - b, lambda a, b, r: int(s32(a) - s32(b) != s32(r & M32)))
    def i_s_sub_u32(self, o, t): self.bin32(o, lambda a, b: a - b, lambda a, b, r: int(b > a))
    def i_s_mul_i32(self, o, t): self.bin32(o, lambda a, b: s32(a) * s32(b))
    def i_s_mul_hi_u32(self, o, t): self.bin32(o, lambda a, b: (a * b) >> 32)
    def i_s_lshl_b32(self, o, t): self.bin32(o, lambda a, b: a << (b & 31), lambda a, b, r: int((r & M32) != 0))
    def i_s_lshr_b32(self, o, t): self.bin32(o, lambda a, b: a >> (b & 31), lambda a, b, r: int((r & M32) != 0))
    def i_s_ashr_i32(self, o, t): self.bin32(o, lambda a, b: s32(a) >> (b & 31), lambda a, b, r: int((r & M32) != 0))
    def i_s_and_b32(self, o, t): self.bin32(o, lambda a, b: a & b, lambda a, b, r: int((r & M32) != 0))
    def i_s_or_b32(self, o, t): self.bin32(o, lambda a, b: a | b, lambda a, b, r: int((r & M32) != 0))
    def i_s_xor_b32(self, o, t): self.bin32(o, lambda a, b: a ^ b, lambda a, b, r: int((r & M32) != 0))
    def i_s_andn2_b32(self, o, t): self.bin32(o, lambda a, b: a & ~b, lambda a, b, r: int((r & M32) != 0))
    def i_s_min_i32(self, o, t): self.bin32(o, lambda a, b: min(s32(a), s32(b)), lambda a, b, r: int(s32(a) < s32(b)))
    def i_s_max_i32(self, o, t): self.bin32(o, lambda a, b: max(s32(a), s32(b)), lambda a, b, r: int(s32(a) > s32(b)))
    def i_s_min_u32(self, o, t): self.bin32(o, lambda a, b: min(a, b), lambda a, b, r: int(a < b))
    def i_s_max_u32(self, o, t): self.bin32(o, lambda a, b: max(a, b), lambda a, b, r: int(a > b))
    def i_s_lshl1_add_u32(self, o, t): self.bin32(o, lambda a, b: (a << 1) + b, lambda a, b, r: int(r > M32))
    def i_s_lshl2_add_u32(self, o, t): self.bin32(o, lambda a, b: (a << 2) + b, lambda a, b, r: int(r > M32))
    def i_s_lshl3_add_u32(self, o, t): self.bin32(o, lambda a, b: (a << 3) + b, lambda a, b, r: int(r > M32))
    def i_s_lshl4_add_u32(self, o, t): self.bin32(o, lambda a, b: (a << 4) + b, lambda a, b, r: int(r > M32))

    def un32(self, o, f):
        a = self.sval(o[1])
        self.s[o[0]] = None if a is None else f(a) & M32

    def i_s_brev_b32(self, o, t): self.un32(o, lambda a: int('{:032b}'.format(a)[::-1], 2))
    def i_s_not_b32(self, o, t):
        self.un32(o, lambda a: ~a)
        self.scc = None if self.s[o[0]] is None else int(self.s[o[0]] != 0)
    def i_s_sext_i32_i16(self, o, t): self.un32(o, lambda a: ((a & 0xFFFF) ^ 0x8000) - 0x8000)
    def i_s_sext_i32_i8(self, o, t): self.un32(o, lambda a: ((a & 0xFF) ^ 0x80) - 0x80)
    def i_s_abs_i32(self, o, t):
        self.un32(o, lambda a: abs(s32(a)))
        self.scc = None if self.s[o[0]] is None else int(self.s[o[0]] != 0)

    def i_s_bfe_u32(self, o, t):
        self.bin32(o, lambda a, b: (a >> (b & 31)) & ((1 << ((b >> 16) & 0x7f)) - 1), lambda a, b, r: int((r & M32) != 0))

    def i_s_addc_u32(self, o, t):
        a, b = self.sval(o[1]), self.sval(o[2])
        if a is None or b is None or self.scc is None:
            self.s[o[0]], self.scc = None, None
            return
        r = a + b + self.scc
        self.s[o[0]], self.scc = r & M32, int(r > M32)

    def i_s_subb_u32(self, o, t):
        a, b = self.sval(o[1]), self.sval(o[2])
        if a is None or b is None or self.scc is None:
            self.s[o[0]], self.scc = None, None
            return
        r = a - b - self.scc
        self.s[o[0]], self.scc = r & M32, int(b + self.scc > a)

    def i_s_addk_i32(self, o, t):
        a, k = self.s.get(o[0]), self.sval(o[1])
        k = s32(((k & 0xFFFF) ^ 0x8000) - 0x8000)
        if a is None:
            self.scc = None
            return
        r = s32(a) + k
        self.s[o[0]], self.scc = r & M32, int(r != s32(r & M32))

    def i_s_mulk_i32(self, o, t):
        a, k = self.s.get(o[0]), self.sval(o[1])
        k = s32(((k & 0xFFFF) ^ 0x8000) - 0x8000)
        self.s[o[0]] = None if a is None else (s32(a) * k) & M32

    def bin64(self, o, f):
        a, b = self.sval64(o[1]), self.sval64(o[2])
        if a is None or b is None:
            self.set64(o[0], None)
            self.scc = None
            return
        r = f(a, b) & ((1 << 64) - 1)
        self.set64(o[0], r)
        self.scc = int(r != 0)

    def i_s_and_b64(self, o, t): self.bin64(o, lambda a, b: a & b)
    def i_s_or_b64(self, o, t):
        a, b = self.sval64(o[1]), self.sval64(o[2])
        full = (1 << 64) - 1
        if a == full or b == full:          # whatever the other (possibly unknown) operand is
            self.set64(o[0], full); self.scc = 1; return
        if o[0] == 'exec' and (a is None) != (b is None):
            # the end of a structured region: exec (unknown inside it: it followed a compare of data) | the saved mask
            self.set64('exec', a if b is None else b); self.scc = None; return
        self.bin64(o, lambda a, b: a | b)
    def i_s_xor_b64(self, o, t): self.bin64(o, lambda a, b: a ^ b)
    def i_s_andn2_b64(self, o, t): self.bin64(o, lambda a, b: a & ~b)
    def i_s_orn2_b64(self, o, t): self.bin64(o, lambda a, b: a | ~b)
    def i_s_lshl_b64(self, o, t):
        a, b = self.sval64(o[1]), self.sval(o[2])
        if a is None or b is None:
            self.set64(o[0], None); self.scc = None; return
        r = (a << (b & 63)) & ((1 << 64) - 1)
        self.set64(o[0], r); self.scc = int(r != 0)
    def i_s_lshr_b64(self, o, t):
        a, b = self.sval64(o[1]), self.sval(o[2])
        if a is None or b is None:
            self.set64(o[0], None); self.scc = None; return
        r = a >> (b & 63)
        self.set64(o[0], r); self.scc = int(r != 0)
    def i_s_ashr_i64(self, o, t):
        a, b = self.sval64(o[1]), self.sval(o[2])
        if a is None or b is None:
            self.set64(o[0], None); self.scc = None; return
        sa = a - (1 << 64) if a >> 63 else a
        r = (sa >> (b & 63)) & ((1 << 64) - 1)
        self.set64(o[0], r); self.scc = int(r != 0)
    def i_s_not_b64(self, o, t):
        a = self.sval64(o[1])
        self.set64(o[0], None if a is None else (~a) & ((1 << 64) - 1)); self.scc = None if a is None else int(((~a) & ((1 << 64) - 1)) != 0)

    def i_s_cselect_b32(self, o, t):
        a, b = self.sval(o[1]), self.sval(o[2])
        self.s[o[0]] = None if self.scc is None else (a if self.scc else b)
    def i_s_cselect_b64(self, o, t):
        a, b = self.sval64(o[1]), self.sval64(o[2])
        self.set64(o[0], None if self.scc is None else (a if self.scc else b))

    def scmp(self, o, f, signed):
        a, b = self.sval(o[0]), self.sval(o[1])
        if a is None or b is None:
            self.scc = None
            return
        if signed:
            a, b = s32(a), s32(b)
        self.scc = int(f(a, b))

    def i_s_cmp_eq_u32(self, o, t): self.scmp(o, lambda a, b: a == b, False)
    def i_s_cmp_lg_u32(self, o, t): self.scmp(o, lambda a, b: a != b, False)
    def i_s_cmp_eq_i32(self, o, t): self.scmp(o, lambda a, b: a == b, True)
    def i_s_cmp_lg_i32(self, o, t): self.scmp(o, lambda a, b: a != b, True)
    def i_s_cmp_lt_i32(self, o, t): self.scmp(o, lambda a, b: a < b, True)
    def i_s_cmp_le_i32(self, o, t): self.scmp(o, lambda a, b: a <= b, True)
    def i_s_cmp_gt_i32(self, o, t): self.scmp(o, lambda a, b: a > b, True)
    def i_s_cmp_ge_i32(self, o, t): self.scmp(o, lambda a, b: a >= b, True)
    def i_s_cmp_lt_u32(self, o, t): self.scmp(o, lambda a, b: a < b, False)
    def i_s_cmp_le_u32(self, o, t): self.scmp(o, lambda a, b: a <= b, False)
    def i_s_cmp_gt_u32(self, o, t): self.scmp(o, lambda a, b: a > b, False)
    def i_s_cmp_ge_u32(self, o, t): self.scmp(o, lambda a, b: a >= b, False)
    def i_s_cmp_eq_u64(self, o, t):
        a, b = self.sval64(o[0]), self.sval64(o[1]); self.scc = None if a is None or b is None else int(a == b)
    def i_s_cmp_lg_u64(self, o, t):
        a, b = self.sval64(o[0]), self.sval64(o[1]); self.scc = None if a is None or b is None else int(a != b)

    def i_s_load_dword(self, o, t): self.sload(o, 1)
    def i_s_load_dwordx2(self, o, t): self.sload(o, 2)
    def i_s_load_dwordx4(self, o, t): self.sload(o, 4)
    def i_s_load_dwordx8(self, o, t): self.sload(o, 8)
    def i_s_load_dwordx16(self, o, t): self.sload(o, 16)

    def sload(self, o, n):
        base = self.get64(o[1])
        off = self.sval(o[2].split()[0]) if len(o) > 2 else 0
        m = re.search(r'offset:(\S+)', ' '.join(o))
        if m:
            off += int(m.group(1), 0)
        a = base + off - self.KBASE
        assert 0 <= a and a + 4 * n <= len(self.kernarg), ('scalar load outside the kernel arguments', o)
        m = re.match(r's\[(\d+):(\d+)\]', o[0])
        first = int(m.group(1)) if m else int(o[0][1:])
        for k in range(n):
            self.s['s%d' % (first + k)] = int.from_bytes(self.kernarg[a + 4 * k:a + 4 * k + 4], 'little')

    # ---- branches
    def jump(self, label):
        self.pc = self.labels[label]

    def i_s_branch(self, o, t): self.jump(o[0])
    def i_s_cbranch_scc0(self, o, t):
        if self.scc is None: raise Poison('branch on poison scc: ' + t)
        if not self.scc: self.jump(o[0])
    def i_s_cbranch_scc1(self, o, t):
        if self.scc is None: raise Poison('branch on poison scc: ' + t)
        if self.scc: self.jump(o[0])
    def i_s_cbranch_vccz(self, o, t):
        v = self.get64('vcc')
        if v is None: raise Poison('branch on poison vcc: ' + t)
        if v == 0: self.jump(o[0])
    def i_s_cbranch_vccnz(self, o, t):
        v = self.get64('vcc')
        if v is None: raise Poison('branch on poison vcc: ' + t)
        if v != 0: self.jump(o[0])
    def i_s_cbranch_execz(self, o, t):
        v = self.get64('exec')
        if v is not None and v == 0: self.jump(o[0])       # poison exec: assume some lane is on
    def i_s_cbranch_execnz(self, o, t):
        v = self.get64('exec')
        if v is None or v != 0: self.jump(o[0])

    def i_s_and_saveexec_b64(self, o, t):
        ex, src = self.get64('exec'), self.sval64(o[1])
        self.set64(o[0], ex)
        self.set64('exec', None if ex is None or src is None else ex & src)
        self.scc = None
    def i_s_or_saveexec_b64(self, o, t):
        ex, src = self.get64('exec'), self.sval64(o[1])
        self.set64(o[0], ex)
        self.set64('exec', None if ex is None or src is None else ex | src)
        self.scc = None
    def i_s_andn2_saveexec_b64(self, o, t):
        ex, src = self.get64('exec'), self.sval64(o[1])
        self.set64(o[0], ex)
        self.set64('exec', None if ex is None or src is None else src & ~ex)
        self.scc = None

    # ---- vector ALU subset
    def vbin(self, o, f):
        a, b = self.vsrc(o[1]), self.vsrc(o[2])
        self.vset(o[0], None if a is None or b is None else f(a.astype(np.uint64), b.astype(np.uint64)) & np.uint64(M32))

    @staticmethod
    def sx(x):
        return x.astype(np.uint32).view(np.int32).astype(np.int64)

    def i_v_mov_b32_e32(self, o, t): self.vset(o[0], self.vsrc(o[1]))
    def i_v_mov_b32_e64(self, o, t): self.vset(o[0], self.vsrc(o[1]))
    def i_v_add_u32_e32(self, o, t): self.vbin(o, lambda a, b: a + b)
    def i_v_add_u32_e64(self, o, t): self.vbin(o, lambda a, b: a + b)
    def i_v_sub_u32_e32(self, o, t): self.vbin(o, lambda a, b: a - b)
    def i_v_subrev_u32_e32(self, o, t): self.vbin(o, lambda a, b: b - a)
    def i_v_and_b32_e32(self, o, t): self.vbin(o, lambda a, b: a & b)
    def i_v_or_b32_e32(self, o, t): self.vbin(o, lambda a, b: a | b)
    def i_v_xor_b32_e32(self, o, t): self.vbin(o, lambda a, b: a ^ b)
    def i_v_lshlrev_b32_e32(self, o, t): self.vbin(o, lambda a, b: b << (a & np.uint64(31)))
    def i_v_lshrrev_b32_e32(self, o, t): self.vbin(o, lambda a, b: b >> (a & np.uint64(31)))
    def i_v_mul_u32_u24_e32(self, o, t): self.vbin(o, lambda a, b: (a & np.uint64(0xFFFFFF)) * (b & np.uint64(0xFFFFFF)))
    def i_v_mul_lo_u32(self, o, t): self.vbin(o, lambda a, b: a * b)

    def i_v_ashrrev_i32_e32(self, o, t):
        a, b = self.vsrc(o[1]), self.vsrc(o[2])
        self.vset(o[0], None if a is None or b is None else (self.sx(b) >> (a.astype(np.int64) & 31)).astype(np.uint64) & np.uint64(M32))
    def i_v_min_i32_e32(self, o, t):
        a, b = self.vsrc(o[1]), self.vsrc(o[2])
        self.vset(o[0], None if a is None or b is None else np.minimum(self.sx(a), self.sx(b)).astype(np.uint64) & np.uint64(M32))
    def i_v_max_i32_e32(self, o, t):
        a, b = self.vsrc(o[1]), self.vsrc(o[2])
        self.vset(o[0], None if a is None or b is None else np.maximum(self.sx(a), self.sx(b)).astype(np.uint64) & np.uint64(M32))

    def vtri(self, o, f):
        a, b, c = self.vsrc(o[1]), self.vsrc(o[2]), self.vsrc(o[3])
        self.vset(o[0], None if a is None or b is None or c is None else
                  f(a.astype(np.uint64), b.astype(np.uint64), c.astype(np.uint64)) & np.uint64(M32))

    def i_v_mad_u32_u24(self, o, t): self.vtri(o, lambda a, b, c: (a & np.uint64(0xFFFFFF)) * (b & np.uint64(0xFFFFFF)) + c)
    def i_v_lshl_add_u32(self, o, t): self.vtri(o, lambda a, b, c: (a << (b & np.uint64(31))) + c)
    def i_v_lshl_or_b32(self, o, t): self.vtri(o, lambda a, b, c: (a << (b & np.uint64(31))) | c)
    def i_v_add_lshl_u32(self, o, t): self.vtri(o, lambda a, b, c: (a + b) << (c & np.uint64(31)))
    def i_v_add3_u32(self, o, t): self.vtri(o, lambda a, b, c: a + b + c)
    def i_v_and_or_b32(self, o, t): self.vtri(o, lambda a, b, c: (a & b) | c)
    def i_v_bfe_u32(self, o, t): self.vtri(o, lambda a, b, c: (a >> (b & np.uint64(31))) & ((np.uint64(1) << (c & np.uint64(31))) - np.uint64(1)))

    def i_v_bitop3_b32(self, o, t):
        a, b, c = self.vsrc(o[1]), self.vsrc(o[2]), self.vsrc(o[3])
        tt = int(re.search(r'bitop3:(\S+)', t).group(1), 0)
        if a is None or b is None or c is None:
            self.vset(o[0], None); return
        a, b, c = a.astype(np.uint64), b.astype(np.uint64), c.astype(np.uint64)
        r = np.zeros(64, dtype=np.uint64)
        full = np.uint64(M32)
        for idx in range(8):
            if (tt >> idx) & 1:
                ta = a if idx & 4 else (~a) & full
                tb = b if idx & 2 else (~b) & full
                tc = c if idx & 1 else (~c) & full
                r |= ta & tb & tc
        self.vset(o[0], r)

    def v64(self, tok):
        tok = tok.strip().split()[0]
        m = re.match(r'^v\[(\d+):(\d+)\]$', tok)
        if m:
            lo, hi = self.v.get(int(m.group(1))), self.v.get(int(m.group(1)) + 1)
            return None if lo is None or hi is None else lo.astype(np.uint64) | (hi.astype(np.uint64) << np.uint64(32))
        x = self.sval64(tok)
        return None if x is None else np.full(64, x, dtype=np.uint64)

    def vset64(self, tok, val):
        m = re.match(r'^v\[(\d+):(\d+)\]$', tok.strip().split()[0])
        i = int(m.group(1))
        if val is None:
            self.v[i] = self.v[i + 1] = None
            return
        self.vset('v%d' % i, val & np.uint64(M32))
        self.vset('v%d' % (i + 1), val >> np.uint64(32))

    def i_v_lshl_add_u64(self, o, t):
        a, sh, c = self.v64(o[1]), self.sval(o[2]), self.v64(o[3])
        self.vset64(o[0], None if a is None or sh is None or c is None else (a << np.uint64(sh & 63)) + c)

    def i_v_mad_u64_u32(self, o, t):
        a, b, c = self.vsrc(o[2]), self.vsrc(o[3]), self.v64(o[4])
        self.vset64(o[0], None if a is None or b is None or c is None else a.astype(np.uint64) * b.astype(np.uint64) + c)
        if o[1].startswith('s['):
            self.set64(o[1], None)

    def i_v_mad_i64_i32(self, o, t):
        a, b, c = self.vsrc(o[2]), self.vsrc(o[3]), self.v64(o[4])
        self.vset64(o[0], None if a is None or b is None or c is None else
                    (self.sx(a) * self.sx(b)).astype(np.uint64) + c)
        if o[1].startswith('s['):
            self.set64(o[1], None)

    def i_v_mov_b64_e32(self, o, t): self.vset64(o[0], self.v64(o[1]))

    def i_v_accvgpr_write_b32(self, o, t): self.a[int(o[0].strip()[1:])] = self.vsrc(o[1])
    def i_v_accvgpr_read_b32(self, o, t): self.vset(o[0], self.a.get(int(o[1].strip()[1:])))
    def i_v_accvgpr_mov_b32(self, o, t): self.a[int(o[0].strip()[1:])] = self.a.get(int(o[1].strip()[1:]))

    def i_v_mbcnt_lo_u32_b32(self, o, t):
        m, c = self.sval(o[1]), self.vsrc(o[2])
        if m is None or c is None: self.vset(o[0], None); return
        cnt = np.array([bin(m & ((1 << min(k, 32)) - 1)).count('1') for k in range(64)], dtype=np.uint64)
        self.vset(o[0], cnt + c)
    def i_v_mbcnt_hi_u32_b32(self, o, t):
        m, c = self.sval(o[1]), self.vsrc(o[2])
        if m is None or c is None: self.vset(o[0], None); return
        cnt = np.array([bin(m & ((1 << max(k - 32, 0)) - 1)).count('1') for k in range(64)], dtype=np.uint64)
        self.vset(o[0], cnt + c)

    def i_v_readfirstlane_b32(self, o, t):
        a = self.vsrc(o[1])
        self.s[o[0]] = None if a is None else int(a[0])
    def i_v_readlane_b32(self, o, t):
        a, l = self.vsrc(o[1]), self.sval(o[2])
        self.s[o[0]] = None if a is None else int(a[l & 63])
    def i_v_writelane_b32(self, o, t):
        x, l = self.sval(o[1]), self.sval(o[2])
        i = int(o[0][1:])
        cur = np.zeros(64, dtype=np.uint32) if self.v.get(i) is None else self.v[i].copy()
        if x is None:
            raise Poison('an unknown scalar is spilled: ' + t)
        cur[l & 63] = x
        self.v[i] = cur

    def i_v_cndmask_b32_e32(self, o, t):
        a, b, m = self.vsrc(o[1]), self.vsrc(o[2]), self.get64('vcc')
        if a is None or b is None or m is None: self.vset(o[0], None); return
        mask = np.array([(m >> k) & 1 for k in range(64)], dtype=bool)
        self.vset(o[0], np.where(mask, b, a))
    def i_v_cndmask_b32_e64(self, o, t):
        a, b, m = self.vsrc(o[1]), self.vsrc(o[2]), self.sval64(o[3])
        if a is None or b is None or m is None: self.vset(o[0], None); return
        mask = np.array([(m >> k) & 1 for k in range(64)], dtype=bool)
        self.vset(o[0], np.where(mask, b, a))

    def cmp(self, op, ops):
        m = re.match(r'v_cmpx?_(\w+?)_(i32|u32|f32|i64|u64|f64)_e(32|64)', op)
        rel, ty, enc = m.group(1), m.group(2), m.group(3)
        if enc == '32':
            dst, a, b = 'vcc', ops[-2], ops[-1]
            if len(ops) == 3:
                dst = ops[0]
        else:
            dst, a, b = ops[0], ops[1], ops[2]
        res = None
        if ty in ('i32', 'u32'):
            x, y = self.vsrc(a), self.vsrc(b)
            if x is not None and y is not None:
                if ty == 'i32':
                    x, y = self.sx(x), self.sx(y)
                else:
                    x, y = x.astype(np.int64), y.astype(np.int64)
                f = {'lt': x < y, 'le': x <= y, 'gt': x > y, 'ge': x >= y, 'eq': x == y, 'ne': x != y, 'lg': x != y}[rel]
                ex = self.get64('exec')
                if ex is not None:
                    res = sum((1 << k) for k in range(64) if f[k] and (ex >> k) & 1)
        if dst in ('vcc', 'exec') or dst.startswith('s['):
            self.set64(dst, res)
        else:
            raise RuntimeError('compare destination ' + dst)
        if op.startswith('v_cmpx'):
            self.set64('exec', res)

    # ---- memory
    def i_scratch_store_dword(self, o, t): self.scr_store(o, 1)
    def i_scratch_store_dwordx2(self, o, t): self.scr_store(o, 2)
    def i_scratch_store_dwordx3(self, o, t): self.scr_store(o, 3)
    def i_scratch_store_dwordx4(self, o, t): self.scr_store(o, 4)
    def i_scratch_load_dword(self, o, t): self.scr_load(o, 1)
    def i_scratch_load_dwordx2(self, o, t): self.scr_load(o, 2)
    def i_scratch_load_dwordx3(self, o, t): self.scr_load(o, 3)
    def i_scratch_load_dwordx4(self, o, t): self.scr_load(o, 4)

    def scr_off(self, o, first):
        txt = ' '.join(o[first:])
        m = re.search(r'offset:(\S+)', txt)
        off = int(m.group(1), 0) if m else 0
        a, b = o[first].split()[0], o[first + 1].split()[0]
        assert a == 'off', 'scratch with a vector address: ' + txt
        if b != 'off':
            off += self.sval(b)
        return off

    def scr_store(self, o, n):
        # form: scratch_store_dword off, v26, off offset:4
        _, regs = self.vrange(o[1])
        f = o[1].strip()[0]
        txt = ' '.join(o)
        m = re.search(r'offset:(\S+)', txt)
        off = int(m.group(1), 0) if m else 0
        if o[2].split()[0] != 'off':
            off += self.sval(o[2].split()[0])
        for k, r in enumerate(regs):
            self.scratch[off + 4 * k] = (self.v if f == 'v' else self.a).get(r)
        self.on_vmem(self, 'scratch_store', o, '')

    def scr_load(self, o, n):
        f, regs = self.vrange(o[0])
        txt = ' '.join(o)
        m = re.search(r'offset:(\S+)', txt)
        off = int(m.group(1), 0) if m else 0
        assert o[1].strip() == 'off'
        if o[2].split()[0] != 'off':
            off += self.sval(o[2].split()[0])
        for k, r in enumerate(regs):
            (self.v if f == 'v' else self.a)[r] = self.scratch.get(off + 4 * k)
        self.on_vmem(self, 'scratch_load', o, '')

    def vmem(self, op, o, t):
        self.on_vmem(self, op, o, t)

    def i_buffer_load_dwordx4(self, o, t):
        self.on_vmem(self, 'buffer_load_dwordx4', o, t); self.poison_dst(o[0])
    def i_buffer_load_dword(self, o, t):
        self.on_vmem(self, 'buffer_load_dword', o, t); self.poison_dst(o[0])
    def i_global_load_lds_dwordx4(self, o, t): self.on_vmem(self, 'global_load_lds_dwordx4', o, t)
    def i_global_load_dword(self, o, t):
        self.on_vmem(self, 'global_load', o, t); self.poison_dst(o[0])
    def i_global_load_dwordx2(self, o, t):
        self.on_vmem(self, 'global_load', o, t); self.poison_dst(o[0])
    def i_global_load_dwordx4(self, o, t):
        self.on_vmem(self, 'global_load', o, t); self.poison_dst(o[0])
    def i_global_store_dword(self, o, t): self.on_vmem(self, 'global_store', o, t)
    def i_global_store_dwordx2(self, o, t): self.on_vmem(self, 'global_store', o, t)
    def i_global_store_dwordx4(self, o, t): self.on_vmem(self, 'global_store', o, t)
    def i_ds_read_b128(self, o, t):
        self.on_vmem(self, 'ds_read_b128', o, t); self.poison_dst(o[0])
    def i_ds_read_b64(self, o, t):
        self.on_vmem(self, 'ds_read_b64', o, t); self.poison_dst(o[0])
    def i_ds_read_b32(self, o, t):
        self.on_vmem(self, 'ds_read_b32', o, t); self.poison_dst(o[0])
    def i_ds_read2_b64(self, o, t): self.poison_dst(o[0])
    def i_ds_read2_b32(self, o, t): self.poison_dst(o[0])
    def i_ds_read2st64_b64(self, o, t): self.poison_dst(o[0])
    def i_ds_write2_b64(self, o, t): pass
    def i_ds_write2_b32(self, o, t): pass
    def i_ds_write_b128(self, o, t): pass
    def i_ds_write_b64(self, o, t): self.on_vmem(self, 'ds_write_b64', o, t)
    def i_ds_write_b32(self, o, t): self.on_vmem(self, 'ds_write_b32', o, t)
    def i_ds_bpermute_b32(self, o, t): self.poison_dst(o[0])
