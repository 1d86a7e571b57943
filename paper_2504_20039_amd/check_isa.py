"""Build-time check of the generated code of the kernels whose hot loops are hand-scheduled.

Two kernels accumulate through hand-written ``v_mfma`` statements and count their own outstanding loads
(``lm_head_wide.hip`` entirely, ``lm_head_pair9.hip`` for its ninth row block).  Both rely on what the compiler does
around those statements: no accumulator moved between the register files, nothing spilled to scratch memory, and no
``s_waitcnt vmcnt`` of the compiler's own inside the loop (it would wait for the kernel's hand-written loads).  A new
toolchain or flag can change that without any error, so the build compiles the two files to assembly text once more and looks at the
loops.
"""
from __future__ import annotations

import os
import re
import subprocess
import tempfile

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")


def _kernels(asm_text):
    """{mangled name: [lines]} of every kernel in an assembly file."""
    out, cur = {}, None
    for line in asm_text.splitlines():
        m = re.match(r"^(_Z\w+):", line)
        if m:
            cur = m.group(1)
            out[cur] = []
        elif cur is not None:
            out[cur].append(line)
            if "s_endpgm" in line:
                cur = None
    return out


def _innermost_loop(lines):
    """Lines of the innermost loop that holds MFMAs: from its header label to the last branch back to that label
    (the loop may hold forward branches of its own)."""
    best = None
    for i, l in enumerate(lines):
        m = re.match(r"^(\.LBB\d+_\d+):", l)
        if not m:
            continue
        back = re.compile(r"s_c?branch\w*\s+" + re.escape(m.group(1)) + r"\b")
        ends = [j for j in range(i + 1, len(lines)) if back.search(lines[j])]
        if not ends:
            continue
        body = lines[i:ends[-1] + 1]
        if any("v_mfma" in x for x in body) and (best is None or len(body) < len(best)):
            best = body
    return best


class _WideChecker:
    """Callbacks for isa_emu.Emu on one wave of k_lm_head_wide: every hidden_t load inside the M rows, every W_lm load inside
    the buffer, every LDS destination inside the slab buffers; and, with loads completing in issue order, no register
    or LDS block read, and no register loaded again, while a load into it is still in flight after the kernel's waits."""
    H, W, PART, DUMP = 0x1000_0000_0000, 0x2000_0000_0000, 0x3000_0000_0000, 0x4000_0000_0000

    def __init__(self, mb, fp8, M, V, d, nblocks, dump):
        self.mb, self.M, self.V, self.d, self.nblocks, self.dump, self.wb = mb, M, V, d, nblocks, dump, 1 if fp8 else 2
        self.fifo, self.pending_reg, self.pending_lds, self.next_id, self.errors = [], {}, {}, 0, []
        self.loads = 0

    def err(self, msg):
        if len(self.errors) < 5:
            self.errors.append(msg)

    def land(self, allowed):
        while len(self.fifo) > allowed:
            i, kind, regs = self.fifo.pop(0)
            table = self.pending_reg if kind == "W" else self.pending_lds
            for r in regs:
                if table.get(r) == i:
                    del table[r]

    def issue(self, kind, regs):
        table = self.pending_reg if kind == "W" else self.pending_lds
        for r in regs:
            if r in table:
                self.err(f"a load into {'v' if kind == 'W' else 'LDS block '}{r} is issued while an earlier one into it is in flight")
            table[r] = self.next_id
        self.fifo.append((self.next_id, kind, regs))
        self.next_id += 1
        self.loads += 1

    def before(self, e, op, o, t):          # data instructions must not read a register with a load in flight
        if op.startswith("v_mfma"):
            srcs = o[1:3]
        elif op.startswith("v_mov_b32_dpp") or op.startswith("v_cvt_scalef32"):
            srcs = [o[1]]
        else:
            return
        for s_ in srcs:
            if re.match(r"^v(\d+|\[)", s_):
                for r in e.vrange(s_)[1]:
                    if r in self.pending_reg:
                        self.err(f"v{r} is read while a load into it is in flight: {t}")

    def memory(self, e, op, o, t):
        import numpy as np
        if op == "s_waitcnt":
            m = re.search(r"vmcnt\((\d+)\)", t)
            if m:
                self.land(int(m.group(1)))
        elif op == "buffer_load_dwordx4":
            voff, soff = e.vsrc(o[1]), e.sval(o[3])
            m = re.match(r"s\[(\d+):", o[2])
            base, nrec = e.get64(f"s[{int(m.group(1))}:{int(m.group(1)) + 1}]"), e.s.get(f"s{int(m.group(1)) + 2}")
            if voff is None or soff is None or base is None or nrec is None:
                self.err("W_lm load with an unknown address: " + t)
            else:
                off = voff.astype(np.int64) + soff
                if base != self.W or nrec != self.V * self.d * self.wb or off.min() < 0 or off.max() + 16 > nrec:
                    self.err(f"W_lm load outside the buffer (offsets {off.min()}..{off.max()} of {nrec}): {t}")
            self.issue("W", e.vrange(o[0])[1])
        elif op == "global_load_lds_dwordx4":
            voff, base, m0 = e.vsrc(o[0]), e.get64(o[1].split()[0]), e.s.get("m0")
            if voff is None or base is None or m0 is None:
                self.err("hidden_t load with an unknown address: " + t)
                self.issue("H", [])
            else:
                a = base + voff.astype(np.int64)
                if a.min() < self.H or a.max() + 16 > self.H + self.M * self.d * 2:
                    self.err(f"hidden_t load outside the M rows: {t}")
                if m0 < 0 or m0 + 1024 > 4 * self.mb * 16 * 128:
                    self.err(f"LDS destination {m0} outside the slab buffers: {t}")
                self.issue("H", [m0 // 1024])
        elif op == "global_store":
            self.fifo.append((self.next_id, "S", []))
            self.next_id += 1
        elif op in ("scratch_store", "scratch_load"):
            self.fifo.append((self.next_id, "X", []))
            self.next_id += 1
        elif op == "ds_read_b128":
            a = e.vsrc(o[1])
            mm = re.search(r"offset:(\S+)", t)
            imm = int(mm.group(1), 0) if mm else 0
            if a is not None:
                for blk in range((int(a.min()) + imm) // 1024, (int(a.max()) + imm + 15) // 1024 + 1):
                    if blk in self.pending_lds:
                        self.err(f"LDS block {blk} is read while the wave's own load into it is in flight: {t}")


def emulate_wide(lines, mb, fp8, dump, M, V, d, wg, wave):
    """One wave of a compiled k_lm_head_wide through the address emulator; returns (problems, loads issued)."""
    import struct
    from .isa_emu import Emu, Poison
    ntiles = (V + 255) // 256
    grid = min(ntiles, 256)
    c = _WideChecker(mb, fp8, M, V, d, ntiles, dump)
    arg = bytearray(512)                                   # LmHeadArgs, ntiles, then the hidden grid and group sizes
    struct.pack_into("<QQiii", arg, 0, c.H, c.W, M, V, d)
    struct.pack_into("<Qi", arg, 32, c.PART, ntiles)
    struct.pack_into("<QQQQQf", arg, 48, c.DUMP if dump else 0, 0, 0, 0, 0, 1.0)
    struct.pack_into("<i", arg, 112, ntiles)
    struct.pack_into("<III", arg, 120, grid, 1, 1)
    struct.pack_into("<HHH", arg, 132, 256, 1, 1)
    e = Emu(lines, bytes(arg), wg, wave * 64, c.memory, c.before)
    try:
        e.run()
    except Poison as p:
        c.err("emulation stopped: " + str(p))
    return c.errors, c.loads


def check(hipcc, flags, verbose=False):
    problems = []
    with tempfile.TemporaryDirectory() as tmp:
        # ---- lm_head_wide.hip: every instantiation
        asm = os.path.join(tmp, "wide.s")
        subprocess.run([hipcc, *flags, "-S", "--cuda-device-only", "-o", asm, os.path.join(CSRC, "lm_head_wide.hip")],
                       check=True, capture_output=True)
        for name, lines in _kernels(open(asm).read()).items():
            m = re.search(r"k_lm_head_wideILi(\d+)ELb(\d)ELb(\d)ELb(\d)ELb(\d)E", name)
            if not m:
                continue
            mb, fp8 = int(m.group(1)), m.group(2) == "1"
            tag = f"lm_head_wide MB={mb}{' fp8' if fp8 else ''}"
            loop = _innermost_loop(lines)
            if loop is None:
                problems.append(f"{name}: no inner loop found")
                continue
            hl = (2 * mb + 3) // 4
            # a trip of the loop: 4 lines of W_lm = 4 hidden_t slabs (8 with FP8 weights) of 2 pieces of 4 * MB MFMAs
            own = {f"vmcnt({hl + 8})"} if fp8 else {f"vmcnt({2 * hl + 16})", f"vmcnt({hl + 16})"}
            for l in loop:
                if "scratch_" in l or "v_accvgpr" in l:
                    problems.append(f"{tag}: '{l.strip()}' inside the slab loop")
                    break
                w = re.search(r"s_waitcnt\s+(vmcnt\(\d+\))", l)
                # (a wait of the compiler's own costs time, not correctness: the logit dump, a debug path, may have one)
                if w and w.group(1) not in own and m.group(3) != "1":
                    problems.append(f"{tag}: compiler wait '{l.strip()}' inside the slab loop")
                    break
            want = (64 if fp8 else 32) * mb
            if sum("v_mfma" in l for l in loop) != want:
                problems.append(f"{tag}: {sum('v_mfma' in l for l in loop)} MFMAs in the loop, expected {want}")
            # the greedy, top-K and sampling instantiations of the smallest and the largest tile, one wave each of a workgroup
            # with two tiles and of the one with the ragged last tile, through the address emulator
            if mb in (8, 17) and m.group(3) == "0":
                M, V, d = 16 * mb - 8, 66000 + 40, 1024
                for wg, wave in ((0, 1), ((V + 255) // 256 - 1 - 256, 3)):
                    try:
                        errs, loads = emulate_wide(lines, mb, fp8, False, M, V, d, wg, wave)
                    except Exception as ex:      # an instruction the emulator does not know: say so, do not fail the build
                        print(f"check_isa: {tag}: address emulation not done ({ex})")
                        break
                    problems += [f"{tag} (emulated, workgroup {wg} wave {wave}): {x}" for x in errs]
                    if verbose:
                        print(f"check_isa: {tag}: workgroup {wg} wave {wave} emulated, {loads} loads checked")
        # ---- lm_head_pair9.hip: nothing spilled and no accumulator moved inside the k loop (its ninth row block lives
        # in VGPRs next to hand-written MFMAs; the code around the loop may spill)
        asm = os.path.join(tmp, "pair9.s")
        subprocess.run([hipcc, *flags, "-S", "--cuda-device-only", "-o", asm, os.path.join(CSRC, "lm_head_pair9.hip")],
                       check=True, capture_output=True)
        for name, lines in _kernels(open(asm).read()).items():
            if "k_lm_head_pair9ILb0E" not in name:        # every instantiation but the logit dump
                continue
            loop = _innermost_loop(lines)
            if loop is None:
                problems.append(f"{name}: no inner loop found")
                continue
            bad = next((l for l in loop if "scratch_" in l or "v_accvgpr" in l), None)
            if bad:
                problems.append(f"lm_head_pair9 ({name[-40:]}): '{bad.strip()}' inside the k loop")
            if sum("v_mfma" in l for l in loop) != 8 * 36:
                problems.append(f"lm_head_pair9: {sum('v_mfma' in l for l in loop)} MFMAs in the k loop, expected 288")
    if problems:
        raise RuntimeError("generated code of a hand-scheduled kernel is not what it relies on:\n  " + "\n  ".join(problems))
    if verbose:
        print("check_isa: hot loops of lm_head_wide and lm_head_pair9 are clean")
