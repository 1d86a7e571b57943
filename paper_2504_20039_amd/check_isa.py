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
