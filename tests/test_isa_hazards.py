"""Generated gfx950 code: no matrix instruction may read a register that an inline-assembly
instruction has just written.

The compiler keeps two wait states between a vector instruction that writes a VGPR and a matrix (MFMA)
instruction that reads it, but it cannot see into inline assembly: a `v_...` written as asm right in
front of an MFMA that consumes its result is issued with too few wait states, and a wave that has its
SIMD to itself then multiplies stale operands (seen once in the few-token kernel; its dequantisation is
plain C since).  The tiled kernel still forms its `v_and_or_b32` in assembly -- safe because that result
never reaches a matrix instruction.  This test compiles the kernels to assembly text (no GPU needed)
and checks exactly that, with a margin."""
import os
import re
import shutil
import subprocess
from concurrent.futures import ThreadPoolExecutor

import pytest

from paper_2406_02913_amd import build as szo_build

WINDOW = 4          # wait states looked back from every matrix instruction (the hardware rule needs 2)


def _regs(tok):
    m = re.match(r"([va])\[(\d+):(\d+)\]$", tok)
    if m:
        return {(m.group(1), i) for i in range(int(m.group(2)), int(m.group(3)) + 1)}
    m = re.match(r"([va])(\d+)$", tok)
    return {(m.group(1), int(m.group(2)))} if m else set()


def asm_results_read_by_mfma(text):
    """[(kernel, asm instruction, mfma instruction, wait states between)] for every matrix instruction
    that reads a register written by an inline-assembly instruction fewer than WINDOW wait states before."""
    found, kernel, hist, in_asm = [], None, [], False
    for line in text.splitlines():
        t = line.strip()
        m = re.match(r"^(\w+):", line)
        if m and not line.startswith("."):
            kernel, hist = m.group(1), []
            continue
        if "ASMSTART" in t:
            in_asm = True
            continue
        if "ASMEND" in t:
            in_asm = False
            continue
        if not t or t[0] in ";." or t.endswith(":"):
            continue
        parts = t.split(None, 1)
        op = parts[0]
        ops = [o.strip() for o in parts[1].split(",")] if len(parts) > 1 else []
        if op.startswith("v_mfma"):
            src = set().union(*[_regs(o) for o in ops[1:]])
            wait = 0
            for h_op, h_ops, h_asm, h_text in reversed(hist):
                if wait >= WINDOW:
                    break
                if h_asm and h_op.startswith("v_") and h_ops and (_regs(h_ops[0]) & src):
                    found.append((kernel, h_text, t, wait))
                wait += 1 + (int(h_ops[0], 0) if h_op == "s_nop" and h_ops else 0)
        hist.append((op, ops, in_asm, t))
        del hist[:-16]
    return found


def test_the_checker_sees_a_planted_hazard():
    planted = """
kern:
	v_mfma_f32_16x16x32_f16 a[0:3], v[4:7], v[8:11], a[0:3]
	;;#ASMSTART
	v_and_or_b32 v9, v20, s2, v21
	;;#ASMEND
	v_lshrrev_b32_e32 v30, 8, v31
	v_mfma_f32_16x16x32_f16 a[0:3], v[4:7], v[8:11], a[0:3]
	s_endpgm
"""
    hits = asm_results_read_by_mfma(planted)
    assert len(hits) == 1 and hits[0][0] == "kern" and hits[0][3] == 1
    # the same instruction outside an assembly block is the compiler's business, and far enough away it is fine
    assert asm_results_read_by_mfma(planted.replace(";;#ASMSTART", "").replace(";;#ASMEND", "")) == []
    assert asm_results_read_by_mfma(planted.replace("v_lshrrev_b32_e32 v30, 8, v31", "s_nop 3")) == []
    # an empty assembly statement (a register pin) writes nothing
    assert asm_results_read_by_mfma("k:\n;;#ASMSTART\n;;#ASMEND\nv_mfma_f32_16x16x32_f16 a[0:3], v[4:7], v[8:11], a[0:3]\n") == []


@pytest.mark.skipif(not (os.path.exists(szo_build.HIPCC) or shutil.which("hipcc")), reason="no hipcc")
def test_no_matrix_instruction_reads_an_inline_assembly_result(tmp_path):
    hipcc = szo_build.HIPCC if os.path.exists(szo_build.HIPCC) else shutil.which("hipcc")

    def to_asm(src):
        out = str(tmp_path / (src + ".s"))
        subprocess.check_call([hipcc, "--cuda-device-only", "-S"] + szo_build.COMMON + szo_build.DEVICE +
                              [os.path.join(szo_build.CSRC, src), "-o", out], stderr=subprocess.DEVNULL)
        return open(out).read()

    with ThreadPoolExecutor(max_workers=3) as pool:
        texts = list(pool.map(to_asm, szo_build.HIP_SOURCES))
    for src, text in zip(szo_build.HIP_SOURCES, texts):
        assert "s_endpgm" in text
        hits = asm_results_read_by_mfma(text)
        assert not hits, (src, hits[:3])
    # the kernels this is about are really in there, matrix instructions included
    assert sum(t.count("v_mfma_f32_32x32x16") for t in texts) > 100 and sum(t.count("v_mfma_f32_16x16x32") for t in texts) > 100
