"""Host-side check of the compiled 64-row prefill kernel.

Its matrix instructions are inline assembly, so the compiler's hazard recognizer does not see them:
a vector instruction that writes a register needs two wait states before a matrix instruction reads
that register as an A or B operand, and nothing inserts them.  The kernel is written so that no such
operand is produced right in front of its consumer (fragments arrive from LDS behind a wait, weights
are packed a slot earlier, constants are pinned in registers); this test compiles the kernel to
assembly and verifies that on the instruction stream, and that nothing was spilled to scratch memory.
"""
import re
import shutil
import subprocess
from pathlib import Path

import pytest

from paper_2501_13629_amd import build

SRC = build.CSRC / "prefill_mfma64.hip"


def _registers(text):
    out = set()
    for m in re.finditer(r"\b([av])(\d+)\b", text):
        out.add((m.group(1), int(m.group(2))))
    for m in re.finditer(r"\b([av])\[(\d+):(\d+)\]", text):
        for r in range(int(m.group(2)), int(m.group(3)) + 1):
            out.add((m.group(1), r))
    return out


def _operands(text):
    parts, cur, depth = [], "", 0
    for ch in text:
        depth += ch == "["
        depth -= ch == "]"
        if ch == "," and depth == 0:
            parts.append(cur)
            cur = ""
        else:
            cur += ch
    return parts + [cur]


@pytest.fixture(scope="module")
def assembly(tmp_path_factory):
    hipcc = build._hipcc()
    if shutil.which(hipcc) is None and not Path(hipcc).exists():
        pytest.skip("no hipcc")
    out = tmp_path_factory.mktemp("codegen") / "prefill_mfma64.s"
    flags = [f for f in build.HIPCC_FLAGS if f != "-fPIC"]
    r = subprocess.run([hipcc, *flags, "-I", str(build.INCLUDE), "-S", "--cuda-device-only", str(SRC), "-o", str(out)],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    return out.read_text().split("\n")


def test_nothing_is_spilled(assembly):
    sizes = [int(l.split(":")[1]) for l in assembly if l.startswith("; ScratchSize:")]
    assert sizes and max(sizes) == 0
    agprs = [int(l.split(":")[1]) for l in assembly if l.startswith("; NumAgprs:")]
    assert agprs and max(agprs) <= 256


def test_no_vector_write_right_before_a_matrix_instruction_reads_it(assembly):
    code, in_asm = [], False  # (line number, instruction text, from inline assembly)
    for i, line in enumerate(assembly):
        if "ASMSTART" in line:
            in_asm = True
            continue
        if "ASMEND" in line:
            in_asm = False
            continue
        text = line.split(";")[0].strip()
        if text and not text.startswith(".") and not text.endswith(":"):
            code.append((i + 1, text, in_asm))
    n_matrix, bad = 0, []
    for k, (ln, text, from_asm) in enumerate(code):
        if not (from_asm and text.startswith("v_mfma")):
            continue
        n_matrix += 1
        ops = _operands(text.split(None, 1)[1])
        sources = _registers(ops[1]) | _registers(ops[2])  # A and B (the accumulator has its own explicit nops)
        wait_states, j = 0, k - 1
        while j >= 0 and wait_states < 2:
            _, prev, prev_asm = code[j]
            j -= 1
            if prev.startswith("s_nop"):
                wait_states += int(prev.split()[1]) + 1
                continue
            wait_states += 1
            if not prev_asm and prev.startswith("v_") and not prev.startswith("v_cmp") and " " in prev:
                if _registers(_operands(prev.split(None, 1)[1])[0]) & sources:
                    bad.append((ln, prev))
    assert n_matrix >= 64, "the matrix instructions were not found"
    assert not bad, bad[:5]
