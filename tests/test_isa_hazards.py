"""Static check of this library's own generated gfx950 code for one measured hardware hazard.

On MI355X a ``v_mfma_f32_16x16x16_bf16`` whose accumulator input (SrcC) is the result of a
``v_mfma_f32_16x16x32_bf16`` issued fewer than 5 wait states earlier reads the registers' OLD contents (a probe
with both instructions in one asm block showed it; 5 or more wait states, the opposite order, and two products of
one shape are fine).  The kernels are written so that this dependent pair never occurs (every 16x16x16 product
accumulates onto zero or onto another 16x16x16 result), but nothing in the language stops a later edit or compiler
from producing it.  This test compiles the translation units that use both shapes to assembly and fails if the
pair appears closer than that, so the property is checked on every build instead of resting on source order."""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2503_01868_amd", "csrc")
SAFE_WAIT_STATES = 5

MFMA = re.compile(r"^\s*(v_mfma_f32_(\d+x\d+x\d+)\w*)\s+([av])\[(\d+):(\d+)\],\s*([^,]+),\s*([^,]+),\s*(.+?)\s*(?:;.*)?$")
REG = re.compile(r"([av])\[(\d+):(\d+)\]")


def assemble(src, tmp_path):
    hipcc = "/opt/rocm/bin/hipcc" if os.path.exists("/opt/rocm/bin/hipcc") else shutil.which("hipcc")
    if not hipcc:
        pytest.skip("hipcc not available")
    out = str(tmp_path / (os.path.basename(src) + ".s"))
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-I" + os.path.join(ROOT, "include"), "-I" + CSRC, "-S", "--cuda-device-only", src, "-o", out]
    proc = subprocess.run(cmd, capture_output=True, text=True)
    assert proc.returncode == 0, proc.stderr[-2000:]
    return open(out).read().splitlines()


def hazards(lines):
    """(line number, text) of every 16x16x16 product that takes a 16x16x32 result as SrcC within the unsafe distance."""
    found = []
    recent = []  # (wait states since issue, register file, lo, hi) of recent 16x16x32 results
    n_mfma = {"16x16x32": 0, "16x16x16": 0}
    for no, line in enumerate(lines, 1):
        text = line.split(";")[0].strip()
        if not text or text.startswith(".") or text.startswith("//"):
            continue
        if text.endswith(":"):  # a label: control flow may join here, forget what was in flight
            recent = []
            continue
        cost = 1
        m_nop = re.match(r"s_nop\s+(\d+)", text)
        if m_nop:
            cost = int(m_nop.group(1)) + 1
        m = MFMA.match(text)
        if m:
            shape = m.group(2)
            if shape in n_mfma:
                n_mfma[shape] += 1
            if shape == "16x16x16":
                c = REG.match(m.group(8).strip())
                if c:
                    for age, rf, lo, hi in recent:
                        if age < SAFE_WAIT_STATES and rf == c.group(1) and not (int(c.group(3)) < lo or int(c.group(2)) > hi):
                            found.append((no, text))
        recent = [(age + cost, rf, lo, hi) for age, rf, lo, hi in recent if age + cost < 16]
        if m and m.group(2) == "16x16x32":
            recent.append((0, m.group(3), int(m.group(4)), int(m.group(5))))
    return found, n_mfma


def test_the_checker_sees_a_planted_pair_and_accepts_a_distant_one():
    bad = ["v_mfma_f32_16x16x32_bf16 v[0:3], v[4:7], v[8:11], v[0:3]", "v_mov_b32 v20, v21",
           "v_mfma_f32_16x16x16_bf16 v[0:3], v[12:13], v[14:15], v[0:3]"]
    assert len(hazards(bad)[0]) == 1
    ok = [bad[0], "s_nop 4", bad[2]]
    assert hazards(ok)[0] == []
    other_regs = [bad[0], "v_mfma_f32_16x16x16_bf16 v[0:3], v[12:13], v[14:15], v[16:19]"]
    assert hazards(other_regs)[0] == []
    reverse = ["v_mfma_f32_16x16x16_bf16 v[0:3], v[12:13], v[14:15], 0", "v_mfma_f32_16x16x32_bf16 v[0:3], v[4:7], v[8:11], v[0:3]"]
    assert hazards(reverse)[0] == []


@pytest.mark.parametrize("unit", ["li_kernels.hip", "mr_bwd_kernels.hip"])
def test_no_short_product_accumulates_onto_a_fresh_long_product(unit, tmp_path):
    lines = assemble(os.path.join(CSRC, unit), tmp_path)
    found, n = hazards(lines)
    assert n["16x16x32"] > 0 and n["16x16x16"] > 0, n  # the unit really uses both shapes (else the check is vacuous)
    assert not found, found[:5]
