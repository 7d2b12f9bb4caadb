"""The hand-written cross-lane multiply of the third-moment kernel, checked in the compiled code (no GPU involved).

`mul_bcast` in csrc/st_moment3.hip is a `v_mul_f32_dpp ... row_newbcast` written as inline assembly (the compiler
materialises a broadcast with two users as an extra move).  Inline assembly is opaque to the compiler's hazard
recogniser, and a DPP operand read needs two wait states after a vector-ALU write of the same register.  The
source relies on the operand coming from an LDS load and on an `s_nop 1` in front of the block; this test holds the
compiler to it: the kernel is compiled to gfx950 assembly and every such instruction must have no vector-ALU
instruction that writes its DPP operand among the two instructions in front of it.
"""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"


def _registers(operand):
    """v7 -> {7}; v[4:7] -> {4,5,6,7}; anything else -> empty."""
    m = re.fullmatch(r"v(\d+)", operand)
    if m:
        return {int(m.group(1))}
    m = re.fullmatch(r"v\[(\d+):(\d+)\]", operand)
    if m:
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    return set()


def test_dpp_operand_of_the_inline_multiply_is_not_freshly_written(tmp_path):
    if not os.path.exists(HIPCC):
        pytest.skip("no hipcc")
    asm = str(tmp_path / "st_moment3.s")
    cmd = [HIPCC, "-O3", "-std=c++17", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-I", os.path.join(ROOT, "include"), "-S", "--cuda-device-only",
           os.path.join(ROOT, "paper_2211_10482_amd", "csrc", "st_moment3.hip"), "-o", asm]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    ins = []
    for line in open(asm):
        line = line.split(";")[0].strip()
        if line and not line.startswith(".") and not line.endswith(":"):
            ins.append(line)
    found = 0
    for i, line in enumerate(ins):
        if not (line.startswith("v_mul_f32_dpp") and "row_newbcast" in line):
            continue
        found += 1
        ops = [o.strip() for o in line.split(None, 1)[1].split(",")]
        src = _registers(ops[1])                      # the operand the cross-lane read applies to
        assert src, line
        for prev in ins[max(0, i - 2):i]:
            if not prev.startswith("v_") or prev.startswith("v_cmp") or prev.startswith("v_nop"):
                continue
            dst = _registers(prev.split(None, 1)[1].split(",")[0].strip())
            assert not (dst & src), "vector-ALU write of the DPP operand too close:\n  %s\n  %s" % (prev, line)
    # 32 broadcast products per K-step over the eight per-wave code streams, four K-steps each, two template instances
    assert found >= 32 * 4, "the inline multiply was not found in the compiled kernel (%d)" % found
