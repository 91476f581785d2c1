"""Static check of the generated gfx950 assembly (CPU only, needs hipcc).

The pipelined kernel issues its MFMAs through inline assembly, so the compiler
does not add the wait states the hardware needs between a vector instruction
that writes a VGPR/AccVGPR and an MFMA that reads it (two wait states on this
family).  This test compiles the kernel to assembly and verifies that none of
the two instructions in front of any MFMA is a vector-ALU write to one of the
MFMA's source registers.
"""
import os
import re
import shutil
import subprocess

import pytest

from paper_2512_10411_amd import build

SRC = os.path.join(build.CSRC, "swaa_fwd_pipelined.hip")


def reg_set(tok):
    """'v[4:7]' -> {('v',4),...}; 'a12' -> {('a',12)}; others -> empty."""
    m = re.fullmatch(r"([va])\[(\d+):(\d+)\]", tok)
    if m:
        return {(m.group(1), i) for i in range(int(m.group(2)), int(m.group(3)) + 1)}
    m = re.fullmatch(r"([va])(\d+)", tok)
    if m:
        return {(m.group(1), int(m.group(2)))}
    return set()


def parse(line):
    line = line.split(";")[0].strip()
    if not line or line.endswith(":") or line.startswith("."):
        return None
    parts = line.split(None, 1)
    op = parts[0]
    ops = [t.strip() for t in parts[1].split(",")] if len(parts) > 1 else []
    return op, ops


def is_valu_write(op):
    return op.startswith("v_") and not op.startswith("v_mfma") and not op.startswith("v_cmp") and \
        not op.startswith("v_nop")


@pytest.mark.skipif(shutil.which("hipcc") is None and not os.path.exists("/opt/rocm/bin/hipcc"),
                    reason="hipcc not available")
def test_no_vector_write_within_two_instructions_of_an_mfma_that_reads_it(tmp_path):
    out = tmp_path / "k.s"
    flags = [f for f in build.HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    cmd = [build.hipcc_path(), *flags, "--cuda-device-only", "-S", "-o", str(out), SRC]
    subprocess.run(cmd, check=True, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
    text = open(out).read()
    # the pipelined kernel addresses LDS absolutely, so it must own all of it
    sizes = re.findall(r"\.amdhsa_group_segment_fixed_size\s+(\d+)", text)
    names = re.findall(r"\.amdhsa_kernel\s+(\S+)", text)
    assert names and len(sizes) == len(names)
    for name, size in zip(names, sizes):
        if "pipelined" in name:
            assert int(size) == 0, (name, size)
    insts = [p for p in (parse(ln) for ln in text.splitlines()) if p]
    n_mfma = 0
    problems = []
    for i, (op, ops) in enumerate(insts):
        if not op.startswith("v_mfma"):
            continue
        n_mfma += 1
        srcs = set().union(*[reg_set(t) for t in ops[1:]])
        wait_states = 0
        for back in (1, 2, 3):
            if i - back < 0 or wait_states >= 2:
                break
            pop, pops = insts[i - back]
            if pop == "s_nop":
                wait_states += int(pops[0]) + 1
                continue
            if is_valu_write(pop) and pops and (reg_set(pops[0]) & srcs):
                problems.append((insts[i - back], insts[i]))
            wait_states += 1
    assert n_mfma >= 60, "expected the MFMA-heavy kernel in the assembly"
    assert not problems, problems[:5]
