"""Static check of the generated gfx950 assembly (CPU only, needs hipcc).

The pipelined and the decode kernels issue their MFMAs through inline assembly, so the compiler
does not add the wait states the hardware needs between a vector instruction
that writes a VGPR/AccVGPR and an MFMA that reads it (two wait states on this
family), nor does it know that a vector instruction which reads an MFMA's result
has to wait until the MFMA has finished.  This test compiles the kernels to assembly
and verifies (1) that none of the two instructions in front of any MFMA is a
vector-ALU write to one of the MFMA's source registers, and (2) that no instruction
other than an MFMA reads an MFMA's destination registers within kResultWait wait
states after it, along every path of the control flow.  Both kernels address LDS with absolute byte addresses, so
they must not own any static LDS either.
"""
import os
import re
import shutil
import subprocess

import pytest

from paper_2512_10411_amd import build

# source file, substring of the kernel that addresses LDS absolutely, fewest MFMAs expected
CASES = [("swaa_fwd_pipelined.hip", "pipelined", 60), ("swaa_decode.hip", "decode_split", 16),
         ("swaa_bwd_dq_pipelined.hip", "dq_pipelined", 100)]


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


# wait states after an MFMA before its result may be touched (the 8-pass MFMAs used here
# need 11; the kernels wait 24); an MFMA in between counts as kMfmaIssue, since the matrix
# pipe takes MFMAs in order and finishes each before the one after next starts
kResultWait = 18
kMfmaIssue = 8


def reads_and_writes(op, ops):
    """(registers read, registers written) of a non-MFMA instruction, conservatively."""
    if not ops:
        return set(), set()
    all_regs = set().union(*[reg_set(t) for t in ops])
    store_like = op.startswith(("ds_write", "global_store", "buffer_store", "scratch_store", "v_cmp", "global_load_lds",
                                "v_readfirstlane", "v_readlane"))
    read_modify_write = op.startswith(("v_fmac", "v_mac", "v_permlane", "v_pk_fmac", "v_dot2c", "v_writelane"))
    if store_like:
        return all_regs, set()
    dst = reg_set(ops[0])
    if read_modify_write:
        return all_regs, dst
    return set().union(*[reg_set(t) for t in ops[1:]]) if len(ops) > 1 else set(), dst


def result_hazards(insts, labels):
    """Rule (2): [(mfma, offender)] over all paths within the wait window.  A register that
    another instruction overwrites first no longer holds the MFMA's result and is dropped."""
    problems = []

    def walk(j, dst, ws, mfma, depth):
        dst = set(dst)
        while ws < kResultWait and j < len(insts) and dst:
            op, ops = insts[j]
            if op == "s_endpgm":
                return
            if op.startswith("v_mfma"):
                ws += kMfmaIssue
            elif op == "s_nop":
                ws += int(ops[0]) + 1
            elif op == "s_branch":
                j = labels[ops[0]]
                ws += 1
                continue
            elif op.startswith("s_cbranch"):
                if depth < 4:
                    walk(labels[ops[0]], dst, ws + 1, mfma, depth + 1)
                ws += 1
            else:
                reads, writes = reads_and_writes(op, ops)
                if reads & dst:
                    problems.append((mfma, insts[j]))
                    return
                dst -= writes
                ws += 1
            j += 1

    for i, (op, ops) in enumerate(insts):
        if op.startswith("v_mfma"):
            walk(i + 1, reg_set(ops[0]), 0, insts[i], 0)
    return problems


def is_valu_write(op):
    return op.startswith("v_") and not op.startswith("v_mfma") and not op.startswith("v_cmp") and \
        not op.startswith("v_nop")


@pytest.mark.skipif(shutil.which("hipcc") is None and not os.path.exists("/opt/rocm/bin/hipcc"),
                    reason="hipcc not available")
@pytest.mark.parametrize("src,kernel,min_mfma", CASES)
def test_no_vector_write_within_two_instructions_of_an_mfma_that_reads_it(tmp_path, src, kernel, min_mfma):
    SRC = os.path.join(build.CSRC, src)
    out = tmp_path / "k.s"
    flags = [f for f in build.HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    cmd = [build.hipcc_path(), *flags, "--cuda-device-only", "-S", "-o", str(out), SRC]
    subprocess.run(cmd, check=True, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
    text = open(out).read()
    # the kernel addresses LDS absolutely, so its dynamic LDS must start at address 0
    sizes = re.findall(r"\.amdhsa_group_segment_fixed_size\s+(\d+)", text)
    names = re.findall(r"\.amdhsa_kernel\s+(\S+)", text)
    assert names and len(sizes) == len(names)
    for name, size in zip(names, sizes):
        if kernel in name:
            assert int(size) == 0, (name, size)
    assert any(kernel in name for name in names)
    insts, labels = [], {}
    for ln in text.splitlines():
        m = re.match(r"^(\.LBB\d+_\d+):", ln)
        if m:
            labels[m.group(1)] = len(insts)
        p = parse(ln)
        if p:
            insts.append(p)
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
    assert n_mfma >= min_mfma, "expected the MFMA kernel in the assembly"
    assert not problems, problems[:5]
    late = result_hazards(insts, labels)
    assert not late, late[:5]


@pytest.mark.skipif(shutil.which("hipcc") is None and not os.path.exists("/opt/rocm/bin/hipcc"),
                    reason="hipcc not available")
def test_backward_dma_kernels_own_all_lds(tmp_path):
    """The LDS-DMA dK/dV kernel addresses LDS with plain byte addresses from 0 (its MFMAs go
    through compiler builtins, so the wait-state rules above are the compiler's)."""
    out = tmp_path / "b.s"
    flags = [f for f in build.HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    cmd = [build.hipcc_path(), *flags, "--cuda-device-only", "-S", "-o", str(out), os.path.join(build.CSRC, "swaa_bwd.hip")]
    subprocess.run(cmd, check=True, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
    text = open(out).read()
    sizes = re.findall(r"\.amdhsa_group_segment_fixed_size\s+(\d+)", text)
    names = re.findall(r"\.amdhsa_kernel\s+(\S+)", text)
    assert names and len(sizes) == len(names)
    seen = set()
    for name, size in zip(names, sizes):
        for k in ("dkv_dma",):
            if k in name:
                seen.add(k)
                assert int(size) == 0, (name, size)
    assert seen == {"dkv_dma"}
    # and they do not spill (a spill would also mean scratch traffic inside the key loop)
    for name, spill in zip(names, re.findall(r"\.amdhsa_private_segment_fixed_size\s+(\d+)", text)):
        if "dma" in name:
            assert int(spill) == 0, (name, spill)
