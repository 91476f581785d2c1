"""The divisions by launch constants in every kernel's work-item decode are multiplications by
host-made magic numbers (csrc/swaa_common.h, FastDiv).  A host program built from the same header
checks them against the machine's division: all divisors up to 2^16 at the numerators where a wrong
multiplier shows first, and four million random (numerator, divisor) pairs below 2^31.  No GPU."""
import os
import shutil
import subprocess

import pytest

from paper_2512_10411_amd import build

HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.mark.skipif(shutil.which("hipcc") is None and not os.path.exists("/opt/rocm/bin/hipcc"),
                    reason="hipcc not available")
def test_magic_number_division_is_exact_below_two_to_the_31(tmp_path):
    exe = tmp_path / "fastdiv_check"
    cmd = [build.hipcc_path(), "--offload-arch=gfx950", "-O2", "-std=c++17", "-I", build.CSRC,
           "-I", os.path.join(os.path.dirname(HERE), "include"), "-o", str(exe),
           os.path.join(HERE, "host_checks", "fastdiv_check.hip")]
    subprocess.run(cmd, check=True, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
    res = subprocess.run([str(exe)], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    print(res.stdout)
    assert res.returncode == 0, res.stdout
    assert " 0 wrong" in res.stdout
