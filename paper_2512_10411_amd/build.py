"""Builds libswaa.so (HIP, gfx950 only) in-tree with hipcc.

    python -m paper_2512_10411_amd.build
"""
from __future__ import annotations

import os
import shutil
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
SOURCES = [os.path.join(CSRC, f) for f in ("swaa_api.hip", "swaa_fwd_simple.hip", "swaa_fwd_pipelined.hip",
                                            "swaa_decode.hip", "swaa_bwd.hip", "swaa_bwd_dq_pipelined.hip")]
LIB = os.path.join(PKG, "libswaa.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Wall", "-Wno-unused-value",
    # packed fp32 VALU forms are kept out of the generated code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # S^T accumulators of the builtin MFMAs land in VGPRs (the softmax reads them
    # with vector instructions); the O^T accumulators are pinned to AccVGPRs by hand
    "-mllvm", "-amdgpu-mfma-vgpr-form",
    # no NaN-quieting copies in front of every v_max; the kernels never rely on NaN semantics
    "-fno-honor-nans",
    "-I", os.path.join(ROOT, "include"), "-I", os.path.join(PKG, "csrc"),
]


def hipcc_path() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found: libswaa.so cannot be built")
    return exe


def build_library(verbose: bool = False, extra_flags=(), out: str = LIB) -> str:
    """Compile every HIP source into paper_2512_10411_amd/libswaa.so (or `out`)."""
    tmp = out + ".tmp.%d" % os.getpid()
    cmd = [hipcc_path(), *HIPCC_FLAGS, *extra_flags, "-o", tmp, *SOURCES]
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout)
    if verbose and res.stdout.strip():
        # the host pass warns that it does not know the packed-fp32 feature: harmless
        print("\n".join(ln for ln in res.stdout.splitlines() if "packed-fp32-ops" not in ln))
    os.replace(tmp, out)
    return out


if __name__ == "__main__":
    print(build_library(verbose=True))
