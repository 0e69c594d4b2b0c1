"""Builds paper_2407_13218_amd/liblinr.so (HIP kernels + C ABI) for gfx950 with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "liblinr.so")
SOURCES = [os.path.join(HERE, "csrc", "linr_kernels.hip"), os.path.join(HERE, "csrc", "linr_kernels_select.hip"),
           os.path.join(HERE, "csrc", "linr_api.cpp")]
DEPS = SOURCES + [os.path.join(HERE, "csrc", "linr_internal.h"), os.path.join(HERE, "csrc", "linr_device.h"), os.path.join(ROOT, "include", "linr.h")]


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile for gfx950.  Packed-fp32 instruction selection is switched off."""
    if not force and os.path.exists(LIB) and all(os.path.getmtime(LIB) >= os.path.getmtime(s) for s in DEPS):
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB + f".tmp{os.getpid()}"
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-I" + os.path.join(ROOT, "include"),
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-mllvm", "-amdgpu-mfma-vgpr-form",     # matrix results straight into VGPRs (no AGPR copies)
           "-o", tmp] + SOURCES
    if verbose:
        cmd.insert(1, "-Rpass-analysis=kernel-resource-usage")
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stderr)
        raise RuntimeError("hipcc failed")
    if verbose:
        sys.stderr.write(res.stderr)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
