"""Builds paper_2407_13218_amd/liblinr.so (HIP kernels + C ABI) for gfx950 with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "liblinr.so")
CSRC = os.path.join(HERE, "csrc")
SOURCES = [os.path.join(CSRC, f) for f in ("linr_kernels.hip", "linr_kernels_dense.hip", "linr_kernels_dense_bf16.hip", "linr_kernels_select.hip", "linr_api.cpp")]
HEADERS = [os.path.join(CSRC, f) for f in ("linr_internal.h", "linr_device.h", "linr_scan_common.h", "linr_dense.h")] + \
          [os.path.join(ROOT, "include", "linr.h")]
DEPS = SOURCES + HEADERS + [os.path.join(CSRC, "mfma_issue_bench.hip")]
ISSUE_BENCH = os.path.join(HERE, "mfma_issue_bench")  # executable (git-ignored, like the library)
OBJDIR = os.path.join(HERE, "_build")          # object files (git-ignored); only the linked library ships


def _flags(extra=()):
    return ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-I" + os.path.join(ROOT, "include"),
            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",      # no packed-fp32 instruction selection
            "-mllvm", "-amdgpu-mfma-vgpr-form"] + list(extra)                 # matrix results straight into VGPRs


def build(force: bool = True, verbose: bool = False, defines=()) -> str:
    """Compile every translation unit for gfx950 (in parallel), then link the shared object."""
    if not force and os.path.exists(LIB) and all(os.path.getmtime(LIB) >= os.path.getmtime(s) for s in DEPS):
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJDIR, exist_ok=True)
    newest_header = max(os.path.getmtime(h) for h in HEADERS)
    extra = ["-D" + d for d in defines] + (["-Rpass-analysis=kernel-resource-usage"] if verbose else [])

    def compile_one(src):
        obj = os.path.join(OBJDIR, os.path.basename(src) + ".o")
        if not force and os.path.exists(obj) and os.path.getmtime(obj) >= max(os.path.getmtime(src), newest_header):
            return obj, ""
        res = subprocess.run([hipcc] + _flags(extra) + ["-c", src, "-o", obj], capture_output=True, text=True)
        if res.returncode != 0:
            sys.stderr.write(res.stderr)
            raise RuntimeError(f"hipcc failed on {os.path.basename(src)}")
        return obj, res.stderr

    with ThreadPoolExecutor(max_workers=min(5, len(SOURCES))) as pool:
        results = list(pool.map(compile_one, SOURCES))
    if verbose:
        for _, err in results:
            sys.stderr.write(err)
    tmp = LIB + f".tmp{os.getpid()}"
    res = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + [o for o, _ in results],
                         capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stderr)
        raise RuntimeError("link failed")
    os.replace(tmp, LIB)
    # stand-alone micro-benchmark of the matrix / vector issue model the large-batch kernel is designed around
    res = subprocess.run([hipcc] + _flags() + [os.path.join(CSRC, "mfma_issue_bench.hip"), "-o", ISSUE_BENCH], capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stderr)
        raise RuntimeError("hipcc failed on mfma_issue_bench.hip")
    return LIB


if __name__ == "__main__":
    print(build(force="-f" in sys.argv or "--incremental" not in sys.argv, verbose="-v" in sys.argv))
