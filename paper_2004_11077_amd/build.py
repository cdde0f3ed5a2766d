"""Builds libwino.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree.

    python -m paper_2004_11077_amd.build

Objects go to ``_build/`` at the repository root (not committed); the shared
library lands beside this file so that it travels with the source tree.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(ROOT, "_build")
LIB = os.path.join(HERE, "libwino.so")

HIP_SOURCES = ["wino_kernels.hip", "wino_transforms_f2.hip", "wino_transforms_f4.hip",
               "wino_transforms_f6.hip", "wino_fp32.hip", "wino_fused.hip", "wino_noalloc.hip", "wino_conout_f2.hip", "wino_conout_f4.hip", "wino_conout_f6.hip",
               "wino_calibrate_f2.hip", "wino_calibrate_f4.hip", "wino_calibrate_f6.hip",
               "wino_flex_f2.hip", "wino_flex_f4.hip", "wino_flex_f6.hip",
               "wino_backward.hip", "wino_flex_backward_f2.hip", "wino_flex_backward_f4.hip",
               "wino_flex_backward_f6.hip"]
CXX_SOURCES = ["wino_api.cpp"]

COMMON = ["-std=c++20", "-fPIC", "-fconstexpr-steps=200000000", "-Wall", "-Wno-unused-function"]
# -ffp-contract=off: the only fused multiply-adds are the ones written out (the
# casts); the fp32 brackets of the flex kernels round every product and sum.
# Packed fp32 VALU forms are disabled for the device pass.
# -amdgpu-mfma-vgpr-form: MFMA accumulators live in ordinary vector registers, so the
# epilogues read them directly instead of copying them out of the accumulation file.
DEVICE = ["-O3", "--offload-arch=gfx950", "-ffp-contract=off",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-mllvm", "-amdgpu-mfma-vgpr-form"]


# host-only translation units still see the HIP runtime API declarations
HOST = ["-O2", "-x", "c++", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include"]


def _run(cmd):
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in proc.stdout.splitlines()
                    if "packed-fp32-ops" not in l)
    if proc.returncode != 0:
        raise RuntimeError("command failed: %s\n%s" % (" ".join(cmd), out))
    return out


def _stale(obj, deps):
    if not os.path.exists(obj):
        return True
    t = os.path.getmtime(obj)
    return any(os.path.getmtime(d) > t for d in deps)


def build(force=True, jobs=None, verbose=True):
    """Compile every source and link libwino.so.  ``force=False`` skips
    objects newer than all sources and headers."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    headers = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith((".hpp", ".h"))]
    headers.append(os.path.join(ROOT, "include", "wino.h"))
    tasks = []
    objs = []
    for src in HIP_SOURCES + CXX_SOURCES:
        path = os.path.join(CSRC, src)
        obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
        objs.append(obj)
        if force or _stale(obj, [path] + headers):
            flags = COMMON + (DEVICE if src.endswith(".hip") else HOST)
            tasks.append([hipcc] + flags + ["-c", path, "-o", obj])
    jobs = jobs or min(len(tasks), os.cpu_count() or 1) or 1
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        for out in ex.map(_run, tasks):
            if verbose and out.strip():
                print(out)
    if tasks or not os.path.exists(LIB):
        _run([hipcc, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(force="--incremental" not in sys.argv)
