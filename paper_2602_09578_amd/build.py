"""Builds libmarl_decode.so for gfx950 with hipcc, in-tree (paper_2602_09578_amd/lib/)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

_PKG = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_PKG)
CSRC = os.path.join(_PKG, "csrc")
LIB_DIR = os.path.join(_PKG, "lib")
LIB_PATH = os.path.join(LIB_DIR, "libmarl_decode.so")
SOURCES = ["api.hip", "plan_kernel.hip", "attn_kernels.hip", "logprob_kernels.hip",
           "kv_cache_kernels.hip", "sample_kernels.hip", "grpo_kernels.hip", "prefill_kernels.hip", "balancer.hip", "pack_kernels.hip", "page_pool.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I" + os.path.join(_ROOT, "include"), "-I" + CSRC]
# Device code of these files never produces or consumes a NaN in floating-point arithmetic
# (masked scores are -inf, unused value slots are cleared as integers), so the compiler may drop
# the canonicalising v_max it otherwise puts in front of every maximum of a matrix-core result:
# the vector ALU is the busiest unit of the attention kernels.  Host code keeps its NaN checks.
_NO_NANS = ["-Xarch_device", "-fno-honor-nans"]
FILE_FLAGS = {"prefill_kernels.hip": _NO_NANS, "attn_kernels.hip": _NO_NANS}


def build_library(verbose: bool = False, extra_flags=(), out_path: str = LIB_PATH) -> str:
    """Compiles every source (always, also when a built library exists) and links."""
    os.makedirs(LIB_DIR, exist_ok=True)
    objdir = os.path.join(LIB_DIR, "_build", os.path.basename(out_path))
    os.makedirs(objdir, exist_ok=True)

    def compile_one(src):
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        cmd = [HIPCC, *FLAGS, *FILE_FLAGS.get(src, []), *extra_flags, "-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        out = "\n".join(l for l in r.stdout.splitlines() if "not a recognized feature" not in l)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed for {src}:\n{out}")
        if verbose and out.strip():
            print(out)
        return obj

    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", out_path, *objs]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout)
    return out_path


if __name__ == "__main__":
    print(build_library(verbose=True, extra_flags=sys.argv[1:]))
