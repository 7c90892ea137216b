"""Compile libspd.so (HIP kernels + host library) for gfx950, in-tree."""
from __future__ import annotations

import os
import shutil
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libspd.so")
SOURCES = ["spd_kernels.hip", "spd_fused.hip", "spd_sampler.hip", "spd_prefill.hip", "spd_lib.cpp", "ngram_table.cpp"]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found")
    return exe


def build_library(verbose: bool = False, out: str = LIB) -> str:
    """Always recompiles.  -ffp-contract=off: the kernels spell out every fused
    multiply-add they want; packed-fp32 instruction selection is disabled."""
    cmd = [hipcc(), "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
           "-ffp-contract=off", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wno-unused-command-line-argument",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-x", "hip"]
    cmd += os.environ.get("SPD_EXTRA_DEFS", "").split()      # experiments only, e.g. -DSPD_FUSED_NT=512
    cmd += [os.path.join(CSRC, s) for s in SOURCES]
    cmd += ["-o", out]
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    log = "\n".join(l for l in (res.stdout + res.stderr).splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + log)
    if verbose and log.strip():
        print(log)
    return out


if __name__ == "__main__":
    print(build_library(verbose=True))
