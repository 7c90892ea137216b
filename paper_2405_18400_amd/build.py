"""Compile libspd.so (HIP kernels + host library) for gfx950, in-tree."""
from __future__ import annotations

import os
import shutil
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libspd.so")
SOURCES = ["spd_kernels.hip", "spd_fused.hip", "spd_sampler.hip", "spd_prefill.hip", "spd_noalloc.hip", "spd_lib.cpp", "ngram_table.cpp"]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found")
    return exe


def build_library(verbose: bool = False, out: str = LIB) -> str:
    """Always recompiles: every source to an object file (in parallel), then one link.
    -ffp-contract=off: the kernels spell out every fused multiply-add they want;
    packed-fp32 instruction selection is disabled."""
    flags = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-ffp-contract=off",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
             "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    noise = "is not a recognized feature for this target"
    logs = []

    def run(cmd):
        res = subprocess.run(cmd, capture_output=True, text=True)
        log = "\n".join(l for l in (res.stdout + res.stderr).splitlines() if noise not in l)
        if res.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + log)
        logs.append(log)

    with tempfile.TemporaryDirectory(prefix="spd_build_") as tmp:
        objs = [os.path.join(tmp, os.path.splitext(s)[0] + ".o") for s in SOURCES]
        with ThreadPoolExecutor(max_workers=min(len(SOURCES), os.cpu_count() or 1)) as pool:
            list(pool.map(lambda so: run([hipcc(), *flags, "-x", "hip", "-c", os.path.join(CSRC, so[0]), "-o", so[1]]),
                          zip(SOURCES, objs)))
        run([hipcc(), "--offload-arch=gfx950", "-fPIC", "-shared", *objs, "-o", out])
    if verbose and any(l.strip() for l in logs):
        print("\n".join(l for l in logs if l.strip()))
    return out


if __name__ == "__main__":
    print(build_library(verbose=True))
