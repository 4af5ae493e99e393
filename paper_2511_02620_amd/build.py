"""Build libdifr.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree.

``python -m paper_2511_02620_amd.build`` compiles every source under ``csrc/`` and links
``paper_2511_02620_amd/libdifr.so``.  Nothing is built at import time: tests, the smoke check and
the benchmark load what this step left behind.
"""
from __future__ import annotations

import concurrent.futures
import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libdifr.so")
SOURCES = ["api.hip", "gumbel.hip", "ipt.hip", "fused.hip", "likelihood.hip", "ipt_filtered.hip", "nucleus.hip", "lmhead.hip", "reduce.hip"]

# -packed-fp32-ops is switched off: the compiler must not form packed fp32 instructions.
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc", "-Wall",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def _compile(src: str) -> str:
    obj = os.path.join(BUILD, os.path.splitext(src)[0] + ".o")
    cmd = [hipcc()] + HIPCC_FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if proc.returncode:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, proc.stdout))
    noise = "'-packed-fp32-ops' is not a recognized feature"
    out = "\n".join(l for l in proc.stdout.splitlines() if noise not in l and l.strip())
    if out:
        sys.stderr.write(out + "\n")
    return obj


def build(verbose: bool = True) -> str:
    os.makedirs(BUILD, exist_ok=True)
    with concurrent.futures.ThreadPoolExecutor(max_workers=4) as pool:
        objs = list(pool.map(_compile, SOURCES))
    tmp = LIB + ".tmp.%d" % os.getpid()
    cmd = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-rdc", "-o", tmp] + objs
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if proc.returncode:
        raise RuntimeError("link failed:\n%s" % proc.stdout)
    os.replace(tmp, LIB)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build()
