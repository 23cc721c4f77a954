"""Build the HIP library (gfx950) in-tree: paper_2010_04678_amd/libcals_hip.so.

hipcc cross-compiles without a GPU.  Each translation unit is compiled to an object in parallel,
then linked into one shared library that exports the C-ABI of include/cals.h.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libcals_hip.so")
OBJDIR = os.path.join(HERE, "_build")
SOURCES = ["mttkrp_wm1.hip", "mttkrp_wm2.hip", "mttkrp_wm3.hip", "mttkrp_wm4.hip", "mttkrp_rows_a.hip", "mttkrp_rows_b.hip", "mttkrp.hip", "update.hip", "linesearch.hip", "nnls.hip", "yardstick.hip", "reuse.hip", "krp.hip", "cals_api.hip"]
# yardstick.hip: its MFMA-only loop must keep the accumulators in place (VGPR form of the matrix instructions;
# otherwise the compiler copies them between register files every iteration and the probe measures the copies)
# mttkrp_rows_*.hip: with the default (accumulation-register) form of the matrix instructions the register allocator
# keeps these kernels' accumulators in vector registers and copies all of them in and out around every row tile; in
# the vector-register form they stay in place (the variants are sized to fit 256 vector registers)
EXTRA_FLAGS = {"yardstick.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"],
               "mttkrp_rows_a.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"],
               "mttkrp_rows_b.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"]}
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
         "-packed-fp32-ops", "-Wno-unused-command-line-argument"]


def _newest_source() -> float:
    t = 0.0
    for root in (CSRC, os.path.join(os.path.dirname(HERE), "include")):
        for f in os.listdir(root):
            t = max(t, os.path.getmtime(os.path.join(root, f)))
    return t


def is_stale() -> bool:
    return not os.path.exists(LIB) or os.path.getmtime(LIB) < _newest_source()


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile every HIP source for gfx950 and link the shared library.  Raises on failure."""
    if not force and not is_stale():
        return LIB
    os.makedirs(OBJDIR, exist_ok=True)

    def compile_one(src: str) -> str:
        obj = os.path.join(OBJDIR, src.replace(".hip", ".o"))
        cmd = ["hipcc", *FLAGS, *EXTRA_FLAGS.get(src, []), "-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed for %s:\n%s" % (src, r.stderr))
        if verbose and r.stderr.strip():
            sys.stderr.write(r.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    r = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n%s" % r.stderr)
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose=True))
