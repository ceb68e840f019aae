"""Build the C-ABI library libcg.so for gfx950 with hipcc (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libcg.so")
PROBE_SRC = os.path.join(ROOT, "bench_mfma_probe.hip")  # MFMA issue-rate microbenchmark of bench.py, not part of libcg
PROBE_LIB = os.path.join(ROOT, "libbench_mfma_probe.so")
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-fvisibility=hidden",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument"]


# share_gemm.hip is compiled once per group of kernel instantiations (-DCG_INST_GROUP): the groups compile side by side.
UNITS = [("cg_api.hip", "cg_api.o", []), ("share_gemm_f64.hip", "share_gemm_f64.o", []), ("prf.hip", "prf.o", []),
         ("share_gemm_small.hip", "share_gemm_small.o", []),
         ("share_gemm.hip", "share_gemm_g0.o", ["-DCG_INST_GROUP=0"]),
         ("share_gemm.hip", "share_gemm_g1.o", ["-DCG_INST_GROUP=1"]),
         ("share_gemm.hip", "share_gemm_g2.o", ["-DCG_INST_GROUP=2"])]


def build(verbose: bool = False) -> str:
    """Compile every HIP source (in parallel) and link libcg.so next to this file."""
    objs, procs = [], []
    for src, obj_name, defs in UNITS:
        obj = os.path.join(CSRC, obj_name)
        cmd = ["hipcc", *FLAGS, *defs, "-I", os.path.join(ROOT, "include"), "-I", CSRC,
               "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd))
        procs.append((cmd, subprocess.Popen(cmd)))
        objs.append(obj)
    for cmd, proc in procs:
        if proc.wait() != 0:
            raise subprocess.CalledProcessError(proc.returncode, cmd)
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    cmd = ["hipcc", *FLAGS, "-shared", "-o", PROBE_LIB, PROBE_SRC]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
