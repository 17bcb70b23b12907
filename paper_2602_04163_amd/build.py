"""Builds libbpdq.so (the C-ABI library) for gfx950 with hipcc, in-tree.

    python -m paper_2602_04163_amd.build
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libbpdq.so")
# the heaviest translation units first: the pool starts them first
SOURCES = ["group_sweep_k3_g256.hip",
           "group_sweep_k3_g256u.hip", "group_sweep_k2_g256.hip", "group_sweep_k2_g256u.hip",
           "group_sweep_k1_g256.hip", "group_sweep_k1_g256u.hip", "group_sweep_k4.hip",
           "group_sweep_k3.hip", "group_sweep_k2.hip", "group_sweep_k1.hip", "hessian.hip", "prepare.hip", "quantize.hip", "order.hip", "gemv.hip", "ceilings.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument", "-Wno-unknown-attributes",
]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    out = "\n".join(l for l in (res.stdout + res.stderr).splitlines()
                    if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)


def build(verbose: bool = True) -> str:
    """Compile every translation unit (in parallel) and link libbpdq.so."""
    from concurrent.futures import ThreadPoolExecutor
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    compile_flags = [f for f in FLAGS if f != "-shared"]
    jobs = []
    for src in SOURCES:
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        jobs.append(([hipcc] + compile_flags + ["-c", os.path.join(CSRC, src), "-o", obj], obj))
    with ThreadPoolExecutor(max_workers=min(len(jobs), os.cpu_count() or 4)) as ex:
        list(ex.map(lambda j: _run(j[0], verbose), jobs))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + [j[1] for j in jobs] + ["-o", LIB],
         verbose)
    return LIB


if __name__ == "__main__":
    build()
    sys.exit(0)
