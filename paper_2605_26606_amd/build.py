"""Builds the HIP library in-tree: paper_2605_26606_amd/libpc.so (gfx950 only)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libpc.so")
KERNEL_BENCH = os.path.join(HERE, "kernel_bench")   # standalone driver of the hot kernels (tuning, counter runs)
SOURCES = ["api.hip", "elementwise.hip", "gemm.hip", "gemm_skinny.hip", "attention.hip", "sampler.hip", "allocation.hip", "scheduler.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         # packed-fp32 instructions are kept out of the generated code on purpose
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    return "hipcc"


def _run(cmd):
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in p.stdout.splitlines() if "packed-fp32-ops" not in l)
    if p.returncode != 0:
        raise RuntimeError("build step failed: %s\n%s" % (" ".join(cmd), out))
    return out


def build(verbose: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    cc = _hipcc()
    objs = [os.path.join(OBJ, s.replace(".hip", ".o")) for s in SOURCES]

    def one(i):
        return _run([cc, *FLAGS, "-c", os.path.join(CSRC, SOURCES[i]), "-o", objs[i]])

    with ThreadPoolExecutor(max_workers=min(6, os.cpu_count() or 1)) as ex:
        outs = list(ex.map(one, range(len(SOURCES))))
    outs.append(_run([cc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]))
    outs.append(_run([cc, *[f for f in FLAGS if f != "-fPIC"], "-Wno-unused-value", os.path.join(CSRC, "kernel_bench.hip"),
                      "-o", KERNEL_BENCH]))
    if verbose:
        sys.stdout.write("\n".join(o for o in outs if o.strip()) + "\n")
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
