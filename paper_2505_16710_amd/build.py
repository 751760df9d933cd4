"""Build the HIP library (libseco_hip.so) for gfx950, in-tree.

`python -m paper_2505_16710_amd.build` or `build_library()`; also builds nothing else.
Objects go to `_build/` next to the sources; the shared library lands in the package
directory, where the ctypes binding looks for it.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(HERE, "libseco_hip.so")

SOURCES = [
    "seco_api.hip",
    "seco_select.cpp",
    "elementwise.hip",
    "kernels_f32.hip",
    "fwd_bf16.hip",
    "fwd4_bf16.hip",
    "fwd4_split_bf16.hip",
    "bwd_dq_bf16.hip",
    "bwd_dkdv_bf16.hip",
]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# -packed-fp32-ops off: the compiler must not form packed fp32 instructions from scalar code.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-I", INCLUDE, "-I", CSRC,
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function", "-Wno-inline-asm"]
# Machine scheduler strategy of the compiler, per source file (measured on the benchmark shapes, every strategy
# tried on every matrix-core kernel): keeping memory (LDS) instructions in clauses is 3 % faster than the default
# on the forward kernels and at least as good on the dK/dV kernel; the dQ kernels are 3 % faster with the
# iterative ILP scheduler.
SCHED = {"bwd_dq_bf16.hip": "iterative-ilp"}
SCHED_DEFAULT = "max-memory-clause"
# the 4-wavefront forward, whose source interleaves two instruction streams by hand, is 2 % faster when the
# scheduler does not cluster memory operations (its split instantiation would spill registers with that option)
PER_FILE = {"fwd4_bf16.hip": ["-mllvm", "-misched-cluster=false"]}


def _compile(src, extra=()):
    obj = os.path.join(CSRC, "_build", os.path.splitext(src)[0] + ".o")
    sched = ["-mllvm", "-amdgpu-sched-strategy=" + SCHED.get(src, SCHED_DEFAULT)]
    cmd = [HIPCC, *FLAGS, *sched, *PER_FILE.get(src, []), *extra, "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(ln for ln in r.stderr.splitlines() if noise not in ln)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build_library(verbose=True, extra=(), out=None):
    global LIB
    if out:
        LIB = out
    os.makedirs(os.path.join(CSRC, "_build"), exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(lambda s: _compile(s, extra), SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print(f"built {LIB}")
    return LIB


if __name__ == "__main__":
    # usage: python -m paper_2505_16710_amd.build [-o out.so] [extra hipcc flags, e.g. -DSECO_DKDV_RB=2]
    argv = sys.argv[1:]
    out = None
    if argv[:1] == ["-o"]:
        out, argv = argv[1], argv[2:]
    build_library(extra=tuple(argv), out=out)
