"""Compile-time resource check of the matrix-core kernels (no GPU needed: hipcc cross-compiles): none may spill
registers, and each must leave room for two wavefronts per SIMD, which their latency hiding is built on."""
import os
import re
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor

import pytest

from paper_2505_16710_amd import build as B

KERNEL_FILES = ["fwd_bf16.hip", "fwd4_bf16.hip", "fwd4_split_bf16.hip", "bwd_dq_bf16.hip", "bwd_dkdv_bf16.hip"]


def _usage(src):
    sched = ["-mllvm", "-amdgpu-sched-strategy=" + B.SCHED.get(src, B.SCHED_DEFAULT)]
    cmd = [B.HIPCC, *B.FLAGS, *sched, *B.PER_FILE.get(src, []), "-Rpass-analysis=kernel-resource-usage", "-x", "hip",
           "--cuda-device-only", "-c", os.path.join(B.CSRC, src), "-o", os.devnull]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    out = []
    for block in r.stderr.split("Function Name: ")[1:]:
        name = block.split()[0]
        def num(key):
            m = re.search(key + r":\s*(\d+)", block)
            return int(m.group(1)) if m else None
        out.append((name, num("VGPRs Spill"), num("SGPRs Spill"), num(r"Occupancy \[waves/SIMD\]"), num(r"ScratchSize \[bytes/lane\]")))
    return out


def _lane_moves_in_loops(src):
    """Scalar spills are v_writelane / v_readlane pairs: count those that sit in a basic block of a loop."""
    sched = ["-mllvm", "-amdgpu-sched-strategy=" + B.SCHED.get(src, B.SCHED_DEFAULT)]
    with tempfile.TemporaryDirectory() as tmp:
        asm = os.path.join(tmp, "k.s")
        cmd = [B.HIPCC, *B.FLAGS, *sched, *B.PER_FILE.get(src, []), "-x", "hip", "--cuda-device-only", "-S",
               os.path.join(B.CSRC, src), "-o", asm]
        r = subprocess.run(cmd, capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-2000:]
        text = open(asm).read()
    in_loop, found = False, []
    for line in text.splitlines():
        if re.match(r"^\.LBB\d+_\d+:", line):
            in_loop = "Loop" in line         # the compiler annotates the blocks of a loop with its header
        elif re.match(r"^[A-Za-z_.$][\w.$]*:", line):
            in_loop = False
        elif in_loop and re.match(r"\s+v_(readlane|writelane)_b32", line):
            found.append(line.strip())
    return found


@pytest.mark.skipif(not os.path.exists(B.HIPCC), reason="hipcc not found")
def test_matrix_core_kernels_do_not_spill():
    with ThreadPoolExecutor(max_workers=4) as ex:
        results = list(ex.map(_usage, KERNEL_FILES))
    seen, spilling = 0, set()
    for src, kernels in zip(KERNEL_FILES, results):
        assert kernels, src
        for name, vspill, sspill, occ, scratch in kernels:
            if "merge" in name:          # the small merge kernel runs at full occupancy anyway
                continue
            seen += 1
            assert vspill == 0 and scratch == 0, (src, name, vspill, sspill, scratch)
            # scalar values parked in the lanes of a spare vector register (no memory traffic): tolerated in small
            # numbers - the dK/dV kernel, whose two roles are separate instantiations of its body inside one kernel,
            # parks launch constants that way - as long as none of it happens inside a loop (checked below)
            assert sspill <= 24, (src, name, sspill)
            spilling.add(src if sspill else None)
            assert occ is not None and occ >= 2, (src, name, occ)
    assert seen >= 10                    # 1 + 2 forward, 6 dQ, 1 dK/dV instantiations
    for src in sorted(x for x in spilling if x):
        assert _lane_moves_in_loops(src) == [], src
