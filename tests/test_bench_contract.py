"""bench.py contract checks that need no GPU: the multi-GPU request is refused with a message, and the table of
algorithmic work the benchmark divides by matches the closed forms."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "single-GPU" in (r.stdout + r.stderr)


def test_pairs_formula_and_layer_flops():
    sys.path.insert(0, ROOT)
    import bench
    # visible (row, column) pairs of call j: C * jC columns of earlier chunks + the causal triangle with its diagonal
    for C in (1, 7, 128):
        for j in (0, 1, 5):
            brute = sum(j * C + r + 1 for r in range(C))
            assert bench.pairs(j, C) == brute
    # whole layer: sum over calls == N (N + 1) / 2 pairs per head
    N, C = 1024, 128
    assert sum(bench.pairs(j, C) for j in range(N // C)) == N * (N + 1) // 2
