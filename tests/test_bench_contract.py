"""Host-only checks of the benchmark's command-line contract and its bookkeeping helpers."""
import os
import subprocess
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench  # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert res.returncode != 0
    assert "ONE MI355X" in res.stderr
    assert res.stdout.strip() == ""


def test_search_sizes_follow_from_the_per_seed_iterations():
    # 6 seeds of the hand-worked example: iterations [1, 0, 1, 0, 0, 2] with max_iter 3
    # -> searches of 6, 6, 3, 3, 1, 1 live queries (see tests/golden/handworked_walk.json)
    counts = bench.searches_from_iters(np.array([1, 0, 1, 0, 0, 2]), 6, 3)
    assert counts[:6] == [6, 6, 3, 3, 1, 1]
    # a seed that never converges stays live in every search
    counts = bench.searches_from_iters(np.array([0, -1]), 2, 2)
    assert counts == [2, 2, 1, 1]
    assert len(bench.searches_from_iters(np.zeros(4, dtype=int), 4, 10)) == 20
