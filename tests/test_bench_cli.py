"""Host-side behaviour of bench.py that needs no GPU."""
import os
import subprocess
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_synthetic_head_accuracies_are_valid_cumulative_rates():
    sys.path.insert(0, ROOT)
    import bench
    P = bench.synthetic_hit_rates()
    assert P.shape == (len(bench.HEAD_TOP1), bench.HEAD_K_MAX)
    assert (P >= 0).all() and (P <= 1).all() and (np.diff(P, axis=1) >= 0).all()
    assert (np.diff(P[:, 0]) < 0).all()          # later heads are less accurate
