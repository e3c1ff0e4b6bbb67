"""bench.py's command line, without a GPU: more than one GPU is refused with a message that says so, and the
workload arithmetic the JSON line is built from (visible pairs, condensation bytes) matches closed forms."""
import os
import subprocess
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert p.returncode != 0
    assert "ONE GPU" in p.stderr and "--gpus" in p.stderr
    assert p.stdout.strip() == ""                      # no JSON line for a run that did not happen


def test_pair_count_closed_forms():
    sys.path.insert(0, ROOT)
    import bench
    from paper_2604_12452_amd import inputs
    # dense (g = 1 keeps every token): L (L + 1) / 2 pairs
    assert bench.pair_count(1000, 0, 1) == 1000 * 1001 // 2
    # window longer than the sequence: nothing is condensed
    assert bench.pair_count(500, 600, 16) == 500 * 501 // 2
    # brute force on a small case: row t sees m_t representatives and the raw tokens m_t g .. t
    L, w, g = 257, 40, 8
    brute = sum(max(0, (t + 1 - w) // g) + (t + 1 - max(0, (t + 1 - w) // g) * g) for t in range(L))
    assert bench.pair_count(L, w, g) == brute
    # the 128K configuration: 663 M visible pairs per head, 23.09 TFLOP per launch, 159.5 MB condensed
    wl = inputs.configs()["cfg4"]
    assert abs(bench.pair_count(wl.L, wl.w, wl.g) - 663e6) < 1e6
    flops = 2.0 * (wl.d_qk + wl.d_v) * wl.B * wl.H * bench.pair_count(wl.L, wl.w, wl.g)
    assert abs(flops - 23.09e12) < 0.01e12
    assert abs(bench.condense_bytes(wl, 8128) - 159.5e6) < 0.3e6      # m = (131072 - 1024) / 16 groups
    rows = np.array([0, 100, 256], dtype=np.int64)
    assert bench.pair_count(L, w, g, rows) == sum(max(0, (t + 1 - w) // g) + (t + 1 - max(0, (t + 1 - w) // g) * g) for t in rows)
