"""Host-side pieces of bench.py: the paper's communication-load context printed beside
the measurement (Sec. 2.1; the x78 of Table 1's first row), the traffic figure read
from the committed counter summary, and the one-GPU rule."""
import os
import subprocess
import sys

import bench
from paper_2011_06495_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_comm_load_context_reproduces_the_paper_s_first_row():
    w = W.C2.with_size(W.C2.d, K=111_740)                 # phi = 1e-2 on ResNet-18's size
    c = bench.comm_load_context(w)
    assert c["bits_per_position"] == 9                    # log2(1/phi) rounded up, + 2 (Sec. 2.1)
    assert c["Q_loc_bits"] == 9 * 111_740 and c["Q_val_bits"] == 32 * 111_740
    assert abs(c["compression"] - 78.0) <= 0.1            # Table 1, SSGD-MV
    assert bench.comm_load_context(W.C4)["bits_per_position"] == 12      # phi = 1e-3 (Sec. 3)


def test_traffic_summary_is_read_and_sane():
    t, source = bench.measured_traffic("C4")
    algorithmic = 12 * 16 * 11_173_962
    assert t is not None and algorithmic <= t <= 1.2 * algorithmic
    assert source == os.path.join("profiles", "vote_step_C4_hbm_counters.txt")
    assert bench.measured_traffic("no such workload") == (None, None)


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout.strip() == ""
