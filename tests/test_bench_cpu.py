"""Host-side checks of the benchmark's contract that need no GPU."""
import os
import subprocess
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True,
                       text=True, cwd=ROOT)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_algorithmic_work_per_kernel():
    sys.path.insert(0, ROOT)
    import bench
    n = np.array([400, 400], dtype=np.int64)
    m = np.array([390, 400], dtype=np.int64)
    # norm pass: every token row once plus 12 bytes per token
    bound, amount, unit, peak = bench.kernel_work("k_norms", n, m, 1280, 2, 100)
    assert (bound, unit, peak) == ("hbm", "GB/s", 8000.0)
    assert amount == 800 * 1280 * 2 + 12 * 800
    # merge: rows in, kept rows out, plan in
    bound, amount, _, _ = bench.kernel_work("k_merge", n, m, 1280, 2, 100)
    assert bound == "hbm" and amount == 800 * 1280 * 2 + 790 * 1280 * 2 + 4 * 390 * 10
    # with many pruned tokens the merge is arithmetic-bound and runs on the matrix cores
    big_n, big_m = np.array([4512], dtype=np.int64), np.array([2783], dtype=np.int64)
    bound, amount, unit, peak = bench.kernel_work("k_merge", big_n, big_m, 1280, 2, 100)
    assert (bound, unit, peak) == ("mfma", "TFLOP/s", 2500.0) and amount == 2.0 * 2783 * 1729 * 1280
    # Sinkhorn is priced as fp64 vector work on every workload: two sweeps of multiply-adds
    # over the augmented matrix per iteration ...
    bound, amount, unit, peak = bench.kernel_work("k_sinkhorn", big_n, big_m, 1280, 2, 100, 0.05, 0.2)
    assert (bound, unit, peak) == ("alu", "TFLOP/s", 78.6) and amount == 4.0 * 100 * 2784 * 1730
    bound, amount, unit, _ = bench.kernel_work("k_sinkhorn_regs", n, m, 1280, 2, 100)
    assert (bound, unit) == ("alu", "TFLOP/s") and amount == 4.0 * 100 * (391 * 11 + 401 * 1)
    # ... and what the multi-workgroup kernels stream per call is a figure beside it: the fp32
    # kernel matrix once per iteration, fp64 when exp's range exceeds fp32, nothing when every
    # image fits a register-resident shape
    assert bench.sinkhorn_streamed_bytes(big_n, big_m, 100, 0.05, 0.2) == 4.0 * 100 * 2783 * 1729
    assert bench.sinkhorn_streamed_bytes(big_n, big_m, 100, 0.02, 0.2) == 8.0 * 100 * 2783 * 1729
    assert bench.sinkhorn_streamed_bytes(n, m, 100, 0.05, 0.2) == 0.0


def test_oracle_fanout_counts_every_image():
    """The all-cores oracle timing deals the images to worker processes and reports images/s."""
    sys.path.insert(0, ROOT)
    import bench
    fan = bench.oracle_fanout(2, 6, 3)
    assert fan["cores"] == 3 and fan["unit"] == "images/s" and fan["value"] > 0
