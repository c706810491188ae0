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
    # multi-workgroup Sinkhorn: the fp32 kernel matrix once per iteration
    bound, amount, unit, _ = bench.kernel_work("k_sinkhorn", big_n, big_m, 1280, 2, 100, 0.05, 0.2)
    assert (bound, unit) == ("hbm", "GB/s") and amount == 4.0 * 100 * 2783 * 1729
    # a temperature whose exp range exceeds fp32 keeps the matrix in fp64
    _, amount64, _, _ = bench.kernel_work("k_sinkhorn", big_n, big_m, 1280, 2, 100, 0.02, 0.2)
    assert amount64 == 2 * amount
