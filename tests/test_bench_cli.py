"""bench.py's command line without a GPU: one GPU only, and the algorithmic byte counts it reports."""
import importlib.util
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "one GPU" in (r.stderr + r.stdout)


def test_algorithmic_bytes_of_the_benchmark_shape():
    spec = importlib.util.spec_from_file_location("bench", os.path.join(ROOT, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    rows, cols = bench.ROWS, bench.COLS
    assert (rows, cols) == (28672, 8192)
    groups = rows * cols // 8
    ab = bench.algorithmic_bytes(rows, cols, 24, 2, 1)
    index, codes, rownorm = groups * 3, groups * 2 // 8, rows * 4        # 24-bit indices, 2-bit codes
    assert ab["gemv"] == index + codes + rownorm + cols * 2 + rows * 4   # + x (bf16) + y (float32)
    assert ab["decode"] == index + codes + rownorm + rows * cols * 2
    assert ab["encode"] == rows * cols * 2 + index + codes + rownorm
