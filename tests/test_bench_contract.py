"""bench.py's command-line contract where it can be checked without a GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=60)
    assert r.returncode != 0 and "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_byte_accounting_of_the_round():
    sys.path.insert(0, ROOT)
    import bench
    W, d = 16, 11_200_000
    wp = W * d
    # line 6 as its own pass: 24 k + 16 + 8 / W bytes per worker-parameter
    assert bench.model_round_bytes(W, d, 2) == wp * (48 + 16 + 0.5)
    # line 6 inside the last step: 24 k + 8 + 8 / W (k >= 2), 28 + 8 / W ... at k = 1 the step reads the stored models anyway
    assert bench.moved_round_bytes(W, d, 2, "fused_tail") == wp * (48 + 8 + 0.5)
    assert bench.moved_round_bytes(W, d, 1, "fused_tail") == wp * (24 + 4 + 0.5)
    assert bench.moved_round_bytes(W, d, 4, "graph_fused_tail") == wp * (96 + 8 + 0.5)
    # the mean formed inside the first step: no pass over the stored models for it
    assert bench.moved_round_bytes(W, d, 2, "head_fused_tail") == wp * (48 + 4 + 0.5)
    # k = 1 under that schedule: mean, step and line 6 in one pass, the mean only written
    assert bench.moved_round_bytes(W, d, 1, "head_fused_tail") == wp * 24.25
    assert bench.moved_round_bytes(W, d, 1, "head_separate") == wp * (24 + 12.25 + 0.25)
    assert bench.tail_step_bytes(W, d, 2) == wp * 28.25 and bench.tail_step_bytes(W, d, 1) == wp * 24.25
