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


def test_traffic_constants_are_the_counter_figures_of_the_committed_profile():
    """roofline.traffic in the bench line comes from constants in bench.py; they must be the "total GB"
    entries of the per-dispatch counter table under profiles/."""
    sys.path.insert(0, ROOT)
    import bench
    rows = {}
    with open(os.path.join(ROOT, "profiles", "kernels_C2_W16_d11.2M_hbm_counters.md")) as f:
        for line in f:
            cells = [c.strip() for c in line.strip().strip("|").split("|")]
            if len(cells) == 6 and cells[0].startswith("local_step_kernel<"):
                rows[cells[0].split(">")[0] + ">"] = (float(cells[3]), float(cells[4].split()[0]))
    plain = rows["local_step_kernel<true,0,0,false,1,1>"]
    tail = rows["local_step_kernel<true,0,1,false,1,1>"]
    tail_k1 = rows["local_step_kernel<true,0,2,false,1,1>"]
    assert bench.STEP_TRAFFIC_BYTES == plain[0] * 1e9
    assert bench.TAIL_TRAFFIC_BYTES == {1: tail_k1[0] * 1e9, 2: tail[0] * 1e9}
    # and the table's algorithmic column is the byte model the bench uses (rows padded to 4 KiB: W x d here)
    W, d = 16, 11_200_000
    assert abs(plain[1] * 1e9 - 24 * W * d) < 1e5
    assert abs(tail[1] * 1e9 - bench.tail_step_bytes(W, d, 2)) < 1e5 and abs(tail_k1[1] * 1e9 - bench.tail_step_bytes(W, d, 1)) < 1e5
