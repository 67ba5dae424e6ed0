"""Host-side behaviour of bench.py that needs no GPU: the refusal of more than one GPU and the
rule that ties the recorded HBM traffic figure to the kernel source and to the workload."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench  # noqa: E402
from paper_2603_01501_amd import build  # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode == 2
    assert "--gpus 1" in r.stderr and r.stdout.strip() == ""


def test_traffic_figure_belongs_to_one_kernel_source_and_one_workload():
    # a figure recorded for other kernel code is never reported
    assert bench.recorded_traffic("0" * 64, "7.6B") is None
    # workloads without a counter summary report none
    sha = build.kernel_code_sha256()
    assert bench.recorded_traffic(sha, "1.5B") is None and bench.recorded_traffic(sha, "flat") is None
    # where a summary exists for the current code, the figure is that workload's own:
    # 4 N s bytes of the in-place pass (30 N of the fused AdamW pass) within a per cent
    for name, expected in (("7.6B", 4.0 * 7615487488 * 2), ("0.5B", 4.0 * 494005120 * 4),
                           ("14B-adamw", 30.0 * 14769689600)):
        t = bench.recorded_traffic(sha, name)
        if t is not None:
            assert abs(t / expected - 1.0) < 0.01, (name, t)
