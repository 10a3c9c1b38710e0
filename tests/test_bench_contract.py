"""Host-side parts of bench.py that need no GPU: the one-GPU rule and the profile reader."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       cwd=ROOT, timeout=120)
    assert p.returncode != 0
    assert "ONE GPU" in (p.stdout + p.stderr)
    assert not any(line.startswith("{") for line in p.stdout.splitlines())   # no result line


def test_traffic_figures_come_from_the_committed_counter_summary():
    sys.path.insert(0, ROOT)
    import bench
    for workload, kernel in (("mixtral", "ffn_gate_up"), ("mixtral", "ffn_down"), ("dsv3_ep", "ffn_gate_up")):
        t = bench.measured_traffic(workload, kernel)
        assert t is not None and 1e9 < t < 1e11, (workload, kernel, t)
    assert bench.measured_traffic("tiny", "ffn_gate_up") is None             # never measured: reported as null
