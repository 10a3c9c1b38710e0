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
        t, src = bench.profiled_traffic(workload, kernel)
        assert t is not None and 1e9 < t < 1e11, (workload, kernel, t)
        assert src.startswith("profiles/")
    assert bench.profiled_traffic("tiny", "ffn_gate_up") == (None, None)     # never measured: reported as null


def test_default_workload_is_the_largest_single_gpu_configuration_and_the_others_ride_along():
    sys.path.insert(0, ROOT)
    import bench
    import moe_inputs as mi
    flops = {n: c.N * c.K * c.H * c.F for n, c in mi.CONFIGS.items()}
    assert bench.DEFAULT_WORKLOAD == max(flops, key=flops.get) == "dsv3"
    assert set(bench.DEFAULT_ALSO.split(",")) >= {"mixtral", "gptoss", "dsv3_ep"}
