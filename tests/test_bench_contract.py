"""Host-side checks of bench.py that need no GPU: the one-GPU rule and the measured-traffic table it quotes."""
import importlib.util
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench_module():
    spec = importlib.util.spec_from_file_location("bench_under_test", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=300)
    assert r.returncode != 0
    assert "one GPU" in (r.stderr + r.stdout)


def test_traffic_table_covers_the_reported_kernel_of_both_profiled_workloads():
    bench = _bench_module()
    for workload in ("large_sage", "large_gcn_bf16"):
        t = bench.measured_traffic(workload, "agg_fwd")
        assert t is not None and t > 1e8, workload
    assert bench.measured_traffic("large_sage", "no_such_kernel") is None
