"""Host-side checks of bench.py's command line (no GPU)."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run_bench(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                          timeout=300)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = run_bench("--gpus", "2")
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and "--gpus 2" in r.stderr
    assert r.stdout.strip() == ""          # no JSON line for a run that did not happen


def test_the_traffic_table_names_only_known_workloads_and_kernels():
    sys.path.insert(0, ROOT)
    import bench
    from paper_2303_06182_amd import workloads as wl
    kernels = {"gate_gemm", "topk", "route", "dispatch", "expert_gemm1", "expert_gemm2", "combine"}
    for (workload, kernel), nbytes in bench.MEASURED_TRAFFIC_BYTES.items():
        assert workload in wl.CONFIGS, workload
        assert kernel in kernels, kernel
        assert nbytes > 0
