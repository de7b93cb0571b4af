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


def _section_rows(path, section):
    """(kernel row name, KiB) pairs of one '== <section>' block of a profile summary, read line by line."""
    rows, on = [], False
    for line in open(path):
        if line.startswith("== "):
            on = line.startswith("== " + section)
            continue
        if on and " n=" in line and line.rstrip().endswith("KiB"):
            rows.append((line.split(" n=")[0].strip(), float(line.split()[-2])))
    return rows


def test_roofline_traffic_is_what_the_committed_profiles_say():
    """bench.py's `traffic` figures are read from profiles/ at run time; recompute them here from the raw rows
    (FETCH_SIZE and WRITE_SIZE, each scaled by the 1 GiB calibration kernel's reading) for every committed
    summary, so a refreshed profile and the bench line cannot drift apart."""
    sys.path.insert(0, ROOT)
    import bench
    from paper_2303_06182_amd import workloads as wl
    prof_dir = os.path.join(ROOT, "profiles")
    known = {"gate_gemm", "gate_topk", "topk", "route", "dispatch", "expert_gemm1", "expert_gemm2", "combine", "tile_map"}
    seen = 0
    for fname in sorted(os.listdir(prof_dir)):
        if not (fname.startswith("moe_layer_forward_") and fname.endswith(".txt")):
            continue
        workload = fname[len("moe_layer_forward_"):-4]
        assert workload in wl.CONFIGS, workload
        got = bench.traffic_from_profile(workload)
        assert got and set(got) <= known, (workload, got)
        path = os.path.join(prof_dir, fname)
        fetch, write = _section_rows(path, "FETCH_SIZE"), _section_rows(path, "WRITE_SIZE")
        gib_kib = 1024 * 1024
        f_scale = gib_kib / [v for k, v in fetch if "FunctorOnSelf_add<int>" in k][0]
        w_scale = gib_kib / [v for k, v in write if "FunctorOnSelf_add<int>" in k][0]
        assert 1.9 < f_scale < 2.1 and 0.95 < w_scale < 1.05   # this device: FETCH_SIZE counts half the bytes
        # combine is one launch of one kernel in every workload
        want = 1024 * (f_scale * sum(v for k, v in fetch if k.startswith("combine_kernel")) +
                       w_scale * sum(v for k, v in write if k.startswith("combine_kernel")))
        assert abs(got["combine"] - want) <= 1e-6 * want + 1
        # an expert GEMM is the sum over its launches: bf16 weights (last template argument 0), grouped, ReLU
        def is_gemm1(k):
            if not k.startswith("gemm_bf16_kernel<"):
                return False
            a = [x.strip() for x in k[len("gemm_bf16_kernel<"):-1].split(",")]
            return a[5] == "true" and a[6] == "true" and a[-1] == "0"
        if any(is_gemm1(k) for k, _ in fetch):
            want = 1024 * (f_scale * sum(v for k, v in fetch if is_gemm1(k)) + w_scale * sum(v for k, v in write if is_gemm1(k)))
            assert abs(got["expert_gemm1"] - want) <= 1e-6 * want + 1
            w = wl.CONFIGS[workload]
            assert got["expert_gemm1"] >= w.k * w.T * (w.D + w.F) * 2   # never below the activation bytes alone
        seen += 1
    assert seen >= 4
    assert bench.traffic_from_profile("no_such_workload") == {}


def test_profile_rows_map_to_the_layer_steps():
    sys.path.insert(0, ROOT)
    import bench
    f = bench.profile_kernel_name
    assert f("gemm_bf16_kernel<256, 256, 2, 4, false, true, true, true, 1, 0, 0>") == "expert_gemm1"
    assert f("gemm_bf16_kernel<128, 128, 2, 2, false, false, true, true, 2, 0, 0>") == "expert_gemm2"
    assert f("gemm_bf16_kernel<128, 128, 2, 2, true, false, false, true, 2, 2, 0>") == "gate_gemm"
    assert f("gemm_bf16_kernel<32, 128, 1, 4, false, true, true, true, 2, 4, 8>") is None   # e4m3 weights
    assert f("gemm_bf16_kernel<256, 256, 2, 4, false, false, false, true, 1, 0, 0>") is None  # static baseline's einsum
    assert f("gemm_f32_mfma_kernel<true, true>") == "expert_gemm1"
    assert f("gemm_f32_mfma_kernel<false, false>") == "gate_gemm"
    assert f("route_scan_kernel") == "route" and f("topk_kernel<16, 8, true>") == "topk"
    assert f("at::native::vectorized_elementwise_kernel<4, at::native::CUDAFunctorOnSelf_add<int>, std::") is None
