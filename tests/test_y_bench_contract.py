"""The benchmark's command line: one GPU only, and - on the GPU - one JSON line with the fields
the measurement contract names."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_traffic_figure_comes_from_the_committed_counter_summary():
    """roofline.traffic is read from profiles/ (not pasted into bench.py): the summary holds a
    line per profiled kernel, and each figure is the kernel's algorithmic bytes plus a few
    per cent of tables and partial records at most."""
    sys.path.insert(0, ROOT)
    import bench
    n_act = 2_710_562_816                               # activation elements of ResNet-50 at batch 256
    for name, alg in ((bench.ROCPROF_NAMES["k_statspair_stream"], 8 * n_act),
                      (bench.ROCPROF_NAMES["k_pair_stream"], 8 * n_act),
                      ("k_quant_stream<256, 2, false, false, false, false>", 5 * n_act)):   # the pass's quantize sweep
        t = bench.traffic_from_profile(name)
        assert t is not None, name
        assert alg <= t <= 1.005 * alg, (name, t, alg)
    assert bench.traffic_from_profile("no_such_kernel") is None
    assert bench.traffic_from_profile(bench.ROCPROF_NAMES["k_pair_stream"], "/nonexistent") is None


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True,
                       text=True, timeout=120)
    assert r.returncode != 0 and "ONE GPU" in r.stderr and r.stdout.strip() == ""


@pytest.mark.gpu
def test_json_line_of_a_small_run():
    """ResNet-18 batch 32 (a parity-test set, not the headline workload): every field of the
    contract is present and consistent."""
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", "resnet18", "--steps", "5",
                        "--warmup", "2", "--cpu-sample-elems", "20000000", "--no-single-tensor-extra"],
                       capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.startswith("{")]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for k in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
              "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert k in d, k
    assert d["n_gpus"] == 1 and d["steps"] == 5 and d["warmup"] == 2 and d["unit"] == "GB/s"
    assert d["vs_baseline"] is None and d["dtype"] == "f32" and d["data"] == "synthetic"
    assert d["config"]["workload"] == "resnet18_b32" and "model" not in d["config"]
    rf = d["roofline"]
    assert rf["bound"] == "hbm" and rf["peak"] == 8000.0 and rf["unit"] == "GB/s"
    assert abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-3 and 0.0 < rf["frac"] < 1.0
    assert rf["traffic"] is None                       # counters were taken on the headline workload only
    cb = d["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["cores"] == 1 and cb["value"] > 0 and cb["sample"]
    assert d["cpu_baseline_all_cores"]["cores"] >= 1
    # the headline rate is bytes actually moved over time: it cannot exceed the HBM peak
    assert abs(d["value"] - d["config"]["moved_bytes_per_pass"] / d["ms_per_step"] / 1e6) < 0.01 * d["value"]
    assert 0 < d["value"] < 8000.0 and abs(d["frac_of_hbm_peak"] - d["value"] / 8000.0) < 1e-3
    assert d["three_call_equivalent_GBps"] > d["value"]
    assert cb["elements_covered"] <= 20000000 < cb["elements_total"]
    sp = d["oracle_speedup"]
    assert sp["vs_1_core"] > sp["vs_all_cores"] > 1 and sp["cores"] == d["cpu_baseline_all_cores"]["cores"]
    assert d["pipelined"]["same_order"] is True and 0 < d["pipelined"]["ms_per_step"] <= d["ms_per_step"] * 1.05
    assert "workloads" not in d                        # only the default workload carries the other sets
    assert d["other_pass"]["same_order"] is True
    assert d["ms_per_step_min"] <= d["ms_per_step_median"] and d["cold"]["ms_per_step"] > 0


@pytest.mark.gpu
@pytest.mark.parametrize("mode,kernel", [("fused", "k_quantpair_stream"), ("calls", "k_pair_stream")])
def test_other_pass_forms_report_their_own_dominant_kernel(mode, kernel):
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", "resnet18", "--steps", "5",
                        "--warmup", "2", "--mode", mode, "--single-mode", "--no-cpu-baseline", "--no-cold"],
                       capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stderr[-2000:]
    d = json.loads([l for l in r.stdout.splitlines() if l.startswith("{")][0])
    assert d["roofline"]["kernel"] == kernel and d["roofline"]["avg_launch_ms"] > 0
    assert "cpu_baseline" not in d and "cold" not in d and "other_pass" not in d
    assert set(d["calls"]) == ({"calibrate", "fakequant_pair_metrics"} if mode == "fused"
                               else {"calibrate", "fakequant_metrics", "pair_metrics"})

