"""CPU: the host-side helpers of bench.py (no GPU): the file-system bandwidth probe, and the refusal of more
than one GPU, which is decided before anything touches the device."""
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


def test_file_bandwidth_probe(tmp_path):
    b = _bench_module()
    path = str(tmp_path / "probe.bin")
    r = b.probe_file_bw(path, total=16 << 20, block=1 << 20, threads=2)
    assert set(r) == {"write_Bps", "read_Bps", "duplex_write_Bps", "duplex_read_Bps", "direct"}
    assert all(r[k] > 0 for k in r if k != "direct") and not os.path.exists(path)


def test_more_than_one_gpu_is_refused_without_a_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "4"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_planner_times_compare_like_with_like(capsys):
    """bench.py --planner-times: the library's full search, its single pass and the oracle's single pass at the settled
    planning capacity give one entry list; times are positive; the line is JSON."""
    import json
    import bench
    out = bench.planner_times(names=("tiny_gpt_fp32", "tiny_llama_fp32"))
    line = [l for l in capsys.readouterr().out.splitlines() if l.startswith("{")][-1]
    assert json.loads(line)["planner_wall_time"][0]["workload"] == "tiny_gpt_fp32"
    for r in out["planner_wall_time"]:
        assert r["same_plan"] and r["entries"] > 0 and r["planning_cap_bytes"] <= r["cap_bytes"]
        assert r["library_search_s"] > 0 and r["library_single_s"] > 0 and r["oracle_single_s"] > 0


def test_compute_copy_overlap_of_a_small_timeline():
    """Overlap = time a copy is in flight while a kernel runs, over the time a copy is in flight (unions on both sides)."""
    b = _bench_module()
    kernels = [(0, 100), (150, 250), (240, 300)]                 # union: [0,100) and [150,300)
    copies = [(50, 200), (180, 220), (400, 500)]                  # union: [50,220) and [400,500): 270 busy
    r = b.interval_overlap(kernels, copies)
    assert abs(r["copy_busy_ms"] - 270e-6) < 1e-12 and abs(r["kernel_busy_ms"] - 250e-6) < 1e-12
    assert abs(r["copy_busy_under_kernels_ms"] - (50 + 70) * 1e-6) < 1e-12
    assert abs(r["frac_of_copy_time_with_a_kernel_running"] - 120 / 270) < 1e-12
    assert b.interval_overlap(kernels, [])["frac_of_copy_time_with_a_kernel_running"] is None
