"""GPU: bench.py runs end to end on the small configurations and prints the contract's JSON line (with the
roofline and the CPU baseline), also with the slow tier in a file; more than one GPU is refused."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                          timeout=280, cwd=ROOT)


def test_bench_line_on_the_tiny_configuration():
    r = _bench("--workload", "tiny_gpt_fp32", "--steps", "2", "--warmup", "1")
    assert r.returncode == 0, r.stderr[-2000:]
    d = json.loads(r.stdout.strip().splitlines()[-1])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 2 and d["warmup"] == 1 and d["vs_baseline"] is None
    assert d["value"] > 0 and d["config"]["workload"] == "tiny_gpt_fp32" and d["dtype"] == "fp32"
    rf = d["roofline"]
    assert rf["bound"] == "alu" and rf["peak"] == 157.3 and abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-12
    assert d["cpu_baseline"]["kind"] == "oracle" and d["cpu_baseline"]["value"] > 0 and d["cpu_baseline"]["cores"] >= 1
    assert abs(d["model_predicted_ms_per_step"] - d["ms_per_step"]) < d["ms_per_step"]      # same order of magnitude


def test_bench_with_the_slow_tier_in_a_file(tmp_path):
    r = _bench("--workload", "tiny_llama_fp32", "--steps", "2", "--warmup", "1", "--slow-tier", "file",
               "--file", str(tmp_path / "tier.bin"), "--staging-mb", "8", "--chunk-mb", "1", "--no-cpu-baseline")
    assert r.returncode == 0, r.stderr[-2000:]
    d = json.loads(r.stdout.strip().splitlines()[-1])
    assert d["file_tier"]["file_bytes"] > 0 and d["config"]["channels"] == "one shared" and d["value"] > 0
    assert not os.path.exists(str(tmp_path / "tier.bin"))


def test_bench_refuses_more_than_one_gpu():
    r = _bench("--gpus", "2")
    assert r.returncode == 2 and "one GPU" in r.stderr
