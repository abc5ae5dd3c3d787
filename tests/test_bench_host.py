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
