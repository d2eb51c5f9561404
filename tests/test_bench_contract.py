"""The benchmark's command-line contract that can be checked without a GPU: more than one GPU is refused with a
message (this build measures one GPU), and the measured-traffic table only names workloads that exist."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stdout + r.stderr) or "1 GPU" in (r.stdout + r.stderr) or "single" in (r.stdout + r.stderr).lower()
    assert not any(line.startswith("{") for line in r.stdout.splitlines())       # no result line


def test_traffic_table_names_known_workloads():
    sys.path.insert(0, ROOT)
    import importlib
    bench = importlib.import_module("bench")
    from paper_2507_01652_amd import workloads as wl
    for key in bench.MEASURED_TRAFFIC_BYTES:
        assert key.split(":")[-1] in wl.CONFIGS, key
