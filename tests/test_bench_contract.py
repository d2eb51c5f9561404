"""The benchmark's command-line contract that can be checked without a GPU: more than one GPU is refused with a
message (this build measures one GPU), the headline workload is the large-size prefill, and the traffic figures
quoted in the result line are read from the rocprofv3 summaries under profiles/."""
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


def _bench():
    sys.path.insert(0, ROOT)
    import importlib
    return importlib.import_module("bench")


def test_default_headline_is_the_large_prefill():
    bench = _bench()
    args = bench.parse([])
    assert bench.PREFILL_WORKLOADS[args.workload] == "large_prefill_24x24"
    assert set(args.legs.split(",")) == {"base_prefill", "highres_prefill"}
    assert args.gpus == 1 and args.steps > 0 and args.warmup > 0


def test_traffic_comes_from_the_profile_summaries():
    bench = _bench()
    from paper_2507_01652_amd import workloads as wl
    found = 0
    for kind, pattern in bench.TRAFFIC_FILES.items():
        for name in wl.CONFIGS:
            path = os.path.join(ROOT, "profiles", pattern.format(w=name))
            got = bench.measured_traffic(kind, name)
            if os.path.exists(path):
                assert isinstance(got, int) and got > 0, path
                assert str(got) in open(path).read()
                found += 1
            else:
                assert got is None
    assert found >= 4      # forward x 3 shapes and the decode step at least
