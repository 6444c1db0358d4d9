"""Host-side behaviour of bench.py that needs no GPU."""
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr
    assert r.stdout.strip() == ""          # no JSON line for a run that did not happen


def test_traffic_figure_names_its_source():
    """The HBM traffic that bench.py reports comes from a committed rocprofv3 summary."""
    with open(os.path.join(ROOT, "profiles", "hbm_traffic.json")) as f:
        t = json.load(f)
    for name, rec in t.items():
        assert rec["gate_up_bytes_per_launch"] > 0
        src = rec["source"]
        assert os.path.exists(os.path.join(ROOT, "profiles", src)), src
        with open(os.path.join(ROOT, "profiles", src)) as f:
            assert "FETCH_SIZE" in f.read()
