"""bench.py contract checks that need no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert p.returncode != 0
    assert "ONE GPU" in (p.stderr + p.stdout)


def test_measured_traffic_table_is_well_formed():
    import json
    with open(os.path.join(ROOT, "profiles", "measured_traffic.json")) as fh:
        t = json.load(fh)
    for key, rec in t.items():
        if key.startswith("_"):
            continue
        workload, kernel = key.split(":")
        assert workload and kernel
        assert rec["hbm_bytes_per_step"] > 0
        assert abs(rec["fetch_bytes_per_step"] + rec["write_bytes_per_step"] - rec["hbm_bytes_per_step"]) <= 0.01 * rec["hbm_bytes_per_step"]
        assert os.path.exists(os.path.join(ROOT, rec["source"]))
