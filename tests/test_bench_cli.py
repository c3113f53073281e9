"""Host-side behaviour of bench.py that needs no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                         capture_output=True, text=True, timeout=120)
    assert res.returncode != 0
    assert "ONE GPU" in (res.stdout + res.stderr)


def test_traffic_summaries_exist_for_the_benchmarked_workload():
    # bench.py reports roofline.traffic from the committed counter summary of the workload
    path = os.path.join(ROOT, "profiles", "traffic_llama3_8b_ctx4096.txt")
    text = open(path).read()
    vals = dict(line.split("=") for line in text.splitlines() if "=" in line and not line.startswith("#"))
    fetch, write = int(vals["fetch_bytes "]), int(vals["write_bytes "])
    # one pass over K+V (1 GiB) plus q/out: within 2 % of the algorithmic bytes
    assert abs(fetch + write - 1_074_798_848) / 1_074_798_848 < 0.02
