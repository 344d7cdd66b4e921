"""Host-side behaviour of bench.py that needs no GPU: more than one GPU is refused with a message,
and the HBM traffic of the dominant kernel comes from the committed profile summary together with
the commit it was measured at."""
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_traffic_comes_from_the_profile_summary():
    sys.path.insert(0, ROOT)
    import bench
    traffic, at = bench.measured_traffic("k_dscatter")
    line = [l for l in open(os.path.join(ROOT, "profiles", "bench_llama7b_hbm_traffic.md")) if l.startswith("traffic_bytes:")]
    assert len(line) == 1
    d = json.loads(line[0].split(":", 1)[1])
    assert traffic == d["k_dscatter"] and at == d["measured_at"]
    # fetched + written of the scatter: its three 9-bit streams and little more (the table in the file)
    assert 22.7e9 < traffic < 30e9
    assert bench.measured_traffic("no_such_kernel")[0] is None
