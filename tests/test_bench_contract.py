"""Host-side checks of bench.py's contract that need no GPU: the refusal of more than one GPU, and the profile
records it reads (one per workload, each tied to a library build)."""
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_traffic_records_name_their_build_and_every_timing_record_is_known():
    sys.path.insert(0, ROOT)
    from paper_2508_03854_amd.profile_summary import RECORD
    import bench
    known = set(RECORD.values())
    seen = 0
    for name in sorted(os.listdir(os.path.join(ROOT, "profiles"))):
        if not name.endswith("_traffic.json"):
            continue
        d = json.load(open(os.path.join(ROOT, "profiles", name)))
        assert d["build"].startswith("tbe355 gfx950 ") and len(d["build"].split()[-1]) == 12
        assert name == d["workload"] + "_traffic.json"
        assert set(d["bytes_per_step"]) <= known
        assert all(v >= 0 for v in d["bytes_per_step"].values())
        # bench.py hands the record out for the build it was measured on, and for no other
        assert bench.measured_traffic(d["workload"], d["build"]) == {k: float(v) for k, v in d["bytes_per_step"].items()}
        assert bench.measured_traffic(d["workload"], "tbe355 gfx950 000000000000") is None
        seen += 1
    assert seen >= 1
