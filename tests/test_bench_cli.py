"""Host-side contract of bench.py that needs no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_traffic_constant_matches_the_committed_profile():
    """The HBM traffic that bench.py reports for the dominant kernel is the figure of the committed counter summary."""
    sys.path.insert(0, ROOT)
    import importlib
    bench = importlib.import_module("bench")
    text = open(os.path.join(ROOT, "profiles", "verify_step_llama7b_hbm_traffic.txt")).read()
    line = [l for l in text.splitlines() if l.startswith("gate|up")][0].split()
    fetch_kib, write_kib = float(line[3]), float(line[6])
    assert bench.GATE_UP_7B_TRAFFIC_BYTES == int((fetch_kib * 2.0 + write_kib) * 1024)
