"""The bench line's contract, checked on the device with a short run of the real workload."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.timeout(600)
def test_bench_prints_one_json_line_with_roofline_and_cpu_baseline():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "5", "--warmup", "1", "--no-side-configs",
                        "--cpu-reps", "1"], capture_output=True, text=True, timeout=580)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 5 and d["warmup"] == 1 and d["vs_baseline"] is None and d["data"] == "synthetic"
    assert d["unit"] == "tokens/s" and abs(d["value"] - 5 / (d["ms_per_step"] * 1e-3)) < 1e-6 * d["value"]
    assert "workload" in d["config"] and "invalid" not in d
    rf = d["roofline"]
    assert rf["bound"] == "hbm" and rf["peak"] == 8000.0 and rf["unit"] == "GB/s"
    assert abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-9 and 0.3 < rf["frac"] < 1.0
    assert rf["traffic"] is not None and 1.0 <= rf["traffic"] / rf["bytes_per_launch"] < 1.1
    cb = d["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["unit"] == "tokens/s" and cb["cores"] >= 1 and cb["value"] > 0 and cb["sample"]
    # the 7B verify step streams 13.556 GB: anything far from a few milliseconds means work was skipped or repeated
    assert abs(d["algorithmic_bytes_per_step"] - 13.556e9) < 0.01e9 and 1.5 < d["ms_per_step"] < 10.0


def test_read_probe_reports_plausible_times_and_checks_its_arguments():
    """The plain-read chain behind `bench.py --probes`: times are positive and scale with the bytes; bad sizes are refused."""
    import torch
    from paper_2404_08856_amd import spd
    buf = torch.zeros(96 << 20, dtype=torch.uint8, device="cuda")
    sizes = [4 << 20, 32 << 20]
    us, chain = spd.spd_probe_read_chain(buf, sizes, reps=5)
    assert len(us) == 2 and all(t > 0 for t in us) and chain > 0
    assert us[1] > us[0]                                            # 8 x the bytes
    assert chain >= 0.5 * sum(us)                                   # the chain cannot be much shorter than its kernels
    rate = sizes[1] / us[1] / 1e3                                   # GB/s: at most the pin rate, and not absurdly low
    assert 100.0 < rate < 8000.0
    with pytest.raises(spd.SpdError):
        spd.spd_probe_read_chain(buf, [1000], reps=1)               # not a multiple of 1024
    with pytest.raises(spd.SpdError):
        spd.spd_probe_read_chain(buf, [128 << 20], reps=1)          # more than the buffer holds
