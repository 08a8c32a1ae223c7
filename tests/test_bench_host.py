"""Host-side checks of bench.py (no GPU needed) and, on a GPU, the shape of its JSON line."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402
from paper_2504_04704_amd import synth  # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True)
    assert r.returncode != 0
    assert "ONE GPU" in (r.stdout + r.stderr)


def test_algorithmic_bytes_of_the_headline_workload():
    """Each input element once, each kept element once, plus the int32 positions:
    1024 streams x (2 tensors x 2 B x 128 x (131072 + 33536) + 4 x 33536)."""
    cfg = synth.CONFIGS["cfg4_llama8b_128k_b4"]
    assert cfg.streams == 1024
    assert bench.algorithmic_bytes(cfg.streams, cfg.T, 33536, cfg.D, 2) == 86439362560
    assert bench.algorithmic_bytes(1, 10, 4, 8, 2, with_idx=False) == 2 * 2 * 8 * 14


def test_recorded_traffic_is_read_from_the_profile_summary():
    t = bench.read_traffic("split_pass_cfg4_llama8b_128k_b4_traffic.txt")
    assert t is not None and 86439362560 <= t < 2 * 86439362560      # at least the algorithmic bytes
    assert bench.read_traffic("no_such_file.txt") is None


@pytest.mark.gpu
def test_bench_line_has_the_contract_fields():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--config", "cfg2_llama8b_16k",
                        "--steps", "3", "--warmup", "1", "--cpu-streams", "4"],
                       capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.startswith("{")]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better",
                "scaling", "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 3 and d["warmup"] == 1 and d["vs_baseline"] is None
    assert d["config"]["workload"] == "cfg2_llama8b_16k" and d["data"] == "synthetic"
    roof = d["roofline"]
    assert roof["bound"] == "hbm" and roof["peak"] == 8000.0 and roof["unit"] == "GB/s"
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-12 and 0 < roof["frac"] < 1
    cpu = d["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["cores"] >= 1 and cpu["value"] > 0 and cpu["sample"]
    assert d["value"] > 100 * cpu["value"]
