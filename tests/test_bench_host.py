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
    for name in ("split_pass_cfg4_llama8b_128k_b4_traffic.txt", "hold_pass_cfg4_llama8b_128k_b4_traffic.txt"):
        t = bench.read_traffic(name)
        assert t is not None and 86439362560 <= t < 2 * 86439362560      # at least the algorithmic bytes
    assert bench.read_traffic("no_such_file.txt") is None


def test_decode_algorithmic_bytes():
    """Config 5, per call: (128 + 112 + 128) rows read, (32 + 128 + 112) written, 512 B of K+V each,
    8192 streams."""
    assert bench.decode_algorithmic_bytes(8192, 128, 112, 32, 128, 2) == 8192 * 640 * 512 == 2684354560


@pytest.mark.gpu
def test_bench_line_has_the_contract_fields():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--config", "cfg2_llama8b_16k",
                        "--steps", "3", "--warmup", "1", "--cpu-streams", "4", "--only-headline"],
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
    for key in ("kernel_ms_median", "kernel_ms_p10", "kernel_ms_p90", "frac_median", "frac_first_alloc",
                "frac_median_of_trials", "frac_of_copy", "copy_gbs", "algorithmic_bytes"):
        assert key in roof, key
    assert roof["kernel_ms_p10"] <= roof["kernel_ms_median"] <= roof["kernel_ms_p90"]
    assert d["dtype"] == "f32" and d["config"]["kv_dtype"] == "bf16" and d["config"]["compute_dtype"] == "f32"


@pytest.mark.gpu
def test_default_bench_run_reports_every_workload():
    """The command the harness runs (defaults; fewer steps and placements here): the headline
    line on the 128K configuration with configurations 2, 3 and the decode step in other_workloads."""
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "3", "--warmup", "1",
                        "--placements", "2", "--cpu-streams", "8"],
                       capture_output=True, text=True, timeout=900)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.startswith("{")]
    assert len(lines) == 1
    d = json.loads(lines[0])
    assert d["config"]["workload"] == "cfg4_llama8b_128k_b4" and d["metric"] == "kv_tokens_compressed_per_sec_128k_ctx"
    assert d["roofline"]["algorithmic_bytes"] == 86439362560 and len(d["config"]["placement_trials_ms"]) == 2
    others = {o["workload"]: o for o in d["config"]["other_workloads"]}
    assert set(others) == {"cfg2_llama8b_16k", "cfg3_llama8b_64k", "cfg5_decode_b32"}
    for o in others.values():
        assert 0 < o["frac"] < 1 and o["ms_p10"] <= o["ms"] <= o["ms_p90"] and o["algorithmic_bytes"] > 0
        assert o["cpu_baseline"]["kind"] == "oracle" and o["cpu_baseline"]["value"] > 0
    for o in ("cfg2_llama8b_16k", "cfg3_llama8b_64k"):
        assert others[o]["kernel"] == "hold_pass_kernel" and others[o]["traffic"] >= others[o]["algorithmic_bytes"]
    abl = {a["variant"]: a for a in d["config"]["scoring_ablations"]}
    assert set(abl) == {"local", "l2"} and all(0 < a["frac"] < 1 for a in abl.values())
    assert abl["local"]["kernel"] == "hold_pass_kernel" and abl["local"]["algorithmic_bytes"] == 86439362560
    assert abl["l2"]["kernel"] == "split_pass_kernel" and abl["l2"]["algorithmic_bytes"] == 60870885376
    dec = others["cfg5_decode_b32"]
    assert dec["steps"] == 64 and dec["length_after_the_first_steps"] == 8384 + 66 * 32
    assert dec["latency_ms_p50"] <= dec["latency_ms_p99"] and dec["algorithmic_bytes"] == 2684354560


def test_placement_pick_keeps_the_fastest_set_and_reports_every_trial():
    from paper_2504_04704_amd import placement
    speeds = iter([16.4, 14.1, 14.8, 16.3])
    built, released = [], []

    def build():
        built.append(object())
        return built[-1]

    times = {}

    def time_ms(ws):
        times[id(ws)] = next(speeds)
        return times[id(ws)]

    kept, trials = placement.pick(build, time_ms, trials=4, release=lambda: released.append(1))
    assert trials == [16.4, 14.1, 14.8, 16.3] and kept is built[1] and len(built) == 4 and len(released) == 5
    kept, trials = placement.pick(lambda: "only", lambda ws: 3.0, trials=0)       # at least one allocation
    assert kept == "only" and trials == [3.0]
