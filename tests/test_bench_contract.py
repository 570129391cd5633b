"""bench.py: what can be checked without a GPU (the refusal of more than one GPU, the algorithmic byte and flop
figures of the headline configuration) and, on a GPU, the keys of the JSON line."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0 and r.stdout.strip() == "" and "ONE GPU" in r.stderr


def test_algorithmic_figures_of_the_headline_configuration():
    import bench
    from paper_2410_01518_amd import synth
    cfg = synth.CONFIGS["c3"]
    ab = bench.algorithmic_bytes(cfg)
    units, e = 256, 2
    k_bytes, q_bytes, rows = units * 4096 * 128 * e, units * 256 * 128 * e, units * 2048 * 128 * e
    assert cfg.units == units and cfg.G * cfg.P == 256
    assert ab["score_stats"] == k_bytes + q_bytes
    assert ab["score_prob"] == k_bytes + q_bytes + units * 4096 * 4
    assert ab["call"] == k_bytes + q_bytes + 3 * rows + units * 2048 * 4 + 4096 * 4 == 689_979_392
    assert bench.algorithmic_flops(cfg) == 2.0 * units * 256 * 4096 * 128


@pytest.mark.gpu
def test_json_line_has_the_contract_keys():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "8", "--warmup", "2", "--cpu-units", "4"],
                       capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 8 and d["warmup"] == 2 and d["unit"] == "calls/s" and d["vs_baseline"] is None
    assert abs(d["value"] * d["ms_per_step"] - 1e3) < 1e-6 * 1e3
    assert "workload" in d["config"] and "model" not in d["config"]
    roof = d["roofline"]
    assert roof["bound"] in ("hbm", "mfma", "alu") and abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-12
    call = d["roofline_call"]                      # the whole call against the HBM peak: the figure the target is stated on
    assert call["bound"] == "hbm" and call["peak"] == 8000.0 and abs(call["frac"] - call["achieved"] / call["peak"]) < 1e-12
    assert abs(call["achieved"] - call["algorithmic_bytes"] / (d["ms_per_step"] * 1e-3) / 1e9) < 1e-6 * call["achieved"]
    assert d["clock_warmup"]["calls"] >= 0
    other = d["other_configs"]                     # the tiny call, the single layer and the streaming use
    assert [o["workload"][:2] for o in other] == ["c1", "c2", "c4"] and all(o["value"] > 0 for o in other)
    cb = d["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["cores"] >= 1 and cb["value"] > 0 and "units" in cb["sample"]
