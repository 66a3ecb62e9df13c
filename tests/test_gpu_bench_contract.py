"""bench.py's one-line contract: a short run prints exactly one JSON line on stdout with the
agreed keys, the roofline and cpu_baseline objects included; more than one GPU is refused."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    res = subprocess.run([sys.executable, "bench.py", "--gpus", "2"], cwd=ROOT, capture_output=True, text=True,
                         timeout=120)
    assert res.returncode != 0
    assert "ONE GPU" in (res.stderr + res.stdout)


@pytest.mark.gpu
def test_a_short_run_prints_one_json_line_with_the_agreed_keys():
    res = subprocess.run([sys.executable, "-u", "bench.py", "--gpus", "1", "--steps", "3", "--warmup", "1"], cwd=ROOT,
                         capture_output=True, text=True, timeout=600)
    assert res.returncode == 0, res.stderr[-2000:]
    lines = [l for l in res.stdout.splitlines() if l.strip()]
    assert len(lines) == 1, lines
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better",
                "scaling", "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 3 and d["warmup"] == 1 and d["higher_is_better"] is True
    assert d["vs_baseline"] is None and d["data"] == "synthetic" and d["dtype"] == "bf16"
    assert "workload" in d["config"] and "model" not in d["config"]
    r = d["roofline"]
    assert r["bound"] == "hbm" and r["unit"] == "GB/s" and r["peak"] == 8000.0
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-3 and 0.3 < r["frac"] < 1.0
    assert r["traffic"] is None or r["traffic"] > 0.9 * r["algorithmic_bytes_per_launch"]
    c = d["cpu_baseline"]
    assert c["kind"] == "oracle" and c["cores"] >= 1 and c["value"] > 0 and c["unit"] == d["unit"] and c["sample"]
    assert d["value"] > 100 * c["value"]          # a sanity bound, not a target
    # the timed run itself is compared with the oracle, and the figure is in the line
    p = d["parity"]
    assert p["attention_within_bar"] and p["attention_max_abs_err"] <= p["bar"] == 2e-3
    for key in ("target_ids_equal", "accepted_equal", "accepted_cu_equal", "out_tokens_equal", "cache_equal"):
        assert p[key] is True, key
    # the whole range of the metric, B = 8 .. 128, is in the same line
    assert [c["config"] for c in d["all_configs"]] == [2, 3, 5] and [c["B"] for c in d["all_configs"]] == [8, 32, 128]
    for c in d["all_configs"]:
        assert c["value"] > 0 and c["ms_per_step"] > 0 and 0.2 < c["roofline"]["frac"] < 1.0
    src = r["traffic_source"]
    assert src is None or (src["stale"] is False) == (r["traffic"] is not None)
