"""The benchmark's output contract, on a short run: one JSON line with the fields the driver
reads, a roofline object against the HBM peak, and a refusal of more than one GPU."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*flags):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *flags], cwd=ROOT, capture_output=True,
                          text=True, timeout=600)


def test_more_than_one_gpu_is_refused_with_a_message():
    p = _run("--gpus", "2")
    assert p.returncode != 0
    assert "ONE GPU" in p.stderr and p.stdout.strip() == ""


@pytest.mark.gpu
def test_short_run_prints_one_json_line_with_the_contract_fields(monkeypatch, capsys):
    import runpy

    monkeypatch.setattr(sys, "argv", ["bench.py", "--steps", "6", "--warmup", "2", "--no-cpu-baseline", "--sweep", "quick"])
    monkeypatch.chdir(ROOT)
    runpy.run_path(os.path.join(ROOT, "bench.py"), run_name="__main__")
    lines = [ln for ln in capsys.readouterr().out.splitlines() if ln.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    assert d["metric"] == "verified_tokens_per_s" and d["unit"] == "tokens/s"
    assert d["n_gpus"] == 1 and d["steps"] == 6 and d["warmup"] == 2
    assert d["higher_is_better"] is True and d["vs_baseline"] is None and d["data"] == "synthetic"
    assert "workload" in d["config"] and "model" not in d["config"]
    assert abs(d["value"] - 8 / (d["ms_per_step"] * 1e-3)) <= 1e-6 * d["value"]  # r = 8 rows per step
    rf = d["roofline"]
    assert rf["bound"] == "hbm" and rf["unit"] == "GB/s" and rf["peak"] == 8000.0
    assert abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-9
    assert 0.2 < rf["frac"] < 1.0
    assert abs(rf["achieved"] - d["algorithmic_bytes_per_step"] / (rf["avg_launch_us"] * 1e-6) / 1e9) <= 1e-6 * rf["achieved"]
    assert rf["traffic"] is None or rf["traffic"] >= 0.9 * d["algorithmic_bytes_per_step"]
    # the other synthetic configurations ride in the same line
    sw = d["sweep"]
    assert not [e for e in sw if "section" in e], [e for e in sw if "section" in e]  # no section failed
    pts = [e for e in sw if e.get("kind") not in ("cache_loop", "concurrent_loop", "draft_level")]
    assert pts and all(e["ms_per_step"] > 0 and 0.1 < e["hbm_frac"] < 1.0 and e["verified_tokens_per_s"] > 0 for e in pts)
    conc = [e for e in sw if e.get("kind") == "concurrent_loop"]
    assert conc and all("error" in e or (e["text_equals_plain_decode"] and e["accepted_tokens_per_s"] > 0) for e in conc)
    pts = [e for e in pts if e.get("kind") != "concurrent_loop"]
    dl = [e for e in sw if e.get("kind") == "draft_level"]
    assert len(dl) == 2 and all(e["ms_per_level"] > 0 and e["calls_per_level"] == (e["K"] + 31) // 32 for e in dl)
    assert sorted(e["calls_side_by_side"] for e in dl) == [1, 2]
    loops = [e for e in sw if e.get("kind") == "cache_loop"]
    assert loops and all("error" in e or (e["accepted_tokens_per_s"] > 0 and 1.0 <= e["mean_accepted_len"] <= e["r"])
                         for e in loops)


@pytest.mark.gpu
def test_timeline_probe_reports_the_ten_phases_of_a_layer(monkeypatch, capsys):
    """bench.py --timeline: the kernel's own time stamps of one decoder layer, on the smallest shape."""
    import runpy

    monkeypatch.setattr(sys, "argv", ["bench.py", "--shape", "tiny", "--timeline", "1", "--sweep", "none", "--no-cpu-baseline"])
    monkeypatch.chdir(ROOT)
    runpy.run_path(os.path.join(ROOT, "bench.py"), run_name="__main__")
    lines = [ln for ln in capsys.readouterr().out.splitlines() if ln.strip()]
    assert len(lines) == 1
    t = json.loads(lines[0])["timeline"]
    assert t["workgroups"] == 256 and len(t["phases"]) == 10
    assert all(v >= 0 for v in t["phases"].values())  # the stamps of a workgroup are in order
    assert 0 < t["layer_total"] < 1000 and abs(sum(t["phases"].values()) - t["layer_total"]) < 0.2 * t["layer_total"] + 1
    assert t["attention_detail"]["workgroups_with_a_task"] >= 1
