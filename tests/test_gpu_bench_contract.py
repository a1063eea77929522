"""bench.py prints one JSON line with the agreed fields: run it briefly on the GPU and check them."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_line_has_the_agreed_fields():
    print("case bench contract", flush=True)
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "5", "--warmup", "2",
                        "--kernel-reps", "2"], capture_output=True, text=True, timeout=600, cwd=ROOT)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.strip().splitlines() if ln.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 5 and d["warmup"] == 2
    assert d["vs_baseline"] is None and d["higher_is_better"] is True and d["data"] == "synthetic"
    assert d["dtype"] == "f32" and "workload" in d["config"] and "model" not in d["config"]
    # the headline is the ImageNet deep-stage bottleneck stack: 36 layers, N = 64
    assert d["config"]["workload"].startswith("config5") and d["config"]["layers"] == 36
    assert d["value"] > 0 and abs(d["value"] - 64 * 36 / (d["ms_per_step"] * 1e-3)) < 1e-6 * d["value"]
    roof = d["roofline"]
    for key in ("bound", "achieved", "peak", "unit", "frac", "traffic"):
        assert key in roof, key
    assert roof["bound"] in ("hbm", "mfma", "alu") and roof["peak"] == 157.3 and roof["unit"] == "TFLOP/s"
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-9 and 0 < roof["frac"] < 1
    cpu = d["cpu_baseline"]
    for key in ("value", "unit", "cores", "kind", "sample"):
        assert key in cpu, key
    assert cpu["kind"] == "oracle" and cpu["value"] > 0 and cpu["cores"] >= 1
    assert cpu["config1_single_thread"]["cores"] == 1 and cpu["config1_single_thread"]["value"] > 0
    assert abs(d["activation_bytes"]["ratio"] - 4 / 32) < 0.01       # K/32 of fp32 (+ row padding)
    big = d["hbm_bound_passes_large"]
    for name in ("read", "write", "copy"):
        assert 0 < big["ceiling_gbs"][name] < 8000.0
    for name in ("pack", "unpack", "bn_relu_pack"):
        assert d["pack_unpack_gbs"][name] > 0
    for name in ("bn_stats", "pack", "unpack", "bn_relu_pack", "bn_bwd"):
        assert 0 < big[name]["frac_of_peak"] < 1 and big[name]["gbs"] > 0
    subs = d["sub_results"]
    assert [x["workload"][:7] for x in subs] == ["config4", "config2", "config4", "config5", "config5"]
    assert all(x["value"] > 0 for x in subs)
    assert subs[4]["K"] == 8 and abs(subs[4]["stored_over_exact"] - 8 / 32) < 0.01
    assert subs[2]["workload"].endswith("--math bf16") and subs[2]["ms_per_step"] < subs[0]["ms_per_step"]
    assert subs[3]["workload"].endswith("--math bf16") and subs[3]["ms_per_step"] < d["ms_per_step"]
