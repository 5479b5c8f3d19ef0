"""The contract of bench.py's output: ONE JSON line with the agreed keys, for the default
workload (few layers and steps so that the test stays short) and for the decode stages."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench(*args):
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], cwd=ROOT,
                       capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.startswith("{")]
    assert len(lines) == 1, r.stdout[-2000:]
    return json.loads(lines[0])


def _common(d, steps, warmup):
    assert d["n_gpus"] == 1 and d["steps"] == steps and d["warmup"] == warmup
    assert d["value"] > 0 and d["ms_per_step"] > 0
    assert d["higher_is_better"] is True and d["scaling"] == "weak"
    assert d["vs_baseline"] is None and d["dtype"] == "bf16" and d["data"] == "synthetic"
    assert isinstance(d["config"]["workload"], str) and "model" not in d["config"]


def test_default_workload_line():
    d = _bench("--layers", "2", "--steps", "2", "--warmup", "1", "--no-others")
    _common(d, 2, 1)
    assert "other_workloads" not in d
    assert d["unit"] == "tokens/s" and d["config"]["workload"] == "c3_qwen8b_128k_mlp"
    r = d["roofline"]
    assert r["bound"] == "mfma" and r["unit"] == "TFLOP/s" and r["peak"] == 2500.0
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-12 and 0.2 < r["frac"] < 1.0
    assert "traffic" in r
    rc = d["roofline_compact"]
    assert rc["bound"] == "hbm" and rc["unit"] == "GB/s" and rc["peak"] == 8000.0 and 0.3 < rc["frac"] < 1.0
    c = d["cpu_baseline"]
    assert c["kind"] == "oracle" and c["value"] > 0 and c["cores"] >= 1 and c["unit"] == "tokens/s"
    assert isinstance(c["sample"], str) and c["sample"]
    assert d["score_max_rel_err_vs_oracle_sample"] < 1e-2
    st = d["stages_ms_per_layer"]
    assert st["score"] > st["compact"] > st["mask"] > 0
    assert st["mask_compact"] > st["compact"]
    rm = d["roofline_mask_compact"]
    assert rm["bound"] == "hbm" and abs(rm["frac"] - rm["achieved"] / rm["peak"]) < 1e-12
    assert rm["algorithmic_bytes_per_launch"] > rc["algorithmic_bytes_per_launch"]


def test_default_line_carries_the_other_workloads():
    # the default run: the headline workload, then every other configuration on the same clock
    d = _bench("--layers", "2", "--steps", "2", "--warmup", "1")
    _common(d, 2, 1)
    assert d["config"]["workload"] == "c3_qwen8b_128k_mlp" and d["cpu_baseline"]["kind"] == "oracle"
    others = d["other_workloads"]
    names = [o["config"]["workload"] for o in others]
    assert names == ["c1_t1k_linear", "c2_llama8b_32k_mlp", "c4_qwen32b_4x64k_linear",
                     "c4_qwen32b_4x64k_mlp", "c5_qwen8b_decode", "c5_qwen8b_decode+attend",
                     "c3_qwen8b_128k_mlp+fused-norm"]
    for o in others[:4]:
        assert o["value"] > 0 and o["unit"] == "tokens/s"
        assert 0.05 < o["config"]["kept_fraction_measured"] < 0.95
        assert o["roofline"]["frac"] > 0 and o["stages_ms_per_layer"]["mask_compact"] > 0
    assert others[2]["roofline"]["bound"] == "hbm" and others[3]["roofline"]["bound"] == "mfma"
    assert others[4]["us_per_layer_step"] > 0 and others[4]["hip_graph"]["us_per_layer_step"] > 0
    assert others[5]["roofline"]["bound"] == "hbm" and 0.3 < others[5]["roofline"]["frac"] < 1.0
    fn = others[6]
    assert fn["roofline"]["bound"] == "mfma" and 0.2 < fn["roofline"]["frac"] < 1.0
    assert len(fn["ms_per_layer"]) == 4 and all(v > 0 for v in fn["ms_per_layer"].values())


def test_decode_lines():
    d = _bench("--config", "c5_qwen8b_decode", "--layers", "2", "--steps", "4", "--warmup", "2", "--graph")
    _common(d, 4, 2)
    assert d["us_per_layer_step"] > 0 and d["hip_graph"]["us_per_layer_step"] > 0
    d = _bench("--config", "c5_qwen8b_decode", "--stage", "attend", "--layers", "1", "--steps", "2",
               "--warmup", "1")
    _common(d, 2, 1)
    assert d["roofline"]["bound"] == "hbm" and 0.3 < d["roofline"]["frac"] < 1.0
    assert d["cpu_baseline"]["kind"] == "oracle"
