"""The benchmark's output contract: one JSON line with the fields the driver reads, the roofline object of the
dominant kernel and the timed oracle baseline.  Runs bench.py as the driver does (a child process), on the small
workload c2 so that it takes seconds."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.timeout(600)
@pytest.mark.parametrize("variant", ["full", "half", "vblock"])
def test_bench_prints_one_json_line_with_the_contract_fields(variant):
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", "c2", "--steps", "5", "--warmup", "2",
                        "--variant", variant], capture_output=True, text=True, timeout=500)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 5 and d["warmup"] == 2 and d["higher_is_better"] is True
    assert d["data"] == "synthetic" and d["vs_baseline"] is None and "workload" in d["config"] and "model" not in d["config"]
    assert d["value"] > 0 and abs(d["value"] - d["config"]["ops_per_step"] / (d["ms_per_step"] * 1e-3) / 1e12) <= 0.01 * d["value"] + 0.01
    rf = d["roofline"]
    for key in ("bound", "achieved", "peak", "unit", "frac", "traffic"):
        assert key in rf, key
    assert rf["bound"] == "mfma" and 0 < rf["frac"] < 1 and abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-3
    cb = d["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["value"] > 0 and cb["cores"] >= 1 and cb["sample"]
    assert d["parity_max_rel_err_vs_oracle"] <= 1e-3 + 2.0 ** -10      # fp16 output rounding on top of the parity bar


@pytest.mark.timeout(300)
def test_bench_decode_mode_prints_an_hbm_roofline_line():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--decode", "1,8,3,3000,128", "--steps", "5", "--warmup", "2"],
                       capture_output=True, text=True, timeout=250)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    assert d["metric"] == "decode_attention_kv_stream" and d["unit"] == "GB/s" and d["n_gpus"] == 1 and d["value"] > 0
    rf = d["roofline"]
    assert rf["bound"] == "hbm" and rf["peak"] == 8000.0 and 0 < rf["frac"] < 1 and abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-3
    assert d["cpu_baseline"]["kind"] == "oracle" and d["parity_max_rel_err_vs_oracle"] <= 1e-3 + 2.0 ** -10
    assert d["max_rel_diff_between_the_two_paths"] <= 2.0 ** -9


def test_bench_shape_mode_prints_one_line_per_shape():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--shape", "1,8,384,640,128,1;2,4,256,256,64,0", "--steps", "3", "--warmup", "1"],
                       capture_output=True, text=True, timeout=250)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [json.loads(ln) for ln in r.stdout.splitlines() if ln.strip()]
    assert len(lines) == 2
    assert lines[0]["config"]["workgroups"] == 8 * 3 and lines[0]["config"]["key_blocks_per_workgroup"] == 4.0   # 3, 4 and 5 blocks
    assert lines[1]["config"]["key_blocks_per_workgroup"] == 2.0
    for d in lines:
        assert d["unit"] == "TOPS" and d["value"] > 0 and d["ms_per_step"] > 0 and 0 < d["frac_of_int8_mfma_peak"] < 1
