"""bench.py's command-line contract: one JSON line with the agreed fields, the
roofline and cpu_baseline objects, and a refusal of more than one GPU."""

import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BENCH = os.path.join(ROOT, "bench.py")

REQUIRED = {"metric": str, "value": float, "unit": str, "n_gpus": int, "steps": int, "warmup": int,
            "ms_per_step": float, "higher_is_better": bool, "scaling": str, "dtype": str, "data": str, "config": dict,
            "roofline": dict}


def test_more_than_one_gpu_is_refused_with_a_message():
    res = subprocess.run([sys.executable, BENCH, "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert res.returncode != 0
    assert "one GPU" in res.stderr or "--gpus 1" in res.stderr
    assert res.stdout.strip() == "", "no result line when nothing was measured"


def _run(*flags):
    res = subprocess.run([sys.executable, BENCH, *flags], capture_output=True, text=True, timeout=300)
    assert res.returncode == 0, res.stderr[-2000:]
    lines = [ln for ln in res.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1, "exactly one line on stdout"
    return json.loads(lines[0])


def _check_common(out, steps, warmup):
    for key, typ in REQUIRED.items():
        assert key in out, key
        assert isinstance(out[key], typ) or (typ is float and isinstance(out[key], int)), (key, out[key])
    assert "vs_baseline" in out and out["vs_baseline"] is None        # the paper reports no figure for this metric
    assert out["n_gpus"] == 1 and out["steps"] == steps and out["warmup"] == warmup
    assert out["unit"] == "GB/s" and out["higher_is_better"] is True and out["data"] == "synthetic"
    assert "workload" in out["config"] and "model" not in out["config"]
    r = out["roofline"]
    assert r["bound"] == "hbm" and r["unit"] == "GB/s" and r["peak"] == 8000.0
    assert r["frac"] == pytest.approx(r["achieved"] / r["peak"], abs=1e-3)
    assert "traffic" in r
    dense = out["config"]["dense_bytes_per_step"]
    assert out["value"] == pytest.approx(dense / (out["ms_per_step"] * 1e-3) / 1e9, rel=2e-3)


@pytest.mark.gpu
def test_small_workload_prints_one_json_line_with_roofline_and_cpu_baseline():
    out = _run("--workload", "cfg1", "--steps", "3", "--warmup", "1", "--cpu-sample-elems", "200000")
    _check_common(out, 3, 1)
    assert out["config"]["workload"].startswith("cfg1")
    c = out["cpu_baseline"]
    assert c["kind"] == "oracle" and c["unit"] == "GB/s" and c["cores"] >= 1 and c["value"] > 0 and c["sample"]


@pytest.mark.gpu
def test_topk_modes_print_the_same_contract():
    for extra in ((), ("--fused-topk",)):
        out = _run("--workload", "cfg1", "--block", "64", "--topk-frac", "0.05", "--steps", "3", "--warmup", "1",
                   "--no-cpu-baseline", *extra)
        _check_common(out, 3, 1)
        assert out["config"]["topk_blocks_kept"] == round(0.05 * (1 << 20) / 64)
        assert out["roofline"]["kernel"] == ("topk_score_kernel" if extra else "encode_scan_kernel")
