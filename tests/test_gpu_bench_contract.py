"""bench.py prints ONE JSON line with the agreed fields (run here on the reduced workload)."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(300)]
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_json_contract():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", "mid", "--steps", "2",
                          "--warmup", "1", "--cpu-rows", "8", "--secondary", "none"], capture_output=True, text=True, cwd=ROOT)
    assert res.returncode == 0, res.stderr[-2000:]
    lines = [l for l in res.stdout.strip().splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better",
                "scaling", "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 2 and d["warmup"] == 1 and d["higher_is_better"] is True
    assert d["vs_baseline"] is None and d["dtype"] == "bf16" and d["data"] == "synthetic"
    assert "workload" in d["config"] and "model" not in d["config"]
    r = d["roofline"]
    assert r["bound"] == "mfma" and r["unit"] == "TFLOP/s" and r["peak"] == 2500.0
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-12 and "traffic" in r
    assert abs(r["frac_measured"] - r["achieved"] / r["peak_measured"]) < 1e-12   # beside the datasheet figure
    c = d["cpu_baseline"]
    assert c["kind"] == "oracle" and c["cores"] == 1 and c["nproc"] >= 1 and c["value"] > 0
    assert isinstance(c["sample"], str)
    names = [x["call"].split()[0] for x in d["calls"]]
    for n in ("decide", "decide_metric", "gather", "scatter", "mass", "compress", "select", "compact"):
        assert n in names, n
    for x in d["calls"]:
        assert x["ms"] > 0 and abs(x["frac"] - x["achieved"] / x["peak"]) < 1e-12
        assert x["frac_measured"] > x["frac"]        # the measured rates are below the datasheet's
    assert d["value"] > 0 and d["ms_per_step"] > 0
    assert set(d["stage_ms_alone"]) == {"decide", "scatter", "attend", "mass", "compress"}
    assert d["streams"] == "one" and set(d["stage_ms"]) == {"decide", "scatter", "attend", "mass", "compress"}


def test_bench_overlap_mode_runs_mass_and_selection_on_a_second_stream():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", "mid", "--steps", "2",
                          "--warmup", "1", "--no-cpu", "--overlap", "--secondary", "none"], capture_output=True, text=True, cwd=ROOT)
    assert res.returncode == 0, res.stderr[-2000:]
    d = json.loads(res.stdout.strip().splitlines()[-1])
    assert d["streams"].startswith("two") and "compact" in d["stage_ms"] and d["value"] > 0


def test_bench_reports_a_second_workload_in_the_same_line():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", "mid", "--steps", "2",
                          "--warmup", "1", "--no-cpu", "--secondary", "mid"], capture_output=True, text=True,
                         cwd=ROOT)
    assert res.returncode == 0, res.stderr[-2000:]
    d = json.loads(res.stdout.strip().splitlines()[-1])
    assert "secondary" not in d                     # same workload twice: nothing to add
    # the default pair is (C3, C2): checked at full size by the round's bench run, not here


def test_bench_refuses_more_than_one_gpu():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True,
                         text=True, cwd=ROOT)
    assert res.returncode == 2 and "ONE GPU" in res.stderr
