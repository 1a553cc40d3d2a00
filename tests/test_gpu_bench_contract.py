"""The benchmark's output contract, on the small configuration: one JSON line with the metric, the
per-stage times, the roofline object of the dominant kernel and the CPU-oracle baseline."""
import io
import json
import os
import sys
from contextlib import redirect_stdout

import pytest

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402


def test_one_json_line_with_roofline_and_cpu_baseline(monkeypatch):
    monkeypatch.setattr(sys, "argv", ["bench.py", "--config", "0", "--steps", "2", "--warmup", "1", "--no-supplementary"])
    buf = io.StringIO()
    with redirect_stdout(buf):
        bench.main()
    lines = [ln for ln in buf.getvalue().splitlines() if ln.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 2 and d["warmup"] == 1 and d["higher_is_better"] is False
    assert d["unit"] == "ms/layer" and d["value"] > 0 and abs(d["value"] - d["ms_per_step"]) < 1e-9
    assert d["dtype"] == "bf16" and d["data"] == "synthetic" and "workload" in d["config"]
    r = d["roofline"]
    assert r["bound"] == "mfma" and r["unit"] == "TFLOP/s" and r["peak"] == 2500.0
    assert 0 < r["frac"] < 1 and abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-9
    c = d["cpu_baseline"]
    assert c["kind"] == "oracle" and c["cores"] >= 1 and c["value"] > 0 and c["unit"] == "ms/layer" and c["sample"]
    st = d["stages_ms"]
    assert abs(st["search"] + st["threshold"] + st["sparse_attention"] - st["end_to_end"]) < 0.25 * st["end_to_end"]
    # the oracle agrees with the GPU on the rows it was timed on
    assert c["parity_on_sample"]["score_max_rel_err"] < 5e-4 and c["parity_on_sample"]["O_max_abs_err"] < 2e-2
