"""bench.py's one JSON line on the smallest workload: the keys the benchmark contract names are there, the figures
are consistent with each other, and the oracle baseline is part of the line.  Runs bench.main() in this process."""
import contextlib
import io
import json
import os
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_line_on_the_tiny_workload(monkeypatch):
    sys.path.insert(0, ROOT)
    import bench
    monkeypatch.setattr(sys, "argv", ["bench.py", "--workload", "tiny", "--configs", "none", "--steps", "5",
                                      "--warmup", "2", "--reps", "3", "--cpu-batches", "2"])
    out = io.StringIO()
    with contextlib.redirect_stdout(out):
        assert bench.main() == 0
    lines = [l for l in out.getvalue().splitlines() if l.strip()]
    assert len(lines) == 1, "exactly one line on stdout"
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "ms_per_step_median",
                "higher_is_better", "scaling", "vs_baseline", "dtype", "data", "config", "roofline", "roofline_sampler",
                "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 5 and d["warmup"] == 2 and d["unit"] == "seeds/s"
    assert d["higher_is_better"] is True and d["vs_baseline"] is None and d["data"] == "synthetic"
    assert d["config"]["workload"].startswith("tiny") and "model" not in d["config"]
    batch = 1024
    assert d["value"] == pytest.approx(batch / (d["ms_per_step"] * 1e-3), rel=2e-2)
    assert d["ms_per_step_min"] <= d["ms_per_step_median"] <= d["ms_per_step_max"]
    r = d["roofline"]
    assert r["bound"] in ("hbm", "mfma", "alu") and r["unit"] == "GB/s" and r["peak"] == 8000.0
    assert 0 < r["frac"] <= 1 and r["frac"] == pytest.approx(r["achieved"] / r["peak"], abs=1e-3)
    assert "traffic" in r
    s = d["roofline_sampler"]
    assert 0 < s["frac"] <= 1 and s["bytes_per_call"] > 0 and s["bitmap_atomics_per_call"] > 0
    c = d["cpu_baseline"]
    assert c["kind"] == "oracle" and c["unit"] == "seeds/s" and c["value"] > 0 and c["cores"] >= 1 and c["sample"]
    assert d["value"] > c["value"]
