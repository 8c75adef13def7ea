"""The benchmark's output contract: one JSON line with the agreed keys, and a refusal of more than one GPU."""
import contextlib
import io
import json
import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)
import bench  # noqa: E402


def _run(argv):
    out, err = io.StringIO(), io.StringIO()
    with contextlib.redirect_stdout(out), contextlib.redirect_stderr(err):
        rc = bench.main(argv)
    return rc, out.getvalue(), err.getvalue()


def test_more_than_one_gpu_is_refused_with_a_message():
    rc, out, err = _run(["--gpus", "2"])
    assert rc != 0 and out.strip() == ""
    assert "one GPU" in err


@pytest.mark.gpu
def test_default_workload_prints_one_json_line_with_the_agreed_keys():
    rc, out, _ = _run(["--layers", "2", "--steps", "2", "--warmup", "1", "--no-full-prefill"])
    assert rc == 0
    lines = [ln for ln in out.splitlines() if ln.strip()]
    assert len(lines) == 1, "exactly one line on stdout"
    j = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in j, key
    assert j["n_gpus"] == 1 and j["steps"] == 2 and j["warmup"] == 1
    assert j["vs_baseline"] is None and j["data"] == "synthetic" and j["dtype"] == "bf16"
    assert j["higher_is_better"] is True and j["value"] > 0 and j["ms_per_step"] > 0
    assert j["config"]["workload"] == "long_doc_8k" and "model" not in j["config"]
    r = j["roofline"]
    assert r["bound"] == "mfma" and r["unit"] == "TFLOP/s" and r["peak"] == 2500.0
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-3 and r["traffic"] > 0
    c = j["cpu_baseline"]
    assert c["kind"] == "oracle" and c["value"] > 0 and c["cores"] >= 1 and c["sample"] and c["unit"]
