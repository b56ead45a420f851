"""GPU: bench.py prints ONE JSON line with the fields its contract names (run on the smallest workload)."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_line_has_the_contract_fields():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    print("bench.py --workload tiny", flush=True, file=sys.stderr)
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", "tiny", "--steps", "12", "--warmup", "3",
                        "--images", "2", "--also", "none"], capture_output=True, text=True, timeout=280)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1, lines
    j = json.loads(lines[0])
    for k in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
              "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert k in j, k
    assert j["n_gpus"] == 1 and j["steps"] == 12 and j["warmup"] == 3 and j["higher_is_better"] is True
    assert j["data"] == "synthetic" and j["config"]["workload"] == "tiny" and j["dtype"] == "f32"
    assert j["value"] > 0 and j["ms_per_step"] > 0
    rf = j["roofline"]
    for k in ("bound", "achieved", "peak", "unit", "frac", "traffic"):
        assert k in rf, k
    assert rf["bound"] in ("hbm", "mfma", "alu") and abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-9
    cb = j["cpu_baseline"]
    for k in ("value", "unit", "cores", "kind", "sample"):
        assert k in cb, k
    assert cb["kind"] == "oracle" and cb["value"] > 0 and cb["cores"] >= 1
    # whole images: the spread over seeds travels with the mean
    wi = j["config"]["whole_images"]["image_tokens_per_s"]
    assert wi["n"] == 2 and wi["min"] <= wi["mean"] <= wi["max"] and abs(wi["mean"] - j["value"]) < 1e-6 * j["value"]
