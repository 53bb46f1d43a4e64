"""The benchmark's command-line contract: one JSON line with the agreed fields, and a clear refusal of
more than one GPU (this build runs one pipeline stage on one device)."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and not r.stdout.strip()


@pytest.mark.gpu
@pytest.mark.timeout(600)
def test_one_json_line_with_roofline_and_cpu_baseline():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", "tiny", "--steps", "3", "--warmup", "1", "--no-per-config"],
                       capture_output=True, text=True, timeout=500)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for k in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
              "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert k in d, k
    assert d["n_gpus"] == 1 and d["steps"] == 3 and d["warmup"] == 1 and d["vs_baseline"] is None
    assert d["config"]["workload"] == "tiny" and d["dtype"] == "f32" and d["data"] == "synthetic"
    assert abs(d["value"] - 16 / (d["ms_per_step"] * 1e-3)) < 1e-2 * d["value"]
    roof = d["roofline"]
    assert roof["bound"] in ("hbm", "mfma", "alu") and roof["peak"] > 0
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-3
    cb = d["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["value"] > 0 and cb["cores"] >= 1 and "sample" in cb


def test_cpu_baseline_samples_whole_micro_batches():
    """The oracle leg of the benchmark: a sample below one micro-batch takes the first samples of micro-batch 0, a
    larger one whole micro-batches in schedule order; the rate counts exactly the samples that were run."""
    sys.path.insert(0, ROOT)
    import bench
    from stage_inputs import configs as C
    st = C.FULL["tiny"]()
    mb = st["micro_batch"]
    part = bench.cpu_baseline(st, mb - 1)
    assert part["kind"] == "oracle" and part["value"] > 0 and ("%d samples of micro-batch 0" % (mb - 1)) in part["sample"]
    two = bench.cpu_baseline(st, 2 * mb)
    assert ("micro-batches 0..1 (%d samples)" % (2 * mb)) in two["sample"] and two["cores"] >= 1
