"""bench.py and __graft_entry__.smoke() on a small shape: the JSON line carries every field of the measurement
contract, the roofline and CPU-baseline records are filled, and a multi-GPU request is refused."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(args, timeout=300):
    return subprocess.run([sys.executable, "bench.py"] + args, cwd=ROOT, capture_output=True, text=True, timeout=timeout)


@pytest.mark.parametrize("extra", [[], ["--workload", "3", "--f16"], ["--workload", "4", "--bits", "2"]])
def test_bench_json_contract(extra):
    n = "60000" if not extra else "20000"
    r = _run(["--n", n, "--nq", "512", "--steps", "3", "--warmup", "1", "--cpu-queries", "128", "--delete-frac", "0.1"] + extra)
    assert r.returncode == 0, r.stderr[-3000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1, "exactly one JSON line on stdout"
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 3 and d["warmup"] == 1 and d["higher_is_better"] is True
    assert d["unit"] == "queries/s" and d["value"] > 0 and d["data"] == "synthetic" and d["vs_baseline"] is None
    assert "workload" in d["config"] and "model" not in d["config"]
    rf = d["roofline"]
    assert rf["bound"] == "hbm" and rf["unit"] == "GB/s" and rf["peak"] == 8000.0
    assert abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-3 and rf["achieved"] > 0 and rf["kernel_ms"] > 0
    assert rf["kernel"].startswith("beam_search") and rf["traffic"] is None and "traffic_source" in rf
    assert d["config"]["recall_target_met"] == (d["config"]["recall_at_10"] >= 0.95)
    cb = d["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["value"] > 0 and cb["cores"] >= 1 and "sample" in cb
    # the oracle on the exported graph returns what the GPU returned
    assert "identical to the GPU's: 1.0000" in cb["sample"] or extra, cb["sample"]
    assert abs(d["value"] - 512 / (d["ms_per_step"] * 1e-3)) / d["value"] < 0.02
    if "two_batches_in_flight" in d["config"]:   # exact-mode lines: context, never the headline value
        tb = d["config"]["two_batches_in_flight"]
        assert tb["results_equal"] is True and tb["streams"] == 2 and tb["queries_per_s"] > 0
        assert d["value"] != tb["queries_per_s"]
    dl = d["config"]["delete"]
    assert dl["deleted"] == int(0.1 * int(n)) and dl["consolidate_s"] > 0 and dl["compact_s"] >= 0


def test_bench_default_run_covers_the_other_configurations():
    """The default run measures configurations 1, 3, 4 and 5 after the headline; here at 2 % of their sizes."""
    r = _run(["--n", "60000", "--nq", "512", "--steps", "3", "--warmup", "1", "--cpu-queries", "0", "--others-scale", "0.02"], timeout=600)
    assert r.returncode == 0, r.stderr[-3000:]
    d = json.loads([l for l in r.stdout.splitlines() if l.strip()][-1])
    lw = d["config"]["listed_beam_widths"]
    assert [e["L"] for e in lw] == [32, 64, 128, 256] and all(e["queries_per_s"] > 0 and e["kernel"].startswith("beam_search") for e in lw)
    tb = d["config"]["two_batches_in_flight"]
    assert tb["results_equal"] is True and tb["streams"] == 2 and tb["queries_per_s"] > 0
    assert d["config"]["graph_from_final_frontier"]["two_batches_in_flight"]["results_equal"] is True
    others = d["config"]["others"]
    assert [o["workload"].split(":")[0] for o in others] == ["workload 1", "workload 3", "workload 4", "workload 5"]
    for o in others:
        assert o["queries_per_s"] > 0 and 0 < o["recall_at_10"] <= 1 and o["roofline"]["kernel"].startswith("beam_search")
        assert o["roofline"]["kernel_ms"] > 0 and o["roofline"]["bytes_per_launch"] > 0
    assert others[3]["stream"][-1]["N"] == 200000 and others[3]["stream"][-1]["batch_inserts_per_s"] > 0
    assert "centres N(0,0.1^2)" in others[1]["workload"] and "i^-1.0" in others[1]["workload"]


def test_bench_refuses_more_than_one_gpu():
    r = _run(["--gpus", "2"], timeout=60)
    assert r.returncode != 0 and "ONE GPU" in (r.stderr + r.stdout)


def test_smoke_entry():
    r = subprocess.run([sys.executable, "-c", "import __graft_entry__ as g; g.smoke()"], cwd=ROOT, capture_output=True,
                       text=True, timeout=300)
    assert r.returncode == 0, r.stderr[-2000:]
