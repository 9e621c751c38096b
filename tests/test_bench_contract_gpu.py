"""bench.py prints one JSON line with the agreed fields (short run on the GPU)."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run_bench(*args):
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                       timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1, "exactly one line on stdout"
    return json.loads(lines[0])


def test_default_line_has_the_agreed_fields():
    d = run_bench("--steps", "10", "--warmup", "2")
    for key, typ in (("metric", str), ("value", float), ("unit", str), ("n_gpus", int), ("steps", int),
                     ("warmup", int), ("ms_per_step", float), ("higher_is_better", bool), ("scaling", str),
                     ("dtype", str), ("data", str), ("config", dict), ("roofline", dict), ("cpu_baseline", dict)):
        assert isinstance(d[key], typ), key
    assert d["n_gpus"] == 1 and d["steps"] == 10 and d["warmup"] == 2 and d["vs_baseline"] is None
    assert d["unit"] == "TFLOP/s" and d["higher_is_better"] is True and d["data"] == "synthetic"
    assert d["config"]["workload"] == "bert_large_fwd_bwd" and "model" not in d["config"]
    r = d["roofline"]
    assert r["bound"] == "mfma" and r["unit"] == "TFLOP/s" and r["peak"] == 2500.0
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-3
    # the HBM traffic quoted is the stored counter measurement of exactly these kernel sources
    from paper_2208_08124_amd import build
    with open(os.path.join(ROOT, "profiles", "traffic.json")) as fh:
        stored = json.load(fh)
    assert stored["source_id"] == build.source_id(), "profiles/traffic.json was measured on other kernel sources"
    k = stored["kernels"][r["kernel"]]
    assert r["traffic"] == k["fetch_bytes"] + k["write_bytes"] > 0
    # achieved errors against the oracle, and the timed steps once more by HIP events
    p = d["parity"]
    assert p["o_max_abs"] <= 5e-3 and all(p[g + s] <= 1e-2 for g in ("dq", "dk", "dv")
                                          for s in ("_worst_sequence_rel", "_frobenius_rel"))
    assert 0 < d["ms_per_step_events"]["min"] <= d["ms_per_step_events"]["median"]
    c = d["cpu_baseline"]
    assert c["kind"] == "oracle" and c["value"] > 0 and c["cores"] >= 1 and c["unit"] == "TFLOP/s" and c["sample"]
    # value is the useful work of the step over its time
    assert abs(d["value"] - d["useful_flop_per_step"] / (d["ms_per_step"] * 1e-3) / 1e12) < 0.01 * d["value"]


@pytest.mark.parametrize("op,bound", [("unpad", "hbm"), ("layernorm", "hbm"), ("embedding", "hbm")])
def test_other_modes_print_one_line(op, bound):
    d = run_bench("--op", op, "--steps", "5", "--warmup", "1")
    assert d["roofline"]["bound"] == bound and d["value"] > 0 and d["cpu_baseline"]["kind"] == "oracle"
