"""bench.py's one JSON line, on the tiny configuration: the fields the harness reads, their types, and the internal
consistency of the figures (value against its own stream time, the whole step against ms_per_step, roofline
fraction = achieved / peak)."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_line_on_the_tiny_config():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--config", "0", "--steps", "20", "--warmup", "5",
                        "--cpu-baseline-iters", "10"], capture_output=True, text=True, timeout=600, cwd=ROOT)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1, "bench.py prints ONE line on stdout"
    d = json.loads(lines[0])
    for key, typ in (("metric", str), ("value", float), ("unit", str), ("n_gpus", int), ("steps", int), ("warmup", int),
                     ("ms_per_step", float), ("higher_is_better", bool), ("scaling", str), ("dtype", str), ("data", str),
                     ("config", dict), ("roofline", dict), ("cpu_baseline", dict)):
        assert isinstance(d[key], typ), key
    assert d["n_gpus"] == 1 and d["steps"] == 20 and d["warmup"] == 5 and d["vs_baseline"] is None
    assert d["unit"] == "lookups/s" and d["data"] == "synthetic" and d["higher_is_better"] is True
    assert "workload" in d["config"] and "model" not in d["config"]
    assert "fwd+bwd+update" in d["metric"] and "HBM" in d["metric"] and d["backing_table"] == "HBM"
    # value = lookups of a step / median stream time of forward + backward + update
    fbu = d["fwd_bwd_update"]
    n = 256 * 8
    assert d["value"] == fbu["value"] and abs(d["value"] - n / (fbu["median_wall_us_per_step"] * 1e-6)) <= 1e-6 * d["value"]
    whole = d["whole_hot_path"]
    assert abs(whole["value"] - n / (d["ms_per_step"] * 1e-3)) <= 1e-6 * whole["value"]
    assert whole["value"] < d["value"] and whole["loop_ms_per_step"] < d["ms_per_step"]
    for name in ("roofline", "roofline_fwd", "roofline_fwd_bwd_update"):
        rf = d[name]
        assert rf["bound"] == "hbm" and rf["unit"] == "GB/s" and rf["peak"] == 8000.0
        assert abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-12
        assert "traffic" in rf and rf["traffic"] is None          # the counters were read on configs[2], not here
    cpu = d["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["unit"] == "lookups/s" and cpu["cores"] >= 1 and cpu["value"] > 0
    assert isinstance(cpu["sample"], str) and cpu["single_thread"]["cores"] == 1
    assert d["plan"]["ids_per_s"] > 0 and d["cache_apply"]["hbm_table"]["rows_per_s"] > 0
    assert d["pinned_host_end_to_end"]["value"] > 0 and d["pinned_host_end_to_end"]["schedule"] in ("overlapped", "synchronous")
