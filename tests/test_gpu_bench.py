"""bench.py end to end on the smallest configuration: one JSON line with the fields the measurement contract
names, the extras object, and a product rate that agrees with a direct timing of the same call."""
import json
import sys

import pytest

pytestmark = pytest.mark.gpu


def test_bench_line_on_the_small_configuration(capsys, monkeypatch):
    import bench

    monkeypatch.setattr(sys, "argv", ["bench.py", "--config", "1", "--steps", "3", "--warmup", "1", "--extras"])
    bench.main()
    lines = [ln for ln in capsys.readouterr().out.splitlines() if ln.startswith("{")]
    assert len(lines) == 1
    res = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in res, key
    assert res["n_gpus"] == 1 and res["steps"] == 3 and res["vs_baseline"] is None and res["dtype"] == "f32"
    assert res["config"]["workload"].startswith("cfg1") and "model" not in res["config"]
    assert res["value"] > 0 and abs(res["value"] * res["matvec_ms"] - 1000.0) < 1e-6 * 1000.0
    roof = res["roofline"]
    assert roof["bound"] in ("mfma", "hbm") and roof["peak"] > 0 and roof["launches"] > 0
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-12
    cpu = res["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["value"] > 0 and cpu["cores"] >= 1
    ex = res["extras"]
    assert ex["partitions"] >= 1 and ex["matvec_partition_ms"] > 0 and ex["matvec_rop_ms"] > 0
    assert ex["newton_ms_per_iteration"] > 0
