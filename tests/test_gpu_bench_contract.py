"""bench.py prints one JSON line with the fields its users rely on (small workload, a few seconds)."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_line_has_the_contract_fields():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", "config0",
                        "--steps", "3", "--warmup", "1", "--cpu-heads", "1", "--cpu-tokens", "2"],
                       capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for k in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better",
              "scaling", "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert k in d, k
    assert d["n_gpus"] == 1 and d["steps"] == 3 and d["warmup"] == 1
    assert d["unit"] == "ms" and d["higher_is_better"] is False and d["vs_baseline"] is None
    assert d["value"] == d["ms_per_step"] > 0
    assert "workload" in d["config"] and "model" not in d["config"]
    rf = d["roofline"]
    assert rf["bound"] == "hbm" and rf["unit"] == "GB/s" and rf["peak"] == 8000.0
    assert abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-12 and rf["achieved"] > 0
    cb = d["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["cores"] >= 1 and cb["value"] > 0 and cb["sample"]
    hm = d["hbm_measured"]
    assert 100.0 < hm["read_stream_1GiB_GBs"] < 8000.0 and 100.0 < hm["copy_1GiB_read_plus_write_GBs"] < 8000.0
    assert 100.0 < hm["gather_256B_rows_of_1GiB_GBs"] < 8000.0
    assert "traffic" in rf and "helper_workgroups_active_after_timed_region" in rf
    assert "seed_workgroups_active_after_timed_region" in rf
    knn = d["build"]["knn_kernel"]
    assert knn["bound"] == "mfma" and knn["achieved"] > 0
