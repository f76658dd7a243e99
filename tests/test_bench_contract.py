"""bench.py's command line and the JSON line it prints.  Without a GPU: the refusal of more than
one GPU and the bookkeeping of the measured-traffic record; on a GPU: a short run whose one JSON
line must carry every field the benchmark contract names."""
import json
import os
import re
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BENCH = os.path.join(ROOT, "bench.py")


def _run(*args, timeout=600):
    return subprocess.run([sys.executable, BENCH, *args], cwd=ROOT, capture_output=True, text=True, timeout=timeout)


def test_more_than_one_gpu_is_refused_with_a_message():
    res = _run("--gpus", "2")
    assert res.returncode != 0
    assert "one GPU" in (res.stdout + res.stderr)


def test_traffic_record_is_keyed_to_the_kernel_sources():
    sys.path.insert(0, ROOT)
    import bench
    digest = bench.kernel_source_sha256()
    assert re.fullmatch(r"[0-9a-f]{64}", digest)
    assert _run("--kernel-sources-sha256").stdout.strip() == digest
    text = open(bench.TRAFFIC_RECORD).read()
    m = re.search(r"^traffic_bytes_per_launch sample: (\d+) kernel_sources_sha256: ([0-9a-f]{64})$", text, re.M)
    assert m is not None
    got = bench.measured_traffic_bytes()
    if m.group(2) == digest:
        # counters taken with these very sources: reported, and close to the algorithmic bytes
        assert got == int(m.group(1))
        assert 1.0 <= got / (512 * (151_936 * 2 + 16)) < 1.05
    else:
        assert got is None                              # stale record: reported as null


@pytest.mark.gpu
def test_the_json_line_carries_the_contract_fields():
    res = _run("--steps", "5", "--warmup", "2", "--no-other-configs", "--no-restricted")
    assert res.returncode == 0, res.stderr[-2000:]
    lines = [l for l in res.stdout.splitlines() if l.startswith("{")]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better",
                "scaling", "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 5 and d["warmup"] == 2
    assert d["higher_is_better"] is True and d["vs_baseline"] is None and d["data"] == "synthetic"
    assert d["unit"] == "rows/s" and d["value"] > 0
    assert d["value"] == pytest.approx(512 / (d["ms_per_step"] * 1e-3), rel=1e-6)
    assert "workload" in d["config"] and "model" not in d["config"]
    roof = d["roofline"]
    assert roof["bound"] == "hbm" and roof["unit"] == "GB/s" and roof["peak"] == 8000.0
    assert roof["frac"] == pytest.approx(roof["achieved"] / roof["peak"], rel=1e-9)
    assert 0.2 < roof["frac"] < 1.0
    assert roof["traffic"] is None or roof["traffic"] > 1.5e8
    cpu = d["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["unit"] == "rows/s" and cpu["value"] > 0
    assert 1 <= cpu["cores"] <= 16 and isinstance(cpu["sample"], str)
