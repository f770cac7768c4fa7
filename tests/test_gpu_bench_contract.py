"""The benchmark's one-line contract on a real GPU: `python bench.py --gpus 1 --steps K --warmup W` prints exactly one
JSON line on stdout with the agreed keys, the roofline object of the dominant kernel and the CPU-oracle baseline."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.timeout(300)
def test_bench_prints_one_json_line_with_the_agreed_fields():
    print("[case] bench.py --gpus 1 --steps 5 --warmup 2 as a child process", flush=True)
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "1", "--steps", "5", "--warmup", "2"],
                       capture_output=True, text=True, timeout=280, cwd=ROOT)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 5 and d["warmup"] == 2 and d["higher_is_better"] is True
    assert d["vs_baseline"] is None and d["data"] == "synthetic" and d["dtype"] == "bf16" and d["unit"] == "voxels/s"
    assert "workload" in d["config"] and "model" not in d["config"]
    assert abs(d["value"] * d["ms_per_step"] * 1e-3 - 30000) < 30                 # value = voxels of one frame / step time
    roof = d["roofline"]
    assert roof["bound"] == "mfma" and roof["peak"] == 2500.0 and roof["unit"] == "TFLOP/s"
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-4 and 0.02 < roof["frac"] < 1.0
    cpu = d["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["cores"] >= 1 and cpu["value"] > 0 and cpu["unit"] == "voxels/s" and cpu["sample"]


@pytest.mark.timeout(200)
def test_phase_clock_tool_prints_its_table():
    """The optional instrumented build of the layer kernel (csrc/phase_clock.h) runs and reports clocks that add up: as
    a child process, so that this process keeps the product library."""
    from paper_2301_06051_amd.build import PHASE_LIB
    if not os.path.exists(PHASE_LIB):
        pytest.skip("instrumented library not built")
    print("[case] python -m paper_2301_06051_amd.phase_clocks --config 2 as a child process", flush=True)
    r = subprocess.run([sys.executable, "-m", "paper_2301_06051_amd.phase_clocks", "--config", "2"],
                       capture_output=True, text=True, timeout=180, cwd=ROOT)
    assert r.returncode == 0, r.stderr[-2000:]
    rows = {l.split("|")[1].strip(): l.split("|")[2].strip() for l in r.stdout.splitlines() if l.startswith("| ") and "---" not in l}
    clocks = lambda k: int(rows[k].replace(",", ""))
    parts = [k for k in rows if k not in ("phase", "whole tile", "rows")]
    assert len(parts) == 8 and all(clocks(k) > 0 for k in parts)
    assert abs(sum(clocks(k) for k in parts) - clocks("whole tile")) <= len(parts)
    assert 10_000 < clocks("whole tile") < 200_000
