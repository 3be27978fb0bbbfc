"""bench.py's command line, as far as it can be checked without a GPU: more than one GPU is refused
with a message, and the algorithmic byte / flop counts it prices the kernels with are consistent."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "one GPU" in (r.stdout + r.stderr)


def test_algorithmic_work_counts():
    sys.path.insert(0, ROOT)
    import bench
    E, N, P, Q, R, T, d, H, P1 = 1000, 100, 700, 400, 5, 1, 64, 1, 500
    row = d * 4
    bound, nbytes, flops = bench.algorithmic_work("aggregate_fwd", E, N, P, Q, R, T, d, H, P1)
    assert bound == "hbm" and nbytes == E * (row + 8) + N * (row + 8) and flops == 2.0 * E * d
    bound, nbytes, flops = bench.algorithmic_work("typed_linear_bwd", E, N, P, Q, R, T, d, H, P1)
    assert bound == "mfma" and flops == 4.0 * P * d * d
    # dY row + gathered X row + stored row, the gather index, the row selector and the (ds_src, scale) pair per row
    assert nbytes == P * (3 * row + 4) + R * d * d * 4 + P * 4 + P * 8
    # a single-edge pair costs the edge-dot kernel two scalars, not a row, where the row selector is used
    with_sel = bench.algorithmic_work("edge_dot_bwd", E, N, P, Q, R, T, d, H, P1)[1]
    without = bench.algorithmic_work("edge_dot_bwd", E, N, P, Q, R, T, 128, H, P1)[1]
    assert with_sel == E * (row + 16) + N * (2 * row + 8) + P1 * 8
    assert without == E * (512 + 16) + N * (2 * 512 + 8) + P1 * (512 + 4)
    # bf16 rows at width 128 halve the row bytes of the intermediates
    half = bench.algorithmic_work("aggregate_fwd", E, N, P, Q, R, T, 128, 4, 0, bf16=True, layer="hgt")[1]
    assert half == E * (256 + 4 + 16) + N * (256 + 8)


import json

import pytest


@pytest.mark.gpu
def test_bench_line_has_the_contract_fields():
    """One short run of bench.py on the small RGAT workload: exactly one JSON line on stdout with the
    fields the harness reads, the roofline object of the dominant kernel and the oracle's CPU baseline."""
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--config", "2", "--steps", "3", "--warmup", "1"],
                       capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for k in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
              "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert k in d, k
    assert d["n_gpus"] == 1 and d["steps"] == 3 and d["warmup"] == 1 and d["vs_baseline"] is None
    assert d["unit"] == "edges/s" and d["value"] > 0 and d["data"] == "synthetic" and "workload" in d["config"]
    roof = d["roofline"]
    assert roof["bound"] in ("hbm", "mfma", "alu") and roof["unit"] in ("GB/s", "TFLOP/s")
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-9 and "traffic" in roof
    cpu = d["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["value"] > 0 and cpu["cores"] >= 1 and cpu["unit"] == "edges/s" and cpu["sample"]
