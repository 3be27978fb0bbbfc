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
    # single-head RGAT: the fused walk reads row + three indices per edge, s_dst per run; out row + (m, s) + item per node
    bound, nbytes, flops = bench.algorithmic_work("aggregate_fwd", E, N, P, Q, R, T, d, H, P1)
    assert bound == "hbm" and nbytes == E * (row + 12) + Q * 4 + N * (row + 16) and flops == 4.0 * E * d
    # with the softmax in a pass of its own (or several heads): row + pair id + one weight per edge and head
    sep = bench.algorithmic_work("aggregate_fwd", E, N, P, Q, R, T, d, H, P1, sched={"fused_softmax": 0, "row_select": 1})
    assert sep[1] == E * (row + 8) + N * (row + 8) and sep[2] == 2.0 * E * d
    assert bench.algorithmic_work("typed_linear_fwd", E, N, P, Q, R, T, d, H, P1)[1] == P * (2 * row + 4) + R * d * d * 4
    bound, nbytes, flops = bench.algorithmic_work("typed_linear_bwd", E, N, P, Q, R, T, d, H, P1)
    assert bound == "mfma" and flops == 4.0 * P * d * d
    # dY row + gathered X row + stored row, the gather index, the row selector and the (ds_src, scale) pair per row
    assert nbytes == P * (3 * row + 4) + R * d * d * 4 + P * 4 + P * 8
    # a single-edge pair costs the edge-dot kernel two scalars, not a row, where the row selector is used
    with_sel = bench.algorithmic_work("edge_dot_bwd", E, N, P, Q, R, T, d, H, P1)[1]
    without = bench.algorithmic_work("edge_dot_bwd", E, N, P, Q, R, T, 128, H, P1)[1]
    assert with_sel == E * (row + 20) + Q * 4 + N * (2 * row + 16) + P1 * 8
    assert without == E * (512 + 20) + Q * 4 + N * (2 * 512 + 16) + P1 * (512 + 4)
    # reuse that is structural is not charged: the runs of a destination are adjacent, its row is read once
    assert bench.algorithmic_work("run_logit", E, N, P, Q, R, T, d, H, P1, n_dst=90)[1] == Q * 12 + 90 * row
    # the small reduce / combine / finish kernels carry no byte model (and so no GB/s figure)
    for name in ("typed_linear_bwd.reduce", "aggregate_fwd.combine", "edge_softmax.finish", "node_linear_q_bwd.reduce"):
        assert bench.algorithmic_work(name, E, N, P, Q, R, T, 128, 4, 0, bf16=True, layer="hgt") is None
    # HGT with bf16 rows: the query linear's backward accumulates into dX only on the unfolded path
    acc = bench.algorithmic_work("node_linear_q_bwd", E, N, P, Q, R, T, 128, 4, 0, bf16=True, layer="hgt", sched={"hgt_folded": 0})[1]
    fold = bench.algorithmic_work("node_linear_q_bwd", E, N, P, Q, R, T, 128, 4, 0, bf16=True, layer="hgt", sched={"hgt_folded": 1})[1]
    assert acc - fold == N * 512
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
    assert "traffic_source" in roof and d["lib_sha16"] and d["schedule"]["fused_softmax"] == 1
    # the dominant kernel is timed over exactly the steps of the timed region (one launch per step here)
    assert roof["launches_timed"] == 3 and roof["avg_ms"] > 0 and d["ms_per_step_with_events_on_every_kernel"] > 0
    assert roof["kernel"] in {k["name"] for k in d["kernels"]}
    # no kernel is priced above the machine: algorithmic GB/s within the HBM peak, TFLOP/s within the fp32 MFMA peak
    for k in d["kernels"]:
        assert k.get("GBps", 0.0) <= 8000.0 and k.get("TFLOPs", 0.0) <= 157.3, k
    for k, v in d["roofline_steps"].items():
        assert 0.0 < v["frac"] <= 1.0 and abs(v["achieved"] - v["bytes"] / v["ms"] / 1e6) < 1e-6 * v["achieved"], k
    assert set(d["roofline_steps"]) == {"S3_traversal_fwd", "S4_traversal_bwd_dst", "S5_traversal_bwd_pair"}
    cpu = d["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["value"] > 0 and cpu["cores"] >= 1 and cpu["unit"] == "edges/s" and cpu["sample"]


def test_counter_traffic_is_tied_to_the_kernel_sources(tmp_path, monkeypatch):
    """roofline.traffic comes from a committed counter summary and is dropped (null, with the reason) as soon as the
    summary was taken from other kernel sources than the ones in the tree."""
    sys.path.insert(0, ROOT)
    import bench
    sha = bench.library_sha16()
    assert len(sha) == 16 and sha == bench.library_sha16()
    f = tmp_path / "traffic.txt"
    monkeypatch.setattr(bench, "TRAFFIC_TSV", str(f))
    f.write_text(f"# header\n# lib_sha16: {sha}\ntyped_linear_bwd\t3000\t2000\n")
    val, src = bench.counter_traffic("typed_linear_bwd", sha)
    assert val == 5000.0 and "not measured by this run" in src
    assert bench.counter_traffic("edge_dot_bwd", sha)[0] is None
    f.write_text("# lib_sha16: 0123456789abcdef\ntyped_linear_bwd\t3000\t2000\n")
    val, src = bench.counter_traffic("typed_linear_bwd", sha)
    assert val is None and "stale" in src
