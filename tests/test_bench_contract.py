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
    # dY row + gathered X row + stored row, the gather index, ds_src, the row selector and the single-edge scales
    assert nbytes == P * (3 * row + 4) + R * d * d * 4 + P * 4 + P * 4 + P1 * 4
    # a single-edge pair costs the edge-dot kernel two scalars, not a row, where the row selector is used
    with_sel = bench.algorithmic_work("edge_dot_bwd", E, N, P, Q, R, T, d, H, P1)[1]
    without = bench.algorithmic_work("edge_dot_bwd", E, N, P, Q, R, T, 128, H, P1)[1]
    assert with_sel == E * (row + 16) + N * (2 * row + 8) + P1 * 8
    assert without == E * (512 + 16) + N * (2 * 512 + 8) + P1 * (512 + 4)
    # bf16 rows at width 128 halve the row bytes of the intermediates
    half = bench.algorithmic_work("aggregate_fwd", E, N, P, Q, R, T, 128, 4, 0, bf16=True, layer="hgt")[1]
    assert half == E * (256 + 4 + 16) + N * (256 + 8)
