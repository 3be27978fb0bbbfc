"""RGCN layer on the GPU vs the CPU oracle, element by element."""
import numpy as np
import pytest

from oracle import layers as O
from paper_2412_04747_amd import synth
from parity import check, TOL_F32, TOL_BF16

pytestmark = pytest.mark.gpu


def _run(N, R, src, dst, rel, p, d, norm, act, self_loop, bwd=True, tag="", dtype="f32", d_in=None):
    import torch
    from paper_2412_04747_amd.harness import Graph, RgcnLayer
    print(f"rgcn case {tag}: N={N} R={R} E={len(src)} d={d} norm={norm} act={act} W0={self_loop}", flush=True)
    g = Graph(N, R, src, dst, rel)
    L = RgcnLayer(g, d, norm, act, self_loop, dtype=dtype, d_in=d_in)
    tol = TOL_BF16 if dtype == "bf16" else TOL_F32
    W0 = p["W0"] if self_loop else None
    L.load(p["X"], p["W"], W0, p["dOut"])
    L.fwd()
    torch.cuda.synchronize()
    want = O.rgcn_fwd(N, src, dst, rel, p["X"], p["W"], W0, norm, act)
    check(L.out, want, tol, "out")
    if bwd:
        if act != "none":
            # the activation's mask is a decision taken from `out`: both sides take it from the same
            # values (the backward call receives `out` as an argument), so that an output within
            # rounding distance of zero cannot flip a whole gradient entry
            L.out.copy_(torch.from_numpy(np.ascontiguousarray(want, dtype=np.float32)))
        L.bwd()
        torch.cuda.synchronize()
        wg = O.rgcn_bwd(N, src, dst, rel, p["X"], p["W"], W0, p["dOut"], norm, act, out=want)
        for k, v in L.grads().items():
            check(v, wg[k], tol, k)
    g.close()


def test_config1_forward():
    c = synth.config(1)
    _run(c["N"], c["R"], c["src"], c["dst"], c["rel"], c, 32, "in_degree_per_rel", "none", False, bwd=False, tag="C1")


@pytest.mark.parametrize("d", [32, 64, 128])
def test_forward_backward_all_options(d):
    rng, src, dst, rel, _ = synth.tiny(40 + d, N=700, R=5, E=6000)
    p = synth.rgcn_params(rng, 700, 5, d, d, self_loop=True)
    _run(700, 5, src, dst, rel, p, d, "in_degree_per_rel", "none", True, tag=f"d{d}")
    _run(700, 5, src, dst, rel, p, d, "none", "relu", True, tag=f"d{d}-relu")
    _run(700, 5, src, dst, rel, p, d, "none", "none", False, tag=f"d{d}-plain")


@pytest.mark.parametrize("d_in,d", [(32, 64), (64, 32)])
def test_input_width_differs_from_output_width(d_in, d):
    rng, src, dst, rel, _ = synth.tiny(45 + d, N=700, R=5, E=6000)
    dst[:800] = 9           # a hub cut into pieces
    p = synth.rgcn_params(rng, 700, 5, d_in, d, self_loop=True)
    _run(700, 5, src, dst, rel, p, d, "in_degree_per_rel", "none", True, tag=f"widths-{d_in}-{d}", d_in=d_in)
    _run(700, 5, src, dst, rel, p, d, "none", "relu", False, tag=f"widths-{d_in}-{d}-relu", d_in=d_in)


def test_hub_and_isolated_nodes():
    rng, src, dst, rel, _ = synth.tiny(50, N=400, R=3, E=3000)
    dst[:1500] = 3          # hub far above the item length, many nodes left without in-edges
    src[:900] = 5           # one (src, rel) pair feeding many edges
    rel[:900] = 1
    p = synth.rgcn_params(rng, 400, 3, 64, 64, self_loop=True)
    _run(400, 3, src, dst, rel, p, 64, "in_degree_per_rel", "none", True, tag="hub")


@pytest.mark.parametrize("dtype,d", [("f32", 64), ("bf16", 128)])
def test_relu_backward_from_the_gpus_own_output(dtype, d):
    """The ReLU mask of the backward call is taken from the `out` the GPU's own forward wrote (the other cases
    hand both sides the oracle's `out`).  So that no mask bit hangs on rounding, the inputs are built with
    every pre-activation at least 1e-3 away from 0: sources and destinations are disjoint node sets and the
    self-loop weight is the identity, hence a destination's own feature row shifts its own pre-activation only (a source's row
    also moves its destinations, so the nudging is repeated until nothing is left inside the margin)."""
    import torch
    from paper_2412_04747_amd.harness import Graph, RgcnLayer
    N, R, E = 800, 4, 6000
    rng = np.random.default_rng(611)
    src = rng.integers(0, N // 2, E).astype(np.int32)
    dst = rng.integers(N // 2, N, E).astype(np.int32)
    dst[:900] = N // 2 + 3                                       # a hub
    rel = rng.integers(0, R, E).astype(np.int32)
    p = synth.rgcn_params(rng, N, R, d, d, self_loop=True)
    p["W0"] = np.eye(d, dtype=np.float32)
    if dtype == "bf16":
        p = {k: synth.round_to_bf16(v) for k, v in p.items()}
    margin = 4e-3 if dtype == "f32" else 3e-2                    # bf16: a step of X's grid is up to 2^-8 of |x|
    for _ in range(4):
        pre = O.rgcn_fwd(N, src, dst, rel, p["X"], p["W"], p["W0"], "in_degree_per_rel", "none")
        near = np.abs(pre) < margin
        if not near.any():
            break
        X = p["X"].astype(np.float64)
        X[near] += np.where(pre[near] >= 0, 2 * margin, -2 * margin)
        p["X"] = synth.round_to_bf16(X.astype(np.float32)) if dtype == "bf16" else X.astype(np.float32)
    pre = O.rgcn_fwd(N, src, dst, rel, p["X"], p["W"], p["W0"], "in_degree_per_rel", "none")
    assert np.abs(pre).min() >= 1e-3
    print(f"rgcn case relu-own-out {dtype} d={d}: min |pre-activation| {np.abs(pre).min():.2e}", flush=True)
    tol = TOL_BF16 if dtype == "bf16" else TOL_F32
    g = Graph(N, R, src, dst, rel)
    L = RgcnLayer(g, d, "in_degree_per_rel", "relu", True, dtype=dtype)
    L.load(p["X"], p["W"], p["W0"], p["dOut"])
    L.fwd(); L.bwd()                                             # `out` stays the GPU's
    torch.cuda.synchronize()
    want = O.rgcn_fwd(N, src, dst, rel, p["X"], p["W"], p["W0"], "in_degree_per_rel", "relu")
    check(L.out, want, tol, "out")
    assert np.array_equal(L.out.cpu().numpy() > 0, want > 0)
    wg = O.rgcn_bwd(N, src, dst, rel, p["X"], p["W"], p["W0"], p["dOut"], "in_degree_per_rel", "relu", out=want)
    for k, v in L.grads().items():
        check(v, wg[k], tol, k)
    g.close()


def test_empty_graph():
    rng = np.random.default_rng(0)
    p = synth.rgcn_params(rng, 10, 2, 32, 32, self_loop=True)
    e = np.zeros(0, np.int32)
    _run(10, 2, e, e, e, p, 32, "in_degree_per_rel", "none", True, tag="empty")


@pytest.mark.parametrize("d", [32, 64, 128])
def test_small_bf16_all_options(d):
    rng, src, dst, rel, _ = synth.tiny(140 + d, N=700, R=5, E=6000)
    dst[:800] = 3
    p = synth.rgcn_params(rng, 700, 5, d, d, self_loop=True)
    p = {k: (None if v is None else synth.round_to_bf16(v)) for k, v in p.items()}
    _run(700, 5, src, dst, rel, p, d, "in_degree_per_rel", "none", True, tag=f"bf16-d{d}", dtype="bf16")
    _run(700, 5, src, dst, rel, p, d, "none", "relu", False, tag=f"bf16-d{d}-relu", dtype="bf16")


@pytest.mark.parametrize("dtype,d", [("f32", 32), ("bf16", 128)])
def test_many_single_entry_segments(dtype, d):
    """Thousands of destinations with one incoming edge, thousands with two to four, and as many
    (source, relation) pairs with one or two edges: the batched single-entry and short-segment
    aggregation paths, forward (destination-major) and backward (pair-major)."""
    rng = np.random.default_rng(77)
    N, R = 12000, 4
    dst = rng.permutation(N).astype(np.int32)              # every node: in-degree at least 1; 7000 of them exactly 1
    more = np.repeat(np.arange(5000, dtype=np.int32), rng.integers(1, 4, 5000))   # 5000 nodes with 2..4 incoming edges
    hub = rng.integers(0, 50, 600).astype(np.int32)        # a few busier ones on top
    dst = np.concatenate([dst, more, hub])
    src = rng.integers(0, N, len(dst)).astype(np.int32)
    rel = rng.integers(0, R, len(dst)).astype(np.int32)
    src[N:N + 6000] = src[:6000]; rel[N:N + 6000] = rel[:6000]   # 6000 (source, relation) pairs with two edges
    p = synth.rgcn_params(rng, N, R, d, d, self_loop=False)
    if dtype == "bf16":
        p = {k: (None if v is None else synth.round_to_bf16(v)) for k, v in p.items()}
    _run(N, R, src, dst, rel, p, d, "in_degree_per_rel", "none", False, tag=f"singles-{dtype}", dtype=dtype)


def test_scaled_config5_bf16():
    c = synth.config(5, scale=0.01)          # knowledge-graph shaped: 500 relations, many with a handful of edges
    _run(c["N"], c["R"], c["src"], c["dst"], c["rel"], c, 128, "in_degree_per_rel", "none", False, tag="C5/100",
         dtype="bf16")


@pytest.mark.timeout(1100)
def test_config5_full_size_bf16():
    """2.5M nodes, 500 relations (100 of them with fewer than 100 edges), 16M edges, d=128, bf16 inputs."""
    c = synth.config(5)
    _run(c["N"], c["R"], c["src"], c["dst"], c["rel"], c, 128, "in_degree_per_rel", "none", False, tag="C5",
         dtype="bf16")
