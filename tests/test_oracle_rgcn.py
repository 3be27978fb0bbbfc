"""Pins of the RGCN oracle against what Eq. (rgcn) of the thesis fixes."""
import numpy as np
import scipy.sparse as sp

from oracle import layers as O
from paper_2412_04747_amd import synth
from fd import central_fd, assert_close


def _rand(seed, N=12, R=3, E=40, d_in=5, d_out=4, self_loop=True):
    rng, src, dst, rel, _ = synth.tiny(seed, N, R, E)
    p = synth.rgcn_params(rng, N, R, d_in, d_out, self_loop=self_loop)
    p = {k: (None if v is None else v.astype(np.float64)) for k, v in p.items()}
    return src, dst, rel, p


def test_single_relation_is_spmm():
    # R = 1, no self-loop, c = 1: out = A X W with A[v,u] = multiplicity of u->v
    # (the SpMM form in Ch.3 "RGNN Formulation and Operators"); an ordinary GNN
    # is the one-relation special case.
    src, dst, rel, p = _rand(1, R=1, self_loop=False)
    N = p["X"].shape[0]
    A = sp.coo_matrix((np.ones(len(src)), (dst, src)), shape=(N, N)).tocsr()   # duplicates are summed
    want = (A @ p["X"]) @ p["W"][0]
    got = O.rgcn_fwd(N, src, dst, rel, p["X"], p["W"], None, norm="none")
    assert_close(got, want, 1e-12, "spmm")
    # 1/c with c = in-degree: row-normalised A (mean aggregation)
    deg = np.asarray(A.sum(1)).ravel()
    Dinv = sp.diags(np.where(deg > 0, 1.0 / np.maximum(deg, 1), 0.0))
    got = O.rgcn_fwd(N, src, dst, rel, p["X"], p["W"], None, norm="in_degree_per_rel")
    assert_close(got, (Dinv @ A @ p["X"]) @ p["W"][0], 1e-12, "mean")


def test_multi_relation_closed_form():
    # out = relu( X W0 + sum_r D_r^-1 A_r X W_r ), D_r = per-relation in-degree
    src, dst, rel, p = _rand(2, N=15, R=4, E=80)
    N = 15
    want = p["X"] @ p["W0"]
    for r in range(4):
        m = rel == r
        A = sp.coo_matrix((np.ones(m.sum()), (dst[m], src[m])), shape=(N, N)).tocsr()
        deg = np.asarray(A.sum(1)).ravel()
        want = want + sp.diags(np.where(deg > 0, 1.0 / np.maximum(deg, 1), 0.0)) @ (A @ p["X"]) @ p["W"][r]
    got = O.rgcn_fwd(N, src, dst, rel, p["X"], p["W"], p["W0"], norm="in_degree_per_rel", act="none")
    assert_close(got, want, 1e-12, "multi-rel")
    got = O.rgcn_fwd(N, src, dst, rel, p["X"], p["W"], p["W0"], norm="in_degree_per_rel", act="relu")
    assert_close(got, np.maximum(want, 0), 1e-12, "relu")


def test_zero_in_degree_and_empty_graph():
    N, d = 6, 3
    rng = np.random.default_rng(0)
    X = rng.standard_normal((N, d)); W = rng.standard_normal((2, d, d)); W0 = rng.standard_normal((d, d))
    src = np.array([0, 1], np.int32); dst = np.array([2, 2], np.int32); rel = np.array([0, 1], np.int32)
    out = O.rgcn_fwd(N, src, dst, rel, X, W, None)
    assert np.all(out[[0, 1, 3, 4, 5]] == 0)
    assert_close(out[2], X[0] @ W[0] + X[1] @ W[1], 1e-12)
    e = np.zeros(0, np.int32)
    out = O.rgcn_fwd(N, e, e, e, X, W, W0)
    assert_close(out, X @ W0, 1e-12)


def test_edge_order_invariance():
    src, dst, rel, p = _rand(3)
    N = p["X"].shape[0]
    perm = np.random.default_rng(5).permutation(len(src))
    a = O.rgcn_fwd(N, src, dst, rel, p["X"], p["W"], p["W0"])
    b = O.rgcn_fwd(N, src[perm], dst[perm], rel[perm], p["X"], p["W"], p["W0"])
    assert_close(a, b, 1e-12)
    ga = O.rgcn_bwd(N, src, dst, rel, p["X"], p["W"], p["W0"], p["dOut"])
    gb = O.rgcn_bwd(N, src[perm], dst[perm], rel[perm], p["X"], p["W"], p["W0"], p["dOut"])
    for k in ga:
        assert_close(ga[k], gb[k], 1e-12, k)


def test_backward_matches_finite_differences():
    for act in ("none", "relu"):
        src, dst, rel, p = _rand(4 if act == "none" else 6, N=8, R=3, E=25, d_in=4, d_out=3)
        N = 8
        G = p["dOut"]
        if act == "relu":   # keep away from the kink
            out = O.rgcn_fwd(N, src, dst, rel, p["X"], p["W"], p["W0"], act="none")
            assert np.abs(out).min() > 1e-4
        loss = lambda q: float((O.rgcn_fwd(N, src, dst, rel, q["X"], q["W"], q["W0"], act=act) * G).sum())
        g = O.rgcn_bwd(N, src, dst, rel, p["X"], p["W"], p["W0"], G, act=act)
        for name, key in (("X", "dX"), ("W", "dW"), ("W0", "dW0")):
            assert_close(g[key], central_fd(loss, p, name), 1e-6, f"{act} {key}")
