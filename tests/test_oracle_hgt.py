"""Pins of the HGT oracle: dense masked multi-head attention special case, a
dense matrix formulation with typed weights, softmax invariants, finite
differences."""
import numpy as np

from oracle import layers as O
from paper_2412_04747_amd import synth
from fd import central_fd, assert_close


def _simple_graph(rng, N, E, R, T):
    """At most one edge per ordered (u, v) pair so a dense [N, N] mask can hold it."""
    cells = rng.choice(N * N, size=E, replace=False)
    dst, src = (cells // N).astype(np.int32), (cells % N).astype(np.int32)
    rel = rng.integers(0, R, E, dtype=np.int32)
    ntype = rng.integers(0, T, N, dtype=np.int32)
    return src, dst, rel, ntype


def _params(rng, N, T, R, d, H, mu):
    return {k: (None if v is None else v.astype(np.float64))
            for k, v in synth.hgt_params(rng, N, T, R, d, H, with_mu=mu).items()}


def test_identity_edge_weights_is_masked_multihead_attention():
    # T = 1, W_att = W_msg = I, mu = 1: softmax(Q K^T / sqrt(dh) + mask) V Wo per head
    rng = np.random.default_rng(3)
    N, E, d, H = 9, 30, 8, 2
    dh = d // H
    src, dst, rel, _ = _simple_graph(rng, N, E, 3, 1)
    p = _params(rng, N, 1, 3, d, H, False)
    eye = np.broadcast_to(np.eye(dh), (3, H, dh, dh)).copy()
    got = O.hgt_fwd(N, src, dst, rel, None, p["X"], p["Wk"], p["Wq"], p["Wv"], p["Wo"], eye, eye)
    K, Q, V = p["X"] @ p["Wk"][0], p["X"] @ p["Wq"][0], p["X"] @ p["Wv"][0]
    mask = np.full((N, N), -np.inf)
    mask[dst, src] = 0.0
    Z = np.zeros((N, d))
    for h in range(H):
        sl = slice(h * dh, (h + 1) * dh)
        S = Q[:, sl] @ K[:, sl].T / np.sqrt(dh) + mask
        has = np.isfinite(S).any(1)
        A = np.zeros_like(S)
        A[has] = np.exp(S[has] - S[has].max(1, keepdims=True))
        A[has] /= A[has].sum(1, keepdims=True)
        Z[:, sl] = A @ V[:, sl]
    assert_close(got, Z @ p["Wo"][0], 1e-12)


def test_typed_weights_dense_formulation():
    # dense [N, N] tensors with per-node-type and per-relation weights
    rng = np.random.default_rng(4)
    N, E, d, H, R, T = 10, 40, 6, 3, 4, 3
    dh = d // H
    src, dst, rel, ntype = _simple_graph(rng, N, E, R, T)
    p = _params(rng, N, T, R, d, H, True)
    got, alpha = O.hgt_fwd(N, src, dst, rel, ntype, p["X"], p["Wk"], p["Wq"], p["Wv"], p["Wo"],
                           p["Watt"], p["Wmsg"], p["mu"], want_alpha=True)
    K = np.einsum("ni,nij->nj", p["X"], p["Wk"][ntype]).reshape(N, H, dh)
    Q = np.einsum("ni,nij->nj", p["X"], p["Wq"][ntype]).reshape(N, H, dh)
    V = np.einsum("ni,nij->nj", p["X"], p["Wv"][ntype]).reshape(N, H, dh)
    relmat = np.full((N, N), -1)
    relmat[dst, src] = rel
    L = np.full((N, N, H), -np.inf)
    M = np.zeros((N, N, H, dh))
    for v in range(N):
        for u in range(N):
            r = relmat[v, u]
            if r < 0:
                continue
            for h in range(H):
                L[v, u, h] = p["mu"][r, h] * (K[u, h] @ p["Watt"][r, h] @ Q[v, h]) / np.sqrt(dh)
                M[v, u, h] = V[u, h] @ p["Wmsg"][r, h]
    A = np.zeros_like(L)
    for v in range(N):
        if (relmat[v] >= 0).any():
            A[v] = np.exp(L[v] - L[v].max(0, keepdims=True))
            A[v] /= A[v].sum(0, keepdims=True)
    Z = np.einsum("vuh,vuhj->vhj", A, M).reshape(N, d)
    want = np.einsum("ni,nij->nj", Z, p["Wo"][ntype])
    assert_close(got, want, 1e-12)
    assert_close(alpha, A[dst, src], 1e-12, "alpha")
    s = np.zeros((N, H)); np.add.at(s, dst, alpha)
    assert np.abs(s[np.bincount(dst, minlength=N) > 0] - 1).max() < 1e-12


def test_edge_order_invariance_and_isolated_nodes():
    rng, src, dst, rel, ntype = synth.tiny(21, N=12, R=3, E=30, T=2)
    p = _params(rng, 12, 2, 3, 8, 2, True)
    args = (p["X"], p["Wk"], p["Wq"], p["Wv"], p["Wo"], p["Watt"], p["Wmsg"], p["mu"])
    a = O.hgt_fwd(12, src, dst, rel, ntype, *args)
    perm = rng.permutation(len(src))
    b = O.hgt_fwd(12, src[perm], dst[perm], rel[perm], ntype, *args)
    assert_close(a, b, 1e-12)
    iso = np.bincount(dst, minlength=12) == 0
    if iso.any():
        assert np.all(a[iso] == 0)          # zero aggregate times W_out
    ga = O.hgt_bwd(12, src, dst, rel, ntype, *args, p["dOut"])
    gb = O.hgt_bwd(12, src[perm], dst[perm], rel[perm], ntype, *args, p["dOut"])
    for k in ga:
        assert_close(ga[k], gb[k], 1e-12, k)


def test_backward_matches_finite_differences():
    rng, src, dst, rel, ntype = synth.tiny(22, N=7, R=2, E=20, T=2)
    N, d, H = 7, 4, 2
    p = _params(rng, N, 2, 2, d, H, True)
    G = p["dOut"]
    names = ("X", "Wk", "Wq", "Wv", "Wo", "Watt", "Wmsg", "mu")
    fwd = lambda q: O.hgt_fwd(N, src, dst, rel, ntype, *[q[k] for k in names])
    loss = lambda q: float((fwd(q) * G).sum())
    g = O.hgt_bwd(N, src, dst, rel, ntype, *[p[k] for k in names], G)
    for k in names:
        assert_close(g["d" + k], central_fd(loss, p, k), 2e-6, k)
