"""Seeded synthetic inputs for the relational-GNN layer path.

This module only draws random graphs, features and parameters.  It holds none
of the layer arithmetic, so both the CPU oracle's tests and the HIP path's
tests can take their inputs from it without sharing any of the method's code.

The five named workloads mirror the shapes of the heterogeneous graphs the
thesis evaluates on (Table "Heterogeneous graph datasets": e.g. a
2.5M-node / 16M-edge / ~500-relation knowledge graph, a 1.9M-node / 21M-edge
citation graph with few types), which are not available offline.  Degree and
relation-frequency skew follow power laws because that is what makes the
relation-segmented GEMM and the destination-major traversal hard.
"""
from __future__ import annotations

import numpy as np

SEED0 = 20241204


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bfloat16 (ties to even), returned as fp32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32).astype(np.uint64)
    lsb = (bits >> 16) & 1
    bits = (bits + 0x7FFF + lsb) & 0xFFFF0000
    return bits.astype(np.uint32).view(np.float32).reshape(a.shape)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """Upper 16 bits of already-bf16-representable fp32 values (uint16 storage)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> 16).astype(np.uint16).reshape(a.shape)


def zipf_probs(n: int, s: float) -> np.ndarray:
    p = 1.0 / np.arange(1, n + 1, dtype=np.float64) ** s
    return p / p.sum()


def _categorical(rng, p: np.ndarray, size: int) -> np.ndarray:
    cdf = np.cumsum(p)
    cdf[-1] = 1.0
    u = rng.random(size)
    return np.searchsorted(cdf, u, side="right").astype(np.int32)


def powerlaw_dst(rng, n_nodes: int, n_edges: int, alpha: float, max_deg_target: float) -> np.ndarray:
    """Destinations whose in-degrees follow a capped Pareto(alpha) popularity.

    Node weight w = min((1-u)^(-1/(alpha-1)), w_max); each edge picks its
    destination with probability w / sum(w).  w_max is solved by bisection so
    the most popular node expects `max_deg_target` incoming edges.
    """
    u = rng.random(n_nodes)
    raw = (1.0 - u) ** (-1.0 / (alpha - 1.0))
    lo, hi = 1.0, float(raw.max())
    if n_edges * hi / raw.sum() > max_deg_target:
        for _ in range(80):
            mid = 0.5 * (lo + hi)
            if n_edges * mid / np.minimum(raw, mid).sum() > max_deg_target:
                hi = mid
            else:
                lo = mid
        raw = np.minimum(raw, 0.5 * (lo + hi))
    return _categorical(rng, raw / raw.sum(), n_edges)


def _normal(rng, shape, var: float) -> np.ndarray:
    return (rng.standard_normal(shape) * np.sqrt(var)).astype(np.float32)


def graph_uniform(rng, N, R, E):
    src = rng.integers(0, N, E, dtype=np.int32)
    dst = rng.integers(0, N, E, dtype=np.int32)
    rel = rng.integers(0, R, E, dtype=np.int32)
    return src, dst, rel


def graph_skewed(rng, N, R, E, zipf_s, alpha=2.1, max_deg=None, rel_probs=None):
    src = rng.integers(0, N, E, dtype=np.int32)
    dst = powerlaw_dst(rng, N, E, alpha, max_deg if max_deg else max(N / 20.0, 8.0))
    p = zipf_probs(R, zipf_s) if rel_probs is None else rel_probs
    rel = _categorical(rng, p, E)
    return src, dst, rel


def rgcn_params(rng, N, R, d_in, d_out, self_loop=False, x_var=None):
    g = {}
    g["X"] = _normal(rng, (N, d_in), (1.0 / d_in) if x_var is None else x_var)
    g["W"] = _normal(rng, (R, d_in, d_out), 1.0 / d_in)
    g["W0"] = _normal(rng, (d_in, d_out), 1.0 / d_in) if self_loop else None
    g["dOut"] = _normal(rng, (N, d_out), 1.0)
    return g


def rgat_params(rng, N, R, d_in, d_out, x_var=1.0):
    g = {}
    g["X"] = _normal(rng, (N, d_in), x_var)
    g["W"] = _normal(rng, (R, d_in, d_out), 1.0 / d_in)
    g["w_s"] = _normal(rng, (R, d_out), 1.0 / d_out)
    g["w_t"] = _normal(rng, (R, d_out), 1.0 / d_out)
    g["dOut"] = _normal(rng, (N, d_out), 1.0)
    return g


def hgt_params(rng, N, T, R, d, H, with_mu=False):
    dh = d // H
    g = {}
    g["X"] = _normal(rng, (N, d), 1.0)
    for k in ("Wk", "Wq", "Wv", "Wo"):
        g[k] = _normal(rng, (T, d, d), 1.0 / d)
    g["Watt"] = _normal(rng, (R, H, dh, dh), 1.0 / dh)
    g["Wmsg"] = _normal(rng, (R, H, dh, dh), 1.0 / dh)
    g["mu"] = (1.0 + 0.25 * rng.standard_normal((R, H))).astype(np.float32) if with_mu else None
    g["dOut"] = _normal(rng, (N, d), 1.0)
    return g


def typed_graph(rng, N, T, R, E, type_zipf=1.0, rel_zipf=1.0, alpha=2.1, max_deg_frac=1.0 / 20):
    """Nodes of T types (sizes ~ Zipf, ids contiguous per type, i.e. presorted
    by type as the thesis's setup does) and R relations, each tied to one
    (source type, destination type) pair."""
    sizes = np.maximum(1, np.floor(zipf_probs(T, type_zipf) * N)).astype(np.int64)
    sizes[0] += N - sizes.sum()
    start = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    ntype = np.repeat(np.arange(T, dtype=np.int32), sizes)
    rel_st = rng.integers(0, T, R, dtype=np.int32)
    rel_dt = rng.integers(0, T, R, dtype=np.int32)
    rel = _categorical(rng, zipf_probs(R, rel_zipf), E)
    order = np.argsort(rel, kind="stable")
    rel = rel[order]
    src = np.empty(E, np.int32)
    dst = np.empty(E, np.int32)
    cnt = np.bincount(rel, minlength=R)
    off = 0
    for r in range(R):
        c = int(cnt[r])
        if c == 0:
            continue
        st, dt = int(rel_st[r]), int(rel_dt[r])
        src[off:off + c] = start[st] + rng.integers(0, sizes[st], c)
        nd = int(sizes[dt])
        dst[off:off + c] = start[dt] + powerlaw_dst(rng, nd, c, alpha, max(8.0, nd * max_deg_frac))
        off += c
    perm = rng.permutation(E)
    return src[perm], dst[perm], rel[perm], ntype, rel_st, rel_dt


# ----------------------------------------------------------------------------
# Named workloads
# ----------------------------------------------------------------------------

def config(cid: int, scale: float = 1.0, graph_only: bool = False) -> dict:
    """Workload `cid` in 1..5.  `scale` < 1 shrinks node and edge counts (used
    by CPU-side tests); 1.0 is the size the benchmark and full-size parity
    tests run.  `graph_only` leaves the feature and weight tensors out (the
    graph is drawn first, so it is the same either way)."""
    rng = np.random.default_rng(SEED0 + cid)
    s = lambda n: max(16, int(round(n * scale)))
    if cid == 1:      # RGCN fwd, fp32
        N, R, E, d = s(1000), 8, s(10000), 32
        src, dst, rel = graph_uniform(rng, N, R, E)
        g = dict(layer="rgcn", dtype="f32", N=N, T=1, R=R, E=E, d_in=d, d_out=d, H=1,
                 norm="in_degree_per_rel", src=src, dst=dst, rel=rel)
        params = lambda: rgcn_params(rng, N, R, d, d)
    elif cid == 2:    # RGAT fwd+bwd, fp32
        N, R, E, d = s(20000), 50, s(200000), 64
        src, dst, rel = graph_skewed(rng, N, R, E, 1.1, 2.1)
        g = dict(layer="rgat", dtype="f32", N=N, T=1, R=R, E=E, d_in=d, d_out=d, H=1,
                 slope=0.2, src=src, dst=dst, rel=rel)
        params = lambda: rgat_params(rng, N, R, d, d)
    elif cid == 3:    # RGAT fwd+bwd, fp32, headline
        N, R, E, d = s(1000000), 200, s(10000000), 64
        src, dst, rel = graph_skewed(rng, N, R, E, 1.2, 2.1, max_deg=50000.0 * scale)
        g = dict(layer="rgat", dtype="f32", N=N, T=1, R=R, E=E, d_in=d, d_out=d, H=1,
                 slope=0.2, src=src, dst=dst, rel=rel)
        params = lambda: rgat_params(rng, N, R, d, d)
    elif cid == 4:    # HGT fwd+bwd, bf16 inputs
        N, T, R, E, d, H = s(2000000), 8, 30, s(20000000), 128, 4
        src, dst, rel, ntype, rst, rdt = typed_graph(rng, N, T, R, E)
        g = dict(layer="hgt", dtype="bf16", N=N, T=T, R=R, E=E, d_in=d, d_out=d, H=H,
                 src=src, dst=dst, rel=rel, ntype=ntype, rel_src_ntype=rst, rel_dst_ntype=rdt)
        params = lambda: hgt_params(rng, N, T, R, d, H)
    elif cid == 5:    # RGCN fwd+bwd, knowledge-graph shaped, bf16 inputs
        N, R, E, d = s(2500000), 500, s(16000000), 128
        # 400 Zipf(1.0) relations plus a tail of 100 relations with 1..99 edges each
        tail = rng.integers(1, 100, 100).astype(np.float64) * scale
        head = zipf_probs(400, 1.0) * (E - tail.sum())
        p = np.concatenate([head, tail])
        src, dst, rel = graph_skewed(rng, N, R, E, 1.0, 2.1, max_deg=50000.0 * scale, rel_probs=p / p.sum())
        g = dict(layer="rgcn", dtype="bf16", N=N, T=1, R=R, E=E, d_in=d, d_out=d, H=1,
                 norm="in_degree_per_rel", src=src, dst=dst, rel=rel)
        params = lambda: rgcn_params(rng, N, R, d, d, x_var=1.0)
    else:
        raise ValueError(cid)
    if not graph_only:
        g.update(params())
    if g["dtype"] == "bf16":
        for k, v in list(g.items()):
            if isinstance(v, np.ndarray) and v.dtype == np.float32:
                g[k] = round_to_bf16(v)
    g["cid"] = cid
    return g


def tiny(seed: int, N=10, R=3, E=30, T=1):
    """Small uniform random multigraph (duplicates and self-loops allowed)."""
    rng = np.random.default_rng(seed)
    src, dst, rel = graph_uniform(rng, N, R, E)
    ntype = rng.integers(0, T, N, dtype=np.int32) if T > 1 else np.zeros(N, np.int32)
    return rng, src, dst, rel, ntype
