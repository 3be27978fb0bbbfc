"""Pins of the graph-index oracle: brute force with Python sorted() / dicts on
tiny multigraphs, and structural invariants."""
import numpy as np

from oracle import graph_index
from paper_2412_04747_amd import synth


def _brute(N, R, src, dst, rel, ntype, T):
    E = len(src)
    edges = sorted((int(dst[e]), int(rel[e]), int(src[e]), e) for e in range(E))
    pairs = sorted({(int(rel[e]), int(src[e])) for e in range(E)})
    pid = {k: i for i, k in enumerate(pairs)}
    ix = {}
    ix["in_src"] = [s for _, _, s, _ in edges]
    ix["in_rel"] = [r for _, r, _, _ in edges]
    ix["in_eid"] = [e for _, _, _, e in edges]
    ix["in_pair"] = [pid[(r, s)] for _, r, s, _ in edges]
    ix["in_ptr"] = [sum(1 for d, *_ in edges if d < v) for v in range(N + 1)]
    ix["pair_src"] = [s for _, s in pairs]
    ix["pair_rel"] = [r for r, _ in pairs]
    ix["pair_ptr"] = [sum(1 for r, _ in pairs if r < k) for k in range(R + 1)]
    runs, in_run = [], []
    for pos, (d, r, _, _) in enumerate(edges):
        if not runs or runs[-1][:2] != (d, r):
            runs.append((d, r, pos))
        in_run.append(len(runs) - 1)
    ix["in_run"] = in_run
    ix["run_ptr"] = [p for _, _, p in runs] + [E]
    ix["run_dst"] = [d for d, _, _ in runs]
    ix["run_rel"] = [r for _, r, _ in runs]
    ix["in_cnt"] = [sum(1 for (d2, r2, _, _) in edges if (d2, r2) == (d, r)) for d, r, _, _ in edges]
    ix["dst_run_ptr"] = [sum(1 for d, _, _ in runs if d < v) for v in range(N + 1)]
    rr = sorted(range(len(runs)), key=lambda q: (runs[q][1], runs[q][0]))
    ix["relrun_idx"] = rr
    ix["relrun_ptr"] = [sum(1 for _, r, _ in runs if r < k) for k in range(R + 1)]
    tr = sorted(range(E), key=lambda pos: (ix["in_pair"][pos], pos))
    ix["out_epos"] = tr
    ix["out_dst"] = [edges[pos][0] for pos in tr]
    ix["out_ptr"] = [sum(1 for q in ix["in_pair"] if q < p) for p in range(len(pairs) + 1)]
    sp = sorted(range(len(pairs)), key=lambda p: (pairs[p][1], pairs[p][0]))
    ix["srcpair_idx"] = sp
    ix["srcpair_ptr"] = [sum(1 for _, s in pairs if s < v) for v in range(N + 1)]
    perm = sorted(range(N), key=lambda n: (int(ntype[n]), n))
    ix["ntype_perm"] = perm
    ix["ntype_ptr"] = [sum(1 for n in range(N) if ntype[n] < t) for t in range(T + 1)]
    # derived lookups; a set top bit reads as a negative int32
    top = lambda x: x - (1 << 31)
    edges_of = [[pos for pos in range(E) if ix["in_pair"][pos] == p] for p in range(len(pairs))]
    ix["relrun_dst"] = [runs[q][0] for q in rr]
    ix["in_pair_tag"] = [top(p) if len(edges_of[p]) == 1 else p for p in ix["in_pair"]]
    ix["pair_sel_dst"] = [top(edges[edges_of[p][0]][0]) if len(edges_of[p]) == 1 else p for p in range(len(pairs))]
    ix["rel_src_type"] = [next((int(ntype[s]) for r, s in pairs if r == k), 0) for k in range(R)]
    return ix, len(pairs), len(runs)


def test_against_brute_force():
    for seed, (N, R, E, T) in enumerate([(6, 2, 20, 1), (9, 4, 35, 3), (5, 3, 0, 2), (4, 1, 12, 1)]):
        _, src, dst, rel, ntype = synth.tiny(100 + seed, N, R, E, T)
        got = graph_index.build(N, R, src, dst, rel, ntype, T)
        want, P, Q = _brute(N, R, src, dst, rel, ntype, T)
        assert got["P"] == P and got["Q"] == Q
        for k, v in want.items():
            assert got[k].dtype == np.int32
            assert got[k].tolist() == v, k


def test_invariants_on_skewed_graph():
    g = synth.config(2, scale=0.1)
    N, R, E = g["N"], g["R"], g["E"]
    ix = graph_index.build(N, R, g["src"], g["dst"], g["rel"])
    assert ix["in_ptr"][0] == 0 and ix["in_ptr"][-1] == E and np.all(np.diff(ix["in_ptr"]) >= 0)
    assert ix["pair_ptr"][-1] == ix["P"] and ix["run_ptr"][-1] == E
    # every CSR edge maps to the pair holding its (src, rel)
    assert np.array_equal(ix["pair_src"][ix["in_pair"]], ix["in_src"])
    assert np.array_equal(ix["pair_rel"][ix["in_pair"]], ix["in_rel"])
    assert np.array_equal(np.sort(ix["out_epos"]), np.arange(E))
    assert np.array_equal(np.sort(ix["in_eid"]), np.arange(E))
    assert np.array_equal(g["src"][ix["in_eid"]], ix["in_src"])
    # P is the number of distinct (src, rel) pairs: the numerator of the
    # thesis's "entity compaction ratio"
    assert ix["P"] == len(set(zip(g["src"].tolist(), g["rel"].tolist())))
    # permuting the input edges changes only in_eid
    perm = np.random.default_rng(0).permutation(E)
    jx = graph_index.build(N, R, g["src"][perm], g["dst"][perm], g["rel"][perm])
    for k in ix:
        if k != "in_eid":
            assert np.array_equal(ix[k], jx[k]), k
    assert np.array_equal(perm[jx["in_eid"]][np.argsort(perm[jx["in_eid"]])], np.arange(E))
