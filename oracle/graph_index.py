"""Oracle of the graph index (integer bookkeeping), written with numpy sorts.

Canonical orders (every array is int32 and must match the library bit for bit):
  * destination-major CSR: edges sorted by (dst, rel, src, input edge id);
  * unique (source node, relation) pairs, the rows of the compact
    materialization of thesis Ch.3 "Compact Tensor Materialization and Data
    Layout": numbered by rank in ascending (rel, src) order, so that the pairs
    of one relation are contiguous (pair_ptr = the thesis's unique_etype_ptr,
    pair_src = its unique_row_idx);
  * runs: maximal groups of CSR-adjacent edges with the same (dst, rel);
    the run length is c_{v,r} of Eq. (rgcn);
  * relrun: run ids sorted by (rel, dst);
  * pair-major transpose: CSR positions sorted by (pair, CSR position);
  * srcpair: pair ids sorted by (src, rel);
  * node-type segments: node ids sorted by (type, id);
  * derived lookups: relrun_dst = run_dst in relrun order; in_pair_tag = in_pair with bit 31 set
    when the pair has a single edge; pair_sel_dst = the pair id, or for a pair with a single edge
    bit 31 | that edge's destination; rel_src_type = node type of the source of
    the relation's first pair (0 for a relation without edges).
Test infrastructure only.
"""
import numpy as np


def build(N, R, src, dst, rel, ntype=None, T=1):
    src = np.asarray(src, np.int64)
    dst = np.asarray(dst, np.int64)
    rel = np.asarray(rel, np.int64)
    E = len(src)
    eid = np.arange(E, dtype=np.int64)
    order = np.lexsort((eid, src, rel, dst))            # last key is the primary one
    in_src, in_rel, in_dst, in_eid = src[order], rel[order], dst[order], eid[order]
    in_ptr = np.concatenate([[0], np.cumsum(np.bincount(dst, minlength=N))])

    pkey = np.unique(rel * N + src)                     # ascending (rel, src)
    pair_rel, pair_src = pkey // N, pkey % N
    pair_ptr = np.searchsorted(pair_rel, np.arange(R + 1), side="left")
    in_pair = np.searchsorted(pkey, in_rel * N + in_src)
    P = len(pkey)

    rkey = in_dst * R + in_rel
    new_run = np.ones(E, bool)
    new_run[1:] = rkey[1:] != rkey[:-1]
    run_start = np.flatnonzero(new_run)
    Q = len(run_start)
    run_ptr = np.concatenate([run_start, [E]])
    run_dst, run_rel = in_dst[run_start], in_rel[run_start]
    in_run = np.cumsum(new_run) - 1 if E else np.zeros(0, np.int64)
    in_cnt = np.diff(run_ptr)[in_run] if E else np.zeros(0, np.int64)
    dst_run_ptr = np.searchsorted(run_dst, np.arange(N + 1), side="left")
    relrun_idx = np.lexsort((run_dst, run_rel))
    relrun_ptr = np.searchsorted(run_rel[relrun_idx], np.arange(R + 1), side="left")

    out_epos = np.lexsort((np.arange(E), in_pair))
    out_ptr = np.concatenate([[0], np.cumsum(np.bincount(in_pair, minlength=P))])
    out_dst = in_dst[out_epos]

    srcpair_idx = np.lexsort((pair_rel, pair_src))
    srcpair_ptr = np.concatenate([[0], np.cumsum(np.bincount(pair_src, minlength=N))])

    nt = np.zeros(N, np.int64) if ntype is None else np.asarray(ntype, np.int64)
    ntype_perm = np.lexsort((np.arange(N), nt))
    ntype_ptr = np.searchsorted(nt[ntype_perm], np.arange(T + 1), side="left")

    TOP = np.int64(1) << 31
    single = np.diff(out_ptr) == 1                       # pairs with exactly one edge
    first_epos = out_epos[out_ptr[:-1][single]] if P else np.zeros(0, np.int64)
    pair_ids = np.arange(P, dtype=np.int64)
    pair_sel_dst = pair_ids.copy()
    pair_sel_dst[single] = TOP | in_dst[first_epos]
    in_pair_tag = np.where(single[in_pair], TOP | in_pair, in_pair) if E else np.zeros(0, np.int64)
    relrun_dst = run_dst[relrun_idx]
    rel_src_type = np.zeros(R, np.int64)
    has = pair_ptr[1:] > pair_ptr[:-1]
    rel_src_type[has] = nt[pair_src[pair_ptr[:-1][has]]]

    def wrap(a):                                         # bit pattern of a uint32 as int32
        a = np.asarray(a, np.int64)
        return np.where(a >= TOP, a - (TOP << 1), a)

    idx = dict(relrun_dst=relrun_dst, in_pair_tag=wrap(in_pair_tag), pair_sel_dst=wrap(pair_sel_dst),
               rel_src_type=rel_src_type,
               in_ptr=in_ptr, in_src=in_src, in_rel=in_rel, in_eid=in_eid, in_pair=in_pair,
               in_run=in_run, in_cnt=in_cnt,
               pair_ptr=pair_ptr, pair_src=pair_src, pair_rel=pair_rel,
               run_ptr=run_ptr, run_dst=run_dst, run_rel=run_rel, dst_run_ptr=dst_run_ptr,
               relrun_ptr=relrun_ptr, relrun_idx=relrun_idx,
               out_ptr=out_ptr, out_epos=out_epos, out_dst=out_dst,
               srcpair_ptr=srcpair_ptr, srcpair_idx=srcpair_idx,
               ntype_ptr=ntype_ptr, ntype_perm=ntype_perm)
    idx = {k: np.ascontiguousarray(v, dtype=np.int32) for k, v in idx.items()}
    idx["P"], idx["Q"] = P, Q
    idx["max_in_degree"] = int(np.diff(in_ptr).max()) if N else 0
    return idx
