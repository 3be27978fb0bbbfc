"""Host planning of the kernels' work lists (tiles/chunks/slots of the typed-linear kernels,
items of the traversal kernels), checked on the CPU against what the kernels rely on.
The planning header is compiled with g++ into a small test library; no GPU is involved."""
import ctypes as C
import os
import subprocess
import tempfile

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
K = dict(tile_rows=0, max_chunks=1, wide_chunks=2, min_chunks=3, chunk_tiles=4, item_max=5, item_target=6, serial_max=7,
         short_len=8)


@pytest.fixture(scope="module")
def wl():
    out = os.path.join(tempfile.mkdtemp(prefix="rgnn_wl_"), "libwl.so")
    subprocess.check_call(["g++", "-O1", "-std=c++17", "-shared", "-fPIC", "-Wall", "-Werror", "-o", out,
                           os.path.join(HERE, "host", "work_lists_shim.cpp")])
    lib = C.CDLL(out)
    lib.wl_item_cut.argtypes = [C.c_longlong]
    return lib


def _field(fn, which, n_hint=1 << 22):
    buf = np.empty(n_hint, np.int32)
    n = fn(which, buf.ctypes.data_as(C.c_void_p), n_hint)
    assert n <= n_hint
    return buf[:n].copy()


def plan_items(lib, ptr, max_len, min_len=0):
    ptr = np.ascontiguousarray(ptr, np.int32)
    n = lib.wl_plan_items(ptr.ctypes.data_as(C.c_void_p), len(ptr) - 1, max_len, min_len)
    names = ("beg", "end", "row", "slot", "split_row", "split_ptr", "part_item", "part_split", "long_item")
    p = {k: _field(lib.wl_items_field, i) for i, k in enumerate(names)}
    sc = np.zeros(6, np.int32)
    lib.wl_items_scalars(sc.ctypes.data_as(C.c_void_p))
    p.update(num_items=n, num_partials=int(sc[0]), num_split=int(sc[1]), first_single=int(sc[2]), num_single=int(sc[3]),
             first_short=int(sc[4]), num_short=int(sc[5]))
    return p


def plan_tiles(lib, seg_ptr, tile_rows, max_chunks):
    seg_ptr = np.ascontiguousarray(seg_ptr, np.int32)
    n = lib.wl_plan_tiles(seg_ptr.ctypes.data_as(C.c_void_p), len(seg_ptr) - 1, tile_rows, max_chunks)
    names = ("tile_seg", "tile_row0", "tile_row1", "chunk_tile", "chunk_slot", "seg_slot_ptr")
    p = {k: _field(lib.wl_tiles_field, i) for i, k in enumerate(names)}
    sc = np.zeros(3, np.int32)
    lib.wl_tiles_scalars(sc.ctypes.data_as(C.c_void_p))
    p.update(num_tiles=n, num_chunks=int(sc[0]), num_slots=int(sc[1]), num_segs=int(sc[2]))
    return p


def _segments(rng, S, hubs):
    """Segment lengths with empty, single-entry, short and a few very long segments."""
    ln = rng.choice([0, 1, 1, 2, 3, 5, 9, 31, 32, 33, 40], size=S)
    for h in hubs:
        ln[rng.integers(0, S)] = h
    return np.concatenate([[0], np.cumsum(ln)]).astype(np.int32)


@pytest.mark.parametrize("max_len,min_len,hubs", [(256, 0, (257, 256, 1000, 5000)), (32, 0, (33, 64, 700)),
                                                   (64, 2, (65, 129, 300)), (1 << 30, 0, (4000,))])
def test_items_cover_each_segment_once(wl, max_len, min_len, hubs):
    rng = np.random.default_rng(7 + max_len % 1000 + min_len)
    ptr = _segments(rng, 3000, hubs)
    p = plan_items(wl, ptr, max_len, min_len)
    serial_max = wl.wl_constant(K["serial_max"])
    n = p["num_items"]
    ln = p["end"] - p["beg"]
    seg_len = np.diff(ptr)
    # every entry of every kept segment lies in exactly one item of that segment; no item is too long
    cover = np.zeros(ptr[-1], np.int32)
    for i in range(n):
        s = p["row"][i]
        assert ptr[s] <= p["beg"][i] <= p["end"][i] <= ptr[s + 1]
        cover[p["beg"][i]:p["end"][i]] += 1
    kept = np.repeat(seg_len >= min_len, seg_len)
    assert (cover[kept] == 1).all() and (cover[~kept] == 0).all()
    assert ln.max() <= max_len
    # whole segments appear once (also the empty ones, which still own an output row), dropped ones never
    whole = p["slot"] < 0
    rows_whole = np.sort(p["row"][whole])
    expect_whole = np.nonzero((seg_len >= min_len) & (seg_len <= max_len))[0]
    assert np.array_equal(rows_whole, expect_whole)
    assert (ln[whole] == seg_len[p["row"][whole]]).all()
    # order: items longer than short_len by length (longest first, pieces before whole segments of the same
    # length), then the short pieces, then the short whole segments by length
    short_len = wl.wl_constant(K["short_len"])
    klass = np.where(ln > short_len, 0, np.where(~(p["slot"] < 0), 1, 2))
    assert (np.diff(klass) >= 0).all()
    for kl in (0, 2):
        sel = np.nonzero(klass == kl)[0]
        assert (np.diff(ln[sel]) <= 0).all()
        same = sel[:-1][np.diff(ln[sel]) == 0]
        assert not ((p["slot"][same] < 0) & (p["slot"][same + 1] >= 0)).any()
    # cut segments: partial rows numbered 0..num_partials-1, grouped per segment in split_ptr order
    cut = np.nonzero(seg_len > max_len)[0]
    assert p["num_split"] == len(cut) and np.array_equal(p["split_row"], cut)
    assert p["split_ptr"][0] == 0 and p["split_ptr"][-1] == p["num_partials"]
    assert np.array_equal(np.sort(p["slot"][~whole]), np.arange(p["num_partials"]))
    for k, s in enumerate(cut):
        a, b = p["split_ptr"][k], p["split_ptr"][k + 1]
        assert b - a == -(-seg_len[s] // max_len)
        items = p["part_item"][a:b]
        assert (p["slot"][items] == np.arange(a, b)).all() and (p["row"][items] == s).all()
        assert (p["part_split"][a:b] == k).all()
        assert p["beg"][items[0]] == ptr[s] and p["end"][items[-1]] == ptr[s + 1]     # pieces in order
        assert (p["beg"][items[1:]] == p["end"][items[:-1]]).all()
    # the single-entry whole segments are one contiguous range
    single = np.nonzero((ln == 1) & whole)[0]
    assert p["num_single"] == len(single)
    if len(single):
        assert p["first_single"] == single[0] and single[-1] == single[0] + len(single) - 1
    # ... preceded directly by the whole segments with 2..short_len entries
    short = np.nonzero((ln >= 2) & (ln <= short_len) & whole)[0]
    assert p["num_short"] == len(short)
    if len(short):
        assert p["first_short"] == short[0] and short[-1] == short[0] + len(short) - 1
        if len(single):
            assert single[0] == short[-1] + 1
    # long items: more than serial_max entries, or any piece of a cut segment
    assert np.array_equal(p["long_item"], np.nonzero((ln > serial_max) | ~whole)[0])


def test_items_keep_segment_order_within_a_length(wl):
    """Stable order: among whole segments of equal length the output rows ascend, which keeps the
    stores of neighbouring lanes close together."""
    rng = np.random.default_rng(3)
    ptr = _segments(rng, 2000, (300,))
    p = plan_items(wl, ptr, 256)
    ln = p["end"] - p["beg"]
    for length in (0, 1, 2, 4, 5):
        rows = p["row"][(ln == length) & (p["slot"] < 0)]
        assert (np.diff(rows) > 0).all()


def test_items_empty_input(wl):
    p = plan_items(wl, np.zeros(1, np.int32), 256)
    assert p["num_items"] == 0 and p["num_partials"] == 0 and p["num_single"] == 0 and list(p["split_ptr"]) == [0]
    p = plan_items(wl, np.zeros(6, np.int32), 256)          # five empty segments
    assert p["num_items"] == 5 and (p["end"] == p["beg"]).all() and p["num_single"] == 0


def test_item_cut_grows_with_the_list(wl):
    lo, hi, target = wl.wl_constant(K["serial_max"]), wl.wl_constant(K["item_max"]), wl.wl_constant(K["item_target"])
    cuts = [wl.wl_item_cut(t) for t in (0, 1, 10_000, 200_000, 3_000_000, 10_000_000, 10**9)]
    assert cuts[0] == lo and cuts[-1] == hi and cuts == sorted(cuts)
    for t, c in zip((200_000, 3_000_000), cuts[3:5]):
        assert c == hi or c * target >= t                   # fine enough to yield `target` items, or at the cap
        assert c & (c - 1) == 0


@pytest.mark.parametrize("S,max_chunks", [(1, 4096), (7, 4096), (200, 4096), (200, 1024), (500, 64)])
def test_tiles_chunks_and_slots(wl, S, max_chunks):
    rng = np.random.default_rng(11 + S)
    ln = rng.choice([0, 1, 63, 64, 65, 200, 5000], size=S)
    ln[rng.integers(0, S)] = 300_000
    seg_ptr = np.concatenate([[0], np.cumsum(ln)]).astype(np.int32)
    T = wl.wl_constant(K["tile_rows"])
    p = plan_tiles(wl, seg_ptr, T, max_chunks)
    nt, nc = p["num_tiles"], p["num_chunks"]
    assert p["num_segs"] == S
    # tiles: in row order, inside one segment, at most T rows, covering every row once
    assert nt == int(np.sum(-(-ln // T)))
    rows = p["tile_row1"] - p["tile_row0"]
    assert (rows > 0).all() and (rows <= T).all()
    assert (seg_ptr[p["tile_seg"]] <= p["tile_row0"]).all() and (p["tile_row1"] <= seg_ptr[p["tile_seg"] + 1]).all()
    assert rows.sum() == seg_ptr[-1] and (p["tile_row0"][1:] >= p["tile_row1"][:-1]).all()
    # chunks: a partition of the tiles into consecutive, nearly equal ranges
    assert nc <= max_chunks and nc <= max(nt, 1)
    ct = p["chunk_tile"]
    assert ct[0] == 0 and ct[-1] == nt and (np.diff(ct) >= 0).all()
    if nc:
        assert np.diff(ct).max() - np.diff(ct).min() <= 1
    # slots: one per (chunk, segment it touches), numbered in chunk order; a segment's slots are consecutive
    slot_of = []
    nxt = 0
    for c in range(nc):
        assert p["chunk_slot"][c] == nxt
        segs = p["tile_seg"][ct[c]:ct[c + 1]]
        for j, s in enumerate(segs):
            if j == 0 or s != segs[j - 1]:
                slot_of.append(s)
                nxt += 1
    assert p["num_slots"] == nxt
    slot_of = np.asarray(slot_of, np.int64)
    assert (np.diff(slot_of) >= 0).all()
    ssp = p["seg_slot_ptr"]
    assert ssp[0] == 0 and ssp[-1] == nxt
    for s in range(S):
        assert (slot_of[ssp[s]:ssp[s + 1]] == s).all()


# ---------------------------------------------------------------- schedule / layout choice per graph

SCHEDULE_FIELDS = ("item_len", "tile_chunks", "wide_chunks", "rows_bf16", "row_select", "hgt_folded", "fused_softmax",
                   "ws_in_lds", "edge_parallel", "dst_batched_single", "dst_batched_short", "pair_walk_multi_only",
                   "pair_batched_single", "pair_batched_short")
LAYER = dict(rgcn=0, rgat=1, hgt=2)


def graph_counts(c):
    """What the choice depends on, counted from the edge list: destinations with one / with 2..4 incoming edges,
    (source, relation) pairs with one / with 2..4 edges, and whether every relation's sources have one node type."""
    N, R = c["N"], c["R"]
    indeg = np.bincount(c["dst"], minlength=N)
    _, outdeg = np.unique(c["rel"].astype(np.int64) * N + c["src"], return_counts=True)
    cnt = lambda deg, lo, hi: int(((deg >= lo) & (deg <= hi)).sum())
    tied = True
    if c["T"] > 1:
        st = c["ntype"][c["src"]]
        tied = all(len(np.unique(st[c["rel"] == r])) <= 1 for r in range(R))
    return dict(dst=(cnt(indeg, 1, 1), cnt(indeg, 2, 4)), pair=(cnt(outdeg, 1, 1), cnt(outdeg, 2, 4)),
                pair_multi=(0, cnt(outdeg, 2, 4)), tied=tied)


def pick(lib, c, k, heads=None, flags=0, dtype=None):
    dt = dtype or c["dtype"]
    a = np.array([LAYER[c["layer"]], 1 if dt == "bf16" else 0, c["d_out"], heads or c["H"], flags, c["R"], int(k["tied"]),
                  c["E"], *k["dst"], *k["pair"], *k["pair_multi"]], dtype=np.int64)
    out = np.zeros(len(SCHEDULE_FIELDS), np.int32)
    lib.wl_pick_schedule(a.ctypes.data_as(C.c_void_p), out.ctypes.data_as(C.c_void_p))
    return dict(zip(SCHEDULE_FIELDS, (int(v) for v in out)))


# The pick for each of the five workloads (tile chunk counts depend on the device's compute-unit count and are
# not part of this table).  Fields not listed are 0.
EXPECTED_PICK = {
    1: dict(item_len=32),
    2: dict(item_len=32, row_select=1, fused_softmax=1, ws_in_lds=1, dst_batched_short=1, pair_walk_multi_only=1,
            pair_batched_short=1),
    3: dict(item_len=256, row_select=1, fused_softmax=1, ws_in_lds=1, dst_batched_single=1, dst_batched_short=1,
            pair_walk_multi_only=1, pair_batched_short=1),
    4: dict(item_len=256, rows_bf16=1, hgt_folded=1, dst_batched_single=1, dst_batched_short=1, pair_batched_single=1,
            pair_batched_short=1),
    5: dict(item_len=256, rows_bf16=1, row_select=1, dst_batched_single=1, dst_batched_short=1, pair_walk_multi_only=1,
            pair_batched_short=1),
}


@pytest.mark.parametrize("cid", [1, 2, 3, 4, 5])
def test_schedule_pick_for_the_five_workloads(wl, cid):
    import sys
    sys.path.insert(0, os.path.dirname(HERE))
    from paper_2412_04747_amd import synth
    c = synth.config(cid, graph_only=True)
    got = pick(wl, c, graph_counts(c))
    want = dict.fromkeys(SCHEDULE_FIELDS, 0)
    want.update(EXPECTED_PICK[cid])
    assert got == want, {k: (got[k], want[k]) for k in got if got[k] != want[k]}


def test_schedule_flags_force_the_alternatives(wl):
    import sys
    sys.path.insert(0, os.path.dirname(HERE))
    from paper_2412_04747_amd import synth
    c = synth.config(2, graph_only=True)
    k = graph_counts(c)
    k["dst"] = (5000, 5000); k["pair"] = (9000, 7000); k["pair_multi"] = (0, 7000)
    base = pick(wl, c, k)
    assert base["dst_batched_single"] and base["dst_batched_short"] and base["pair_batched_short"] and base["row_select"]
    assert base["fused_softmax"] and base["ws_in_lds"] and not base["edge_parallel"]
    nb = pick(wl, c, k, flags=2)
    assert not any(nb[f] for f in ("dst_batched_single", "dst_batched_short", "pair_batched_single", "pair_batched_short"))
    assert {f: v for f, v in nb.items() if "batched" not in f} == {f: v for f, v in base.items() if "batched" not in f}
    assert not pick(wl, c, k, flags=4)["row_select"] and pick(wl, c, k, flags=4)["pair_walk_multi_only"]
    sep = pick(wl, c, k, flags=16)
    assert not sep["fused_softmax"] and not sep["ws_in_lds"] and not sep["edge_parallel"]
    ep = pick(wl, c, k, flags=1)
    assert ep["edge_parallel"] and not ep["fused_softmax"]
    heads = pick(wl, c, k, heads=4)
    assert heads["fused_softmax"] and heads["row_select"] and heads["pair_walk_multi_only"]
    assert not heads["pair_batched_single"]                 # two or four heads: the row selector serves the single-edge pairs
    eight = pick(wl, c, k, heads=8)
    assert eight["fused_softmax"] and not eight["row_select"] and not eight["pair_walk_multi_only"]
    assert eight["pair_batched_single"]                     # other head counts: the pair-major walk takes every pair
    big_r = dict(c, R=300)                                  # 300 x 64 floats = 75 KB: w_s no longer fits the LDS budget
    assert pick(wl, big_r, k)["fused_softmax"] and not pick(wl, big_r, k)["ws_in_lds"]
    c4 = synth.config(4, scale=0.001, graph_only=True)
    k4 = graph_counts(c4)
    assert k4["tied"] and pick(wl, c4, k4)["hgt_folded"] and not pick(wl, c4, k4, flags=8)["hgt_folded"]
    assert not pick(wl, c4, dict(k4, tied=False))["hgt_folded"]
    assert pick(wl, c4, k4, dtype="f32")["rows_bf16"] == 0
