"""The schedule / layout choice of the library: rgnn_schedule on real graphs agrees with the host-side pick made from
the edge list alone, and every forced alternative (desc.flags) gives the oracle's results too."""
import ctypes as C
import os
import subprocess
import tempfile

import numpy as np
import pytest

from oracle import layers as O
from paper_2412_04747_amd import synth
from parity import check, TOL_F32, TOL_BF16
import test_work_lists as WL

pytestmark = pytest.mark.gpu
HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.fixture(scope="module")
def wl():
    out = os.path.join(tempfile.mkdtemp(prefix="rgnn_wl_"), "libwl.so")
    subprocess.check_call(["g++", "-O1", "-std=c++17", "-shared", "-fPIC", "-o", out, os.path.join(HERE, "host", "work_lists_shim.cpp")])
    return C.CDLL(out)


@pytest.mark.parametrize("cid,scale", [(1, 1.0), (2, 1.0), (3, 0.05), (4, 0.02), (5, 0.05)])
def test_library_pick_equals_host_pick(wl, cid, scale):
    from paper_2412_04747_amd import binding as B
    from paper_2412_04747_amd.harness import Graph
    c = synth.config(cid, scale, graph_only=True)
    print(f"schedule case config {cid} x {scale}: N={c['N']} E={c['E']}", flush=True)
    g = Graph(c["N"], c["R"], c["src"], c["dst"], c["rel"], c.get("ntype") if c["T"] > 1 else None, c["T"])
    k = WL.graph_counts(c)
    layer = WL.LAYER[c["layer"]]
    for flags in (0, 2, 4, 8, 2 | 4 | 8) + ((16, 1) if c["layer"] == "rgat" else ()):
        for heads in ((1, 4) if c["layer"] == "rgat" and not flags & 17 else (c["H"],)):
            desc = B.make_desc(B.RGNN_BF16 if c["dtype"] == "bf16" else B.RGNN_F32, c["d_out"], c["d_out"], heads, flags=flags)
            got = B.rgnn_schedule(g.handle, layer, desc)
            want = WL.pick(wl, c, k, heads=heads, flags=flags)
            got.pop("tile_chunks"); got.pop("wide_chunks"); want.pop("tile_chunks"); want.pop("wide_chunks")
            assert got == want, (flags, heads, {f: (got[f], want[f]) for f in got if got[f] != want[f]})
    g.close()


def _hub_graph(seed, N, R, E, T=1):
    rng, src, dst, rel, ntype = synth.tiny(seed, N=N, R=R, E=E, T=T)
    dst[:E // 5] = 3
    src[E // 5:E // 3] = 5; rel[E // 5:E // 3] = 1
    return rng, src, dst, rel, ntype


@pytest.mark.parametrize("flags", [2, 4, 16, 2 | 4 | 16, 1 | 2 | 4])
@pytest.mark.parametrize("d", [32, 64])
def test_rgat_forced_alternatives(flags, d):
    import torch
    from paper_2412_04747_amd.harness import Graph, RgatLayer
    N, R, E = 9000, 6, 40000
    rng, src, dst, rel, _ = _hub_graph(700 + d, N, R, E)
    print(f"schedule case rgat flags={flags} d={d}", flush=True)
    p = synth.rgat_params(rng, N, R, d, d)
    g = Graph(N, R, src, dst, rel)
    L = RgatLayer(g, d, flags=flags)
    L.load(p["X"], p["W"], p["w_s"], p["w_t"], p["dOut"])
    L.fwd(); L.bwd()
    torch.cuda.synchronize()
    check(L.out, O.rgat_fwd(N, src, dst, rel, p["X"], p["W"], p["w_s"], p["w_t"]), TOL_F32, "out")
    wg = O.rgat_bwd(N, src, dst, rel, p["X"], p["W"], p["w_s"], p["w_t"], p["dOut"])
    for k, v in L.grads().items():
        check(v, wg[k], TOL_F32, k)
    g.close()


@pytest.mark.parametrize("flags", [2, 4, 2 | 4])
def test_rgcn_bf16_forced_alternatives(flags):
    import torch
    from paper_2412_04747_amd.harness import Graph, RgcnLayer
    N, R, E, d = 9000, 6, 40000, 128
    rng, src, dst, rel, _ = _hub_graph(721, N, R, E)
    print(f"schedule case rgcn bf16 flags={flags}", flush=True)
    p = {k: (None if v is None else synth.round_to_bf16(v)) for k, v in synth.rgcn_params(rng, N, R, d, d).items()}
    g = Graph(N, R, src, dst, rel)
    L = RgcnLayer(g, d, "in_degree_per_rel", "none", False, dtype="bf16", flags=flags)
    L.load(p["X"], p["W"], None, p["dOut"])
    L.fwd(); L.bwd()
    torch.cuda.synchronize()
    want = O.rgcn_fwd(N, src, dst, rel, p["X"], p["W"], None, "in_degree_per_rel", "none")
    check(L.out, want, TOL_BF16, "out")
    wg = O.rgcn_bwd(N, src, dst, rel, p["X"], p["W"], None, p["dOut"], "in_degree_per_rel", "none", out=want)
    for k, v in L.grads().items():
        check(v, wg[k], TOL_BF16, k)
    g.close()


@pytest.mark.parametrize("dtype,d", [("f32", 64), ("bf16", 128)])
def test_hgt_unfolded_on_a_graph_that_could_fold(dtype, d):
    import torch
    from paper_2412_04747_amd import binding as B
    from paper_2412_04747_amd.harness import Graph, HgtLayer
    c = synth.config(4, scale=0.002, graph_only=True)
    N, T, R, H = c["N"], c["T"], c["R"], 4
    print(f"schedule case hgt unfolded {dtype} d={d}: N={N} E={c['E']}", flush=True)
    rng = np.random.default_rng(733)
    p = synth.hgt_params(rng, N, T, R, d, H, with_mu=True)
    if dtype == "bf16":
        p = {k: synth.round_to_bf16(v) for k, v in p.items()}
    tol = TOL_BF16 if dtype == "bf16" else TOL_F32
    g = Graph(N, R, c["src"], c["dst"], c["rel"], c["ntype"], T)
    names = ("X", "Wk", "Wq", "Wv", "Wo", "Watt", "Wmsg", "mu")
    want = O.hgt_fwd(N, c["src"], c["dst"], c["rel"], c["ntype"], *[p[k] for k in names])
    wg = O.hgt_bwd(N, c["src"], c["dst"], c["rel"], c["ntype"], *[p[k] for k in names], p["dOut"])
    sizes = {}
    for flags in (0, B.RGNN_FLAG_NO_WEIGHT_FOLDING | B.RGNN_FLAG_NO_BATCHED_WALKS):
        L = HgtLayer(g, d, H, with_mu=True, dtype=dtype, flags=flags)
        assert B.rgnn_schedule(g.handle, B.RGNN_LAYER_HGT, L.desc)["hgt_folded"] == (flags == 0)
        sizes[flags] = B.rgnn_workspace_bytes(g.handle, B.RGNN_LAYER_HGT, L.desc)[2]
        L.load(*[p[k] for k in names], p["dOut"])
        L.fwd(); L.bwd()
        torch.cuda.synchronize()
        check(L.out, want, tol, f"out flags={flags}")
        for k, v in L.grads().items():
            check(v, wg[k], tol, f"{k} flags={flags}")
    assert sizes[0] < max(sizes.values())            # the folded path saves the K and V rows
    g.close()
