"""The layer calls stay inside the `workspace` and `saved` sizes that rgnn_workspace_bytes reports:
both buffers sit between guard zones filled with a pattern, which must be intact after forward and
backward (hub nodes, cut pairs and many relations, so that every partial buffer is in use)."""
import numpy as np
import pytest

from paper_2412_04747_amd import synth

pytestmark = pytest.mark.gpu
GUARD = 1 << 20


def _guarded(nbytes):
    import torch
    n = (max(int(nbytes), 256) + 255) // 256 * 256
    big = torch.full((GUARD + n + GUARD,), 0xA5, dtype=torch.uint8, device="cuda")
    return big, big[GUARD:GUARD + n]


def _intact(big, what):
    import torch
    n = big.numel() - 2 * GUARD
    assert bool((big[:GUARD] == 0xA5).all()), f"{what}: wrote below the buffer"
    assert bool((big[GUARD + n:] == 0xA5).all()), f"{what}: wrote past the reported size"


def _graph(seed, N, R, E, T=1):
    rng, src, dst, rel, ntype = synth.tiny(seed, N=N, R=R, E=E, T=T)
    dst[:E // 4] = 3                                   # a hub cut into many pieces
    src[E // 4:E // 2] = 5; rel[E // 4:E // 2] = 1     # one pair with many edges (cut in the pair-major lists)
    return rng, src, dst, rel, ntype


# flags 32: gradients accumulate (the parameter gradients of the call then live in the workspace too)
# d_in: input width where it differs from the output width d
@pytest.mark.parametrize("dtype,d,heads,flags,d_in", [("f32", 64, 1, 0, None), ("f32", 32, 2, 0, None), ("bf16", 128, 4, 0, None),
                                                      ("f32", 128, 1, 0, None), ("f32", 64, 1, 32, None), ("f32", 64, 4, 32, None),
                                                      ("f32", 64, 1, 0, 32), ("f32", 32, 2, 32, 64), ("f32", 64, 4, 0, 32)])
def test_rgat_stays_inside_its_buffers(dtype, d, heads, flags, d_in):
    import torch
    from paper_2412_04747_amd import binding as B
    from paper_2412_04747_amd.harness import Graph, RgatLayer
    rng, src, dst, rel, _ = _graph(501, 3000, 40, 40000)
    print(f"bounds case rgat {dtype} d_in={d_in or d} d={d} heads={heads} flags={flags}", flush=True)
    g = Graph(3000, 40, src, dst, rel)
    L = RgatLayer(g, d, dtype=dtype, heads=heads, flags=flags, d_in=d_in)
    p = synth.rgat_params(rng, 3000, 40, d_in or d, d)
    if dtype == "bf16":
        p = {k: synth.round_to_bf16(v) for k, v in p.items()}
    L.load(p["X"], p["W"], p["w_s"], p["w_t"], p["dOut"])
    f, b, s = B.rgnn_workspace_bytes(g.handle, B.RGNN_LAYER_RGAT, L.desc)
    wf, L.ws = _guarded(f)
    sv, L.saved = _guarded(s)
    L.fwd()
    torch.cuda.synchronize()
    _intact(wf, "forward workspace"); _intact(sv, "saved")
    wb, L.ws = _guarded(b)
    L.bwd()
    torch.cuda.synchronize()
    _intact(wb, "backward workspace"); _intact(sv, "saved")
    g.close()


@pytest.mark.parametrize("dtype,d,act,w0,flags,d_in", [("f32", 64, "relu", True, 0, None), ("bf16", 128, "relu", True, 0, None),
                                                       ("bf16", 128, "none", False, 0, None), ("bf16", 128, "relu", True, 32, None),
                                                       ("f32", 64, "relu", True, 0, 32), ("f32", 32, "none", True, 32, 64)])
def test_rgcn_stays_inside_its_buffers(dtype, d, act, w0, flags, d_in):
    import torch
    from paper_2412_04747_amd import binding as B
    from paper_2412_04747_amd.harness import Graph, RgcnLayer
    rng, src, dst, rel, _ = _graph(502, 3000, 40, 40000)
    print(f"bounds case rgcn {dtype} d_in={d_in or d} d={d} act={act} W0={w0}", flush=True)
    g = Graph(3000, 40, src, dst, rel)
    L = RgcnLayer(g, d, "in_degree_per_rel", act, w0, dtype=dtype, flags=flags, d_in=d_in)
    p = synth.rgcn_params(rng, 3000, 40, d_in or d, d, self_loop=w0)
    if dtype == "bf16":
        p = {k: (None if v is None else synth.round_to_bf16(v)) for k, v in p.items()}
    L.load(p["X"], p["W"], p["W0"], p["dOut"])
    f, b, s = B.rgnn_workspace_bytes(g.handle, B.RGNN_LAYER_RGCN, L.desc)
    wf, L.ws = _guarded(f)
    L.fwd()
    torch.cuda.synchronize()
    _intact(wf, "forward workspace")
    wb, L.ws = _guarded(b)
    L.bwd()
    torch.cuda.synchronize()
    _intact(wb, "backward workspace")
    g.close()


@pytest.mark.parametrize("tied", [False, True])
@pytest.mark.parametrize("dtype,d,H,flags", [("f32", 64, 2, 0), ("bf16", 128, 4, 0), ("bf16", 64, 4, 0), ("bf16", 128, 4, 32), ("f32", 64, 2, 32)])
def test_hgt_stays_inside_its_buffers(dtype, d, H, flags, tied):
    """`tied`: every relation's sources have one node type (the source's type is set by its relation),
    which selects the path with folded weights and a smaller `saved`."""
    import torch
    from paper_2412_04747_amd import binding as B
    from paper_2412_04747_amd.harness import Graph, HgtLayer
    rng, src, dst, rel, ntype = _graph(503, 3000, 12, 40000, T=3)
    if tied:
        ntype = (np.arange(3000) % 3).astype(np.int32)
        src = (src // 3 * 3 + rel % 3).astype(np.int32)          # source type = relation mod 3
    print(f"bounds case hgt {dtype} d={d} H={H} tied={tied}", flush=True)
    g = Graph(3000, 12, src, dst, rel, ntype, 3)
    L = HgtLayer(g, d, H, with_mu=True, dtype=dtype, flags=flags)
    p = synth.hgt_params(rng, 3000, 3, 12, d, H, with_mu=True)
    if dtype == "bf16":
        p = {k: (None if v is None else synth.round_to_bf16(v)) for k, v in p.items()}
    L.load(p["X"], p["Wk"], p["Wq"], p["Wv"], p["Wo"], p["Watt"], p["Wmsg"], p["mu"], p["dOut"])
    f, b, s = B.rgnn_workspace_bytes(g.handle, B.RGNN_LAYER_HGT, L.desc)
    row = d * (2 if dtype == "bf16" and d == 128 else 4)                 # bytes of one stored row
    rest = 2 * g.P * row + len(src) * H * 4                              # Ka, M and att
    assert (s < rest + 3 * 3000 * row) == tied                           # Q, Z and, unless folded, K and V
    wf, L.ws = _guarded(f)
    sv, L.saved = _guarded(s)
    L.fwd()
    torch.cuda.synchronize()
    _intact(wf, "forward workspace"); _intact(sv, "saved")
    wb, L.ws = _guarded(b)
    L.bwd()
    torch.cuda.synchronize()
    _intact(wb, "backward workspace"); _intact(sv, "saved")
    g.close()
