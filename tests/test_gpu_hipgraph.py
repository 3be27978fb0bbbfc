"""The layer calls only enqueue kernels on the caller's stream (no allocation, no synchronisation, no
memset), so a caller can record them into a HIP graph.  Each replay must reproduce the eager result
bit for bit, with other work and synchronisations between the replays."""
import numpy as np
import pytest

from paper_2412_04747_amd import synth

pytestmark = pytest.mark.gpu


def _capture_and_replay(L, outputs):
    import torch
    L.fwd(); L.bwd()                       # eager reference (also sets kernel attributes before the capture)
    torch.cuda.synchronize()
    ref = [t.clone() for t in outputs()]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        L.fwd(); L.bwd()                   # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            L.fwd(); L.bwd()
    torch.cuda.synchronize()
    for rep in range(3):
        for t in outputs():
            t.fill_(float("nan"))          # eager work between the replays; a replay must rewrite everything
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(ref, outputs()):
            assert torch.equal(a, b), f"replay {rep}"


def test_rgat_fwd_bwd_replays():
    from paper_2412_04747_amd.harness import Graph, RgatLayer
    rng, src, dst, rel, _ = synth.tiny(401, N=3000, R=6, E=30000)
    dst[:2000] = 5                                          # cut hub: partial rows and the combine kernels
    print("hipgraph case rgat: N=3000 R=6 E=30000 d=64", flush=True)
    p = synth.rgat_params(rng, 3000, 6, 64, 64)
    g = Graph(3000, 6, src, dst, rel)
    L = RgatLayer(g, 64)
    L.load(p["X"], p["W"], p["w_s"], p["w_t"], p["dOut"])
    _capture_and_replay(L, lambda: [L.out, L.dX, L.dW, L.dw_s, L.dw_t])
    g.close()


@pytest.mark.parametrize("T", [3, 1])
def test_hgt_bf16_fwd_bwd_replays(T):
    """T = 3: random node types, relations mix source types; T = 1: the path with folded weights."""
    from paper_2412_04747_amd.harness import Graph, HgtLayer
    rng, src, dst, rel, ntype = synth.tiny(402, N=2500, R=5, E=20000, T=T)
    dst[:1500] = 9
    print(f"hipgraph case hgt bf16: N=2500 T={T} R=5 E=20000 d=128 H=4", flush=True)
    p = {k: (None if v is None else synth.round_to_bf16(v)) for k, v in synth.hgt_params(rng, 2500, T, 5, 128, 4, with_mu=True).items()}
    g = Graph(2500, 5, src, dst, rel, ntype if T > 1 else None, T)
    L = HgtLayer(g, 128, 4, with_mu=True, dtype="bf16")
    L.load(p["X"], p["Wk"], p["Wq"], p["Wv"], p["Wo"], p["Watt"], p["Wmsg"], p["mu"], p["dOut"])
    _capture_and_replay(L, lambda: [L.out] + list(L.grads().values()))
    g.close()


def test_rgcn_bf16_fwd_bwd_replays():
    """bf16 rows: per-run scaled rows and the row selector of the backward typed linear."""
    from paper_2412_04747_amd.harness import Graph, RgcnLayer
    rng, src, dst, rel, _ = synth.tiny(403, N=3000, R=7, E=25000)
    dst[:1800] = 4
    print("hipgraph case rgcn bf16: N=3000 R=7 E=25000 d=128", flush=True)
    p = {k: (None if v is None else synth.round_to_bf16(v)) for k, v in synth.rgcn_params(rng, 3000, 7, 128, 128, self_loop=True).items()}
    g = Graph(3000, 7, src, dst, rel)
    L = RgcnLayer(g, 128, "in_degree_per_rel", "relu", True, dtype="bf16")
    L.load(p["X"], p["W"], p["W0"], p["dOut"])
    _capture_and_replay(L, lambda: [L.out] + list(L.grads().values()))
    g.close()
