"""RGNN_FLAG_ACCUMULATE: the backward calls add every gradient to what the caller's buffers hold."""
import numpy as np
import pytest

from paper_2412_04747_amd import synth

pytestmark = pytest.mark.gpu
ACC = 32        # RGNN_FLAG_ACCUMULATE


def _check_adds(make_layer, load, tag):
    """Backward without the flag gives g; with the flag on buffers holding G0 it must leave G0 + g."""
    import torch
    print(f"accumulate case {tag}", flush=True)
    plain = make_layer(0)
    load(plain)
    plain.fwd(); plain.bwd()
    torch.cuda.synchronize()
    g = {k: v.clone() for k, v in plain.grads().items()}
    acc = make_layer(ACC)
    load(acc)
    acc.fwd()
    gen = torch.Generator(device="cuda").manual_seed(1234)
    g0 = {}
    for k, v in acc.grads().items():
        v.copy_(torch.randn(v.shape, device="cuda", generator=gen) * (g[k].abs().max() + 1e-3))
        g0[k] = v.clone()
    acc.bwd()
    torch.cuda.synchronize()
    for k, v in acc.grads().items():
        want = g0[k].double() + g[k].double()
        err = (v.double() - want).abs().max().item() / max(want.abs().max().item(), 1e-30)
        assert err <= 2e-6, (tag, k, err)
    # and a second call adds once more
    acc.bwd()
    torch.cuda.synchronize()
    for k, v in acc.grads().items():
        want = g0[k].double() + 2 * g[k].double()
        err = (v.double() - want).abs().max().item() / max(want.abs().max().item(), 1e-30)
        assert err <= 4e-6, (tag, k, err)


def _hub(seed, N, R, E, T=1):
    rng, src, dst, rel, ntype = synth.tiny(seed, N=N, R=R, E=E, T=T)
    dst[:E // 6] = 3                                  # a destination cut into pieces
    src[E // 6:E // 4] = 5; rel[E // 6:E // 4] = 1    # a pair with many edges
    return rng, src, dst, rel, ntype


@pytest.mark.parametrize("d,H,dtype,flags", [(64, 1, "f32", 0), (32, 1, "f32", 4), (128, 1, "f32", 0), (64, 4, "f32", 0),
                                             (64, 4, "f32", 4), (128, 8, "f32", 0), (64, 1, "bf16", 0)])
def test_rgat(d, H, dtype, flags):
    from paper_2412_04747_amd.harness import Graph, RgatLayer
    N, R, E = 3000, 7, 20000
    rng, src, dst, rel, _ = _hub(900 + d + H, N, R, E)
    p = synth.rgat_params(rng, N, R, d, d)
    if dtype == "bf16":
        p = {k: synth.round_to_bf16(v) for k, v in p.items()}
    g = Graph(N, R, src, dst, rel)
    _check_adds(lambda f: RgatLayer(g, d, 0.2, dtype=dtype, heads=H, flags=flags | f),
                lambda L: L.load(p["X"], p["W"], p["w_s"], p["w_t"], p["dOut"]), f"rgat d={d} H={H} {dtype} flags={flags}")
    g.close()


@pytest.mark.parametrize("d,dtype,self_loop,act", [(64, "f32", True, "relu"), (32, "f32", False, "none"), (128, "bf16", True, "none"),
                                                   (128, "bf16", False, "relu")])
def test_rgcn(d, dtype, self_loop, act):
    from paper_2412_04747_amd.harness import Graph, RgcnLayer
    N, R, E = 3000, 6, 20000
    rng, src, dst, rel, _ = _hub(930 + d, N, R, E)
    p = synth.rgcn_params(rng, N, R, d, d, self_loop=self_loop)
    if dtype == "bf16":
        p = {k: synth.round_to_bf16(v) for k, v in p.items()}
    g = Graph(N, R, src, dst, rel)
    _check_adds(lambda f: RgcnLayer(g, d, act=act, self_loop=self_loop, dtype=dtype, flags=f),
                lambda L: L.load(p["X"], p["W"], p["W0"] if self_loop else None, p["dOut"]), f"rgcn d={d} {dtype} loop={self_loop} {act}")
    g.close()


@pytest.mark.parametrize("d,H,dtype,tied", [(64, 2, "f32", False), (64, 4, "f32", True), (128, 4, "bf16", False), (128, 4, "bf16", True)])
def test_hgt(d, H, dtype, tied):
    from paper_2412_04747_amd.harness import Graph, HgtLayer
    N, R, T, E = 2500, 6, 3, 16000
    rng, src, dst, rel, ntype = _hub(960 + d + H, N, R, E, T=T)
    if tied:
        rel[:] = ntype[src] * 2 + (rel % 2)           # every relation's sources have one node type: the folded path
    p = synth.hgt_params(rng, N, T, R, d, H, with_mu=True)
    if dtype == "bf16":
        p = {k: (None if v is None else synth.round_to_bf16(v)) for k, v in p.items()}
    g = Graph(N, R, src, dst, rel, ntype, T)
    _check_adds(lambda f: HgtLayer(g, d, H, with_mu=True, dtype=dtype, flags=f),
                lambda L: L.load(p["X"], p["Wk"], p["Wq"], p["Wv"], p["Wo"], p["Watt"], p["Wmsg"], p["mu"], p["dOut"]),
                f"hgt d={d} H={H} {dtype} tied={tied}")
    g.close()
