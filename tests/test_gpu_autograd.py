"""The autograd front end: two-layer models trained with a negative-log-likelihood loss (the
training protocol of the thesis' evaluation), checked against the same chain written out with
the CPU oracle's layer functions in fp64."""
import numpy as np
import pytest

from oracle import layers as O
from paper_2412_04747_amd import synth
from parity import check, TOL_F32

pytestmark = pytest.mark.gpu


def _nll_head(h, train, labels):
    """loss = mean over train nodes of -log softmax(h)[label]; returns (loss, dL/dh), fp64."""
    z = h[train]
    z = z - z.max(axis=1, keepdims=True)
    logp = z - np.log(np.exp(z).sum(axis=1, keepdims=True))
    loss = -logp[np.arange(len(train)), labels].mean()
    g = np.exp(logp)
    g[np.arange(len(train)), labels] -= 1.0
    dh = np.zeros_like(h)
    dh[train] = g / len(train)
    return loss, dh


@pytest.mark.parametrize("d0,d,d2", [(64, 64, 64), (32, 64, 32)])       # input, hidden and output width
def test_two_layer_rgat_nll(d0, d, d2):
    import torch
    from paper_2412_04747_amd import autograd as A
    N, R, E = 900, 6, 8000
    rng, src, dst, rel, _ = synth.tiny(301, N=N, R=R, E=E)
    dst[:700] = 11                                  # a hub cut into pieces
    p1, p2 = synth.rgat_params(rng, N, R, d0, d), synth.rgat_params(rng, N, R, d, d2)
    train = rng.choice(N, 300, replace=False)
    labels = rng.integers(0, d2, 300)
    print(f"autograd case rgat2: N={N} R={R} E={E} widths {d0} -> {d} -> {d2}", flush=True)

    g = A.Graph(N, R, src, dst, rel)
    t = lambda a: torch.tensor(a, dtype=torch.float32, device="cuda", requires_grad=True)
    X = t(p1["X"])
    P1 = [t(p1[k]) for k in ("W", "w_s", "w_t")]
    P2 = [t(p2[k]) for k in ("W", "w_s", "w_t")]
    h1 = torch.relu(A.rgat(g, X, *P1))
    h2 = A.rgat(g, h1, *P2)
    logp = torch.log_softmax(h2[torch.as_tensor(train, device="cuda")], dim=1)
    loss = torch.nn.functional.nll_loss(logp, torch.as_tensor(labels, device="cuda"))
    loss.backward()
    torch.cuda.synchronize()

    # the same chain with the oracle, from the same fp32-rounded inputs
    f = lambda a: np.asarray(a, dtype=np.float32).astype(np.float64)
    q1 = {k: f(p1[k]) for k in ("X", "W", "w_s", "w_t")}
    q2 = {k: f(p2[k]) for k in ("W", "w_s", "w_t")}
    a1 = O.rgat_fwd(N, src, dst, rel, q1["X"], q1["W"], q1["w_s"], q1["w_t"])
    r1 = np.maximum(a1, 0.0)
    a2 = O.rgat_fwd(N, src, dst, rel, r1, q2["W"], q2["w_s"], q2["w_t"])
    want_loss, dh2 = _nll_head(a2, train, labels)
    g2 = O.rgat_bwd(N, src, dst, rel, r1, q2["W"], q2["w_s"], q2["w_t"], dh2)
    g1 = O.rgat_bwd(N, src, dst, rel, q1["X"], q1["W"], q1["w_s"], q1["w_t"], g2["dX"] * (a1 > 0))

    assert abs(loss.item() - want_loss) <= 1e-4 * abs(want_loss)
    check(X.grad, g1["dX"], TOL_F32, "dX")
    for tns, k in zip(P1, ("dW", "dw_s", "dw_t")):
        check(tns.grad, g1[k], TOL_F32, "layer1 " + k)
    for tns, k in zip(P2, ("dW", "dw_s", "dw_t")):
        check(tns.grad, g2[k], TOL_F32, "layer2 " + k)
    A.release(g)
    g.close()


def test_rgcn_then_hgt_modules_train():
    """nn.Module front end: RGCN (ReLU, self-loop) feeding an HGT layer; gradients reach every
    parameter and a few optimiser steps lower the loss."""
    import torch
    from paper_2412_04747_amd import autograd as A
    N, T, R, E, d, H = 800, 3, 5, 7000, 64, 2
    rng, src, dst, rel, ntype = synth.tiny(302, N=N, R=R, E=E, T=T)
    print(f"autograd case rgcn+hgt: N={N} T={T} R={R} E={E} d={d} H={H}", flush=True)
    g = A.Graph(N, R, src, dst, rel, ntype=ntype, T=T)
    torch.manual_seed(0)
    l1, l2 = A.RgcnConv(R, d, self_loop=True, act="relu"), A.HgtConv(T, R, d, H)
    X = torch.tensor(synth.rgcn_params(rng, N, R, d, d)["X"], dtype=torch.float32, device="cuda")
    train = torch.as_tensor(rng.choice(N, 400, replace=False), device="cuda")
    labels = torch.as_tensor(rng.integers(0, 8, 400), device="cuda")
    params = list(l1.parameters()) + list(l2.parameters())
    opt = torch.optim.Adam(params, lr=1e-2)
    losses = []
    for step in range(12):
        opt.zero_grad()
        out = l2(g, l1(g, X))
        loss = torch.nn.functional.nll_loss(torch.log_softmax(out[train, :8], dim=1), labels)
        loss.backward()
        if step == 0:
            for q in params:
                assert q.grad is not None and torch.isfinite(q.grad).all() and q.grad.abs().sum() > 0
        opt.step()
        losses.append(loss.item())
    print("losses", [round(v, 4) for v in losses], flush=True)
    assert losses[-1] < 0.95 * losses[0]

    # one more forward/backward of the trained model against the oracle chain
    f = lambda q: q.detach().cpu().numpy().astype(np.float64)
    out = l2(g, l1(g, X))
    dOut = torch.tensor(synth.rgcn_params(rng, N, R, d, d)["dOut"], dtype=torch.float32, device="cuda")
    for q in params:
        q.grad = None
    out.backward(dOut)
    torch.cuda.synchronize()
    a1 = O.rgcn_fwd(N, src, dst, rel, f(X), f(l1.W), f(l1.W0), "in_degree_per_rel", "relu")
    hp = [f(q) for q in (l2.Wk, l2.Wq, l2.Wv, l2.Wo, l2.Watt, l2.Wmsg, l2.mu)]
    a2 = O.hgt_fwd(N, src, dst, rel, ntype, a1, *hp)
    check(out, a2, TOL_F32, "out")
    g2 = O.hgt_bwd(N, src, dst, rel, ntype, a1, *hp, f(dOut))
    g1 = O.rgcn_bwd(N, src, dst, rel, f(X), f(l1.W), f(l1.W0), g2["dX"], "in_degree_per_rel", "relu", out=a1)
    for q, k in zip((l2.Wk, l2.Wq, l2.Wv, l2.Wo, l2.Watt, l2.Wmsg, l2.mu), ("dWk", "dWq", "dWv", "dWo", "dWatt", "dWmsg", "dmu")):
        check(q.grad, g2[k], TOL_F32, "hgt " + k)
    check(l1.W.grad, g1["dW"], TOL_F32, "rgcn dW")
    check(l1.W0.grad, g1["dW0"], TOL_F32, "rgcn dW0")
    A.release(g)
    g.close()


def test_multi_head_function_matches_the_oracle():
    import torch
    from paper_2412_04747_amd import autograd as A
    N, R, E, d, H = 700, 5, 6000, 64, 4
    rng, src, dst, rel, _ = synth.tiny(303, N=N, R=R, E=E)
    p = synth.rgat_params(rng, N, R, d, d)
    print(f"autograd case rgat heads: N={N} R={R} E={E} d={d} H={H}", flush=True)
    g = A.Graph(N, R, src, dst, rel)
    t = lambda a: torch.tensor(a, dtype=torch.float32, device="cuda", requires_grad=True)
    X, W, ws, wt = t(p["X"]), t(p["W"]), t(p["w_s"]), t(p["w_t"])
    out = A.rgat(g, X, W, ws, wt, heads=H)
    out.backward(torch.tensor(p["dOut"], dtype=torch.float32, device="cuda"))
    torch.cuda.synchronize()
    f = lambda a: np.asarray(a, dtype=np.float32).astype(np.float64)
    want = O.rgat_heads_fwd(N, src, dst, rel, f(p["X"]), f(p["W"]), f(p["w_s"]), f(p["w_t"]), H)
    wg = O.rgat_heads_bwd(N, src, dst, rel, f(p["X"]), f(p["W"]), f(p["w_s"]), f(p["w_t"]), f(p["dOut"]), H)
    check(out, want, TOL_F32, "out")
    for tns, k in ((X, "dX"), (W, "dW"), (ws, "dw_s"), (wt, "dw_t")):
        check(tns.grad, wg[k], TOL_F32, k)
    A.release(g)
    g.close()


def test_workspaces_live_and_die_with_their_graph():
    """The front end keeps its scratch buffers on the Graph object: a graph that is dropped takes them along,
    and a later, larger graph (even one that lands on the same Python id) gets buffers of its own size."""
    import gc
    import torch
    from paper_2412_04747_amd import autograd as A, binding as B
    d = 64

    def run(N, R, E, seed):
        rng, src, dst, rel, _ = synth.tiny(seed, N=N, R=R, E=E)
        p = synth.rgat_params(rng, N, R, d, d)
        g = A.Graph(N, R, src, dst, rel)
        t = lambda a: torch.tensor(a, dtype=torch.float32, device="cuda", requires_grad=True)
        out = A.rgat(g, t(p["X"]), t(p["W"]), t(p["w_s"]), t(p["w_t"]))
        out.sum().backward()
        torch.cuda.synchronize()
        f, b, _ = B.rgnn_workspace_bytes(g.handle, B.RGNN_LAYER_RGAT, B.make_desc(B.RGNN_F32, d, d, 1, 0.2))
        (ws, _), = g.workspaces.values()
        assert ws.numel() >= max(f, b)
        return g, max(f, b)

    print("autograd case workspace lifetime", flush=True)
    small, need_small = run(200, 3, 1500, 311)
    small_id = id(small)
    small.close()
    assert small.workspaces == {}
    with pytest.raises(RuntimeError):
        A._bufs(small, B.RGNN_LAYER_RGAT, B.make_desc(), (64, 1))       # a closed graph hands out nothing
    del small
    gc.collect()
    for seed in range(312, 320):                                         # several tries at recycling the id
        big, need_big = run(3000, 6, 40000, seed)
        assert need_big > need_small
        reused = id(big) == small_id
        big.close()
        del big
        gc.collect()
        if reused:
            break
