"""rgnn_rgat_fwd_static (the forward entry point that takes no workspace and allocates nothing)
against rgnn_rgat_fwd on the same inputs, through the C ABI: two calls in a row, the second on a
smaller graph, so that the shared static buffer is seen to be reused with stale contents in it."""
import numpy as np
import pytest

from paper_2412_04747_amd import synth

pytestmark = pytest.mark.gpu


def _case(N, R, E, d, seed, hub, inference):
    import torch
    from paper_2412_04747_amd import binding as B
    from paper_2412_04747_amd.harness import Graph, RgatLayer, _buf, _stream
    print(f"static-scratch case: N={N} R={R} E={E} d={d} inference={inference}", flush=True)
    rng, src, dst, rel, _ = synth.tiny(seed, N=N, R=R, E=E)
    dst[:hub] = 3                                  # one destination long enough to be cut into pieces
    p = synth.rgat_params(rng, N, R, d, d)
    g = Graph(N, R, src, dst, rel)
    L = RgatLayer(g, d)
    L.load(p["X"], p["W"], p["w_s"], p["w_t"], p["dOut"])
    L.fwd()
    torch.cuda.synchronize()
    want_out, want_saved = L.out.clone(), L.saved.clone()
    f, _, s = B.rgnn_workspace_bytes(g.handle, B.RGNN_LAYER_RGAT, L.desc)
    assert f <= B.RGNN_STATIC_SCRATCH_BYTES
    out = torch.full_like(L.out, float("nan"))
    saved = None if inference else _buf(s)
    if saved is not None:
        saved.fill_(0xFF)
    before = torch.cuda.memory_allocated()
    B.rgnn_rgat_fwd_static(g.handle, L.desc, L.X, L.W, L.w_s, L.w_t, out, saved, _stream())
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert torch.equal(out, want_out)                       # same kernels, same order: bit-identical
    if saved is not None:
        want_parts = [t.clone() for t in L.saved_views()]
        L.saved = saved
        for got, want in zip(L.saved_views(), want_parts):     # Hs, s_dst, (m, s): every part the backward reads
            assert torch.equal(got, want)
        L.saved = want_saved
        # the backward call accepts what the static call saved
        L.bwd(); torch.cuda.synchronize()
        ref = {k: v.clone() for k, v in L.grads().items()}
        L.saved = saved
        L.bwd(); torch.cuda.synchronize()
        for k, v in L.grads().items():
            assert torch.equal(v, ref[k]), k
    g.close()


def test_static_scratch_matches_workspace_call_twice():
    _case(3000, 7, 40000, 64, 901, 1500, inference=False)
    _case(400, 3, 2500, 64, 902, 300, inference=False)      # smaller input, same buffer
    _case(900, 4, 6000, 32, 903, 700, inference=True)       # saved == NULL: everything in the static buffer


def test_static_scratch_rejects_oversized_call():
    from paper_2412_04747_amd import binding as B
    from paper_2412_04747_amd.harness import Graph, RgatLayer, _stream
    import torch
    N, R, E, d = 200000, 4, 3000000, 128
    rng = np.random.default_rng(5)
    src = rng.integers(0, N, E).astype(np.int32)
    dst = rng.integers(0, N, E).astype(np.int32)
    rel = rng.integers(0, R, E).astype(np.int32)
    g = Graph(N, R, src, dst, rel)
    desc = B.make_desc(B.RGNN_F32, d, d, 1, 0.2)
    f, _, s = B.rgnn_workspace_bytes(g.handle, B.RGNN_LAYER_RGAT, desc)
    assert f + s > B.RGNN_STATIC_SCRATCH_BYTES
    X = torch.zeros(N, d, device="cuda"); W = torch.zeros(R, d, d, device="cuda")
    w = torch.zeros(R, d, device="cuda"); out = torch.zeros(N, d, device="cuda")
    with pytest.raises(B.RgnnError) as e:
        B.rgnn_rgat_fwd_static(g.handle, desc, X, W, w, w, out, None, _stream())     # inference: saved in scratch too
    assert e.value.status == 5 and "static buffer" in str(e.value)
    g.close()
