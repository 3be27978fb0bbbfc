"""PyTorch autograd front end of the layer library.

`rgat`, `rgcn` and `hgt` are differentiable functions of torch tensors that live on the GPU;
`RgatConv`, `RgcnConv` and `HgtConv` are `torch.nn.Module`s holding the parameters.  Forward and
backward are the C-ABI calls of `binding`; PyTorch only owns the memory, the stream and the
tape.  Everything is fp32 (the training protocol of the thesis' evaluation section: full-graph
training of a two-layer model with a negative-log-likelihood loss).

The workspace of a (layer kind, width, options) combination is allocated once per graph, kept on the
`Graph` object and dropped by `Graph.close()`; every call of that combination on the graph reuses it,
so such calls must not overlap on different streams.
"""
import math

import torch

from . import binding as B
from .harness import Graph, _buf, _stream


def _bufs(graph, layer, desc, key):
    """(workspace, saved size) for a layer configuration on a graph.  The workspace lives in
    `graph.workspaces` (sized by rgnn_workspace_bytes for this very graph), so it can neither outlive
    the graph nor be handed to another one."""
    if graph.handle is None:
        raise RuntimeError("the graph has been closed")
    k = (layer,) + key
    if k not in graph.workspaces:
        f, b, s = B.rgnn_workspace_bytes(graph.handle, layer, desc)
        graph.workspaces[k] = (_buf(max(f, b)), s)
    return graph.workspaces[k]


def release(graph):
    """Drop the cached workspaces of a graph (Graph.close() does the same)."""
    graph.workspaces.clear()


def _f32(t):
    if t is None:
        return None
    if t.dtype != torch.float32 or not t.is_cuda:
        raise TypeError("rgnn autograd functions take fp32 CUDA tensors")
    return t.contiguous()


class _Rgat(torch.autograd.Function):
    @staticmethod
    def forward(ctx, graph, slope, heads, X, W, w_s, w_t):
        X, W, w_s, w_t = _f32(X), _f32(W), _f32(w_s), _f32(w_t)
        d_in, d = W.shape[-2], W.shape[-1]
        desc = B.make_desc(B.RGNN_F32, d_in, d, heads, slope)
        ws, s = _bufs(graph, B.RGNN_LAYER_RGAT, desc, (d_in, d, heads))
        out = torch.empty(graph.N, d, device=X.device)
        saved = _buf(s)
        B.rgnn_rgat_fwd(graph.handle, desc, X, W, w_s, w_t, out, saved, ws, _stream())
        ctx.graph, ctx.desc, ctx.ws, ctx.saved_buf = graph, desc, ws, saved
        ctx.save_for_backward(X, W, w_s, w_t, out)
        return out

    @staticmethod
    def backward(ctx, dOut):
        X, W, w_s, w_t, out = ctx.saved_tensors
        dOut = _f32(dOut)
        dX, dW, dws, dwt = (torch.empty_like(t) for t in (X, W, w_s, w_t))
        B.rgnn_rgat_bwd(ctx.graph.handle, ctx.desc, X, W, w_s, w_t, out, ctx.saved_buf, dOut, dX, dW, dws, dwt, ctx.ws,
                        _stream())
        return None, None, None, dX, dW, dws, dwt


class _Rgcn(torch.autograd.Function):
    @staticmethod
    def forward(ctx, graph, norm, act, X, W, W0):
        X, W, W0 = _f32(X), _f32(W), _f32(W0)
        d_in, d = W.shape[-2], W.shape[-1]
        desc = B.make_desc(B.RGNN_F32, d_in, d, 1, 0.0,
                           B.RGNN_NORM_IN_DEGREE_PER_REL if norm == "in_degree_per_rel" else B.RGNN_NORM_NONE,
                           B.RGNN_ACT_RELU if act == "relu" else B.RGNN_ACT_NONE)
        ws, _ = _bufs(graph, B.RGNN_LAYER_RGCN, desc, (d_in, d, norm, act))
        out = torch.empty(graph.N, d, device=X.device)
        B.rgnn_rgcn_fwd(graph.handle, desc, X, W, W0, out, None, ws, _stream())
        ctx.graph, ctx.desc, ctx.ws, ctx.has_w0 = graph, desc, ws, W0 is not None
        ctx.save_for_backward(X, W, out, *([W0] if W0 is not None else []))
        return out

    @staticmethod
    def backward(ctx, dOut):
        X, W, out, *rest = ctx.saved_tensors
        W0 = rest[0] if ctx.has_w0 else None
        dOut = _f32(dOut)
        dX, dW = torch.empty_like(X), torch.empty_like(W)
        dW0 = torch.empty_like(W0) if W0 is not None else None
        B.rgnn_rgcn_bwd(ctx.graph.handle, ctx.desc, X, W, W0, out, None, dOut, dX, dW, dW0, ctx.ws, _stream())
        return None, None, None, dX, dW, dW0


class _Hgt(torch.autograd.Function):
    @staticmethod
    def forward(ctx, graph, X, Wk, Wq, Wv, Wo, Watt, Wmsg, mu):
        X, Wk, Wq, Wv, Wo, Watt, Wmsg, mu = (_f32(t) for t in (X, Wk, Wq, Wv, Wo, Watt, Wmsg, mu))
        d, H = Wk.shape[-1], Watt.shape[1]
        desc = B.make_desc(B.RGNN_F32, d, d, H)
        ws, s = _bufs(graph, B.RGNN_LAYER_HGT, desc, (d, H))
        out = torch.empty(graph.N, d, device=X.device)
        saved = _buf(s)
        B.rgnn_hgt_fwd(graph.handle, desc, X, Wk, Wq, Wv, Wo, Watt, Wmsg, mu, out, saved, ws, _stream())
        ctx.graph, ctx.desc, ctx.ws, ctx.saved_buf, ctx.has_mu = graph, desc, ws, saved, mu is not None
        ctx.save_for_backward(X, Wk, Wq, Wv, Wo, Watt, Wmsg, out, *([mu] if mu is not None else []))
        return out

    @staticmethod
    def backward(ctx, dOut):
        X, Wk, Wq, Wv, Wo, Watt, Wmsg, out, *rest = ctx.saved_tensors
        mu = rest[0] if ctx.has_mu else None
        dOut = _f32(dOut)
        g = [torch.empty_like(t) for t in (X, Wk, Wq, Wv, Wo, Watt, Wmsg)]
        dmu = torch.empty_like(mu) if mu is not None else None
        B.rgnn_hgt_bwd(ctx.graph.handle, ctx.desc, X, Wk, Wq, Wv, Wo, Watt, Wmsg, mu, out, ctx.saved_buf, dOut, *g, dmu,
                       ctx.ws, _stream())
        return (None, *g, dmu)


def rgat(graph, X, W, w_s, w_t, slope=0.2, heads=1):
    """RGAT layer (listing of the single-headed RGAT layer in the thesis; with heads > 1 each head
    works on its slice of the d columns): out [N, d]."""
    return _Rgat.apply(graph, float(slope), int(heads), X, W, w_s, w_t)


def rgcn(graph, X, W, W0=None, norm="in_degree_per_rel", act="none"):
    """RGCN layer, Eq. (rgcn): out [N, d]."""
    return _Rgcn.apply(graph, norm, act, X, W, W0)


def hgt(graph, X, Wk, Wq, Wv, Wo, Watt, Wmsg, mu=None):
    """HGT layer (figure "HGT and RGAT layer"): out [N, d]; heads = Watt.shape[1]."""
    return _Hgt.apply(graph, X, Wk, Wq, Wv, Wo, Watt, Wmsg, mu)


def _param(*shape, fan_in):
    return torch.nn.Parameter(torch.randn(*shape, device="cuda") / math.sqrt(fan_in))


class RgatConv(torch.nn.Module):
    def __init__(self, num_rels, d, slope=0.2, heads=1, d_in=None):
        """d: output width; d_in: input width when it differs (32 and 64 may be mixed)."""
        super().__init__()
        self.slope, self.heads = slope, heads
        k = d_in or d
        self.W, self.w_s, self.w_t = _param(num_rels, k, d, fan_in=k), _param(num_rels, d, fan_in=d), _param(num_rels, d, fan_in=d)

    def forward(self, graph, X):
        return rgat(graph, X, self.W, self.w_s, self.w_t, self.slope, self.heads)


class RgcnConv(torch.nn.Module):
    def __init__(self, num_rels, d, self_loop=True, norm="in_degree_per_rel", act="none", d_in=None):
        """d: output width; d_in: input width when it differs (32 and 64 may be mixed)."""
        super().__init__()
        self.norm, self.act = norm, act
        k = d_in or d
        self.W = _param(num_rels, k, d, fan_in=k)
        self.W0 = _param(k, d, fan_in=k) if self_loop else None

    def forward(self, graph, X):
        return rgcn(graph, X, self.W, self.W0, self.norm, self.act)


class HgtConv(torch.nn.Module):
    def __init__(self, num_ntypes, num_rels, d, heads, with_mu=True):
        super().__init__()
        dh = d // heads
        self.Wk, self.Wq, self.Wv, self.Wo = (_param(num_ntypes, d, d, fan_in=d) for _ in range(4))
        self.Watt, self.Wmsg = _param(num_rels, heads, dh, dh, fan_in=dh), _param(num_rels, heads, dh, dh, fan_in=dh)
        self.mu = torch.nn.Parameter(torch.ones(num_rels, heads, device="cuda")) if with_mu else None

    def forward(self, graph, X):
        return hgt(graph, X, self.Wk, self.Wq, self.Wv, self.Wo, self.Watt, self.Wmsg, self.mu)


__all__ = ["Graph", "rgat", "rgcn", "hgt", "RgatConv", "RgcnConv", "HgtConv", "release"]
