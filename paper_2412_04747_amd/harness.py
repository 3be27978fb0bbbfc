"""Convenience wrappers used by the tests, the smoke check and the benchmark.

They only allocate device buffers with PyTorch, copy inputs in / results out and
call the C ABI through `binding`; no layer arithmetic happens here.
"""
import numpy as np
import torch

from . import binding as B


def _dev(a, dtype=torch.float32):
    if a is None:
        return None
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda", dtype=dtype)


def _tdtype(name):
    """Storage type of the tensor arguments: "f32", or "bf16" (values must already be
    bf16-representable, e.g. from synth.round_to_bf16, so the conversion is exact)."""
    return (B.RGNN_BF16, torch.bfloat16) if name == "bf16" else (B.RGNN_F32, torch.float32)


def _buf(nbytes):
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device="cuda")


def _stream():
    return torch.cuda.current_stream().cuda_stream


class Graph:
    def __init__(self, N, R, src, dst, rel, ntype=None, T=1, rel_src_ntype=None, rel_dst_ntype=None):
        i32 = lambda a: None if a is None else np.ascontiguousarray(a, dtype=np.int32)
        torch.cuda.init()
        self.workspaces = {}
        self.handle = None
        self.N, self.R, self.T, self.E = int(N), int(R), int(T), len(src)
        self.handle = B.rgnn_graph_create(N, T, R, self.E, B.RGNN_COO, i32(src), i32(dst), i32(rel), i32(ntype),
                                          i32(rel_src_ntype), i32(rel_dst_ntype), B.RGNN_MEM_HOST)
        self.info = B.rgnn_graph_info(self.handle)
        self.P, self.Q = int(self.info.num_pairs), int(self.info.num_runs)
        self.workspaces = {}       # scratch buffers the autograd front end keeps per layer configuration

    def export(self, name):
        which = B.INDEX_NAMES.index(name)
        N, E, P, Q, R, T = self.N, self.E, self.P, self.Q, self.R, self.T
        length = {"in_ptr": N + 1, "pair_ptr": R + 1, "pair_src": P, "pair_rel": P, "run_ptr": Q + 1, "run_dst": Q,
                  "run_rel": Q, "dst_run_ptr": N + 1, "relrun_ptr": R + 1, "relrun_idx": Q, "out_ptr": P + 1,
                  "srcpair_ptr": N + 1, "srcpair_idx": P, "ntype_ptr": T + 1, "ntype_perm": N, "relrun_dst": Q,
                  "pair_sel_dst": P, "rel_src_type": R}.get(name, E)
        return B.rgnn_graph_export(self.handle, which, length)

    def close(self):
        self.workspaces.clear()
        if self.handle is not None:
            B.rgnn_graph_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class RgatLayer:
    """Device buffers for one RGAT layer call pair on a graph."""

    def __init__(self, graph, d, slope=0.2, dtype="f32", heads=1, flags=0, d_in=None):
        """d: output width; d_in: input width when it differs."""
        self.g, self.d, self.H = graph, d, heads
        k = d_in or d
        code, self.tdt = _tdtype(dtype)
        self.desc = B.make_desc(code, k, d, heads, slope, flags=flags)
        f, b, s = B.rgnn_workspace_bytes(graph.handle, B.RGNN_LAYER_RGAT, self.desc)
        self.ws = _buf(max(f, b))
        self.saved = _buf(s)
        N, R = graph.N, graph.R
        self.out = torch.empty(N, d, device="cuda")
        self.dX = torch.empty(N, k, device="cuda")
        self.dW = torch.empty(R, k, d, device="cuda")
        self.dw_s = torch.empty(R, d, device="cuda")
        self.dw_t = torch.empty(R, d, device="cuda")

    def load(self, X, W, w_s, w_t, dOut=None):
        t = self.tdt
        self.X, self.W, self.w_s, self.w_t, self.dOut = _dev(X, t), _dev(W, t), _dev(w_s, t), _dev(w_t, t), _dev(dOut, t)

    def fwd(self):
        B.rgnn_rgat_fwd(self.g.handle, self.desc, self.X, self.W, self.w_s, self.w_t, self.out, self.saved, self.ws,
                        _stream())

    def bwd(self):
        B.rgnn_rgat_bwd(self.g.handle, self.desc, self.X, self.W, self.w_s, self.w_t, self.out, self.saved, self.dOut,
                        self.dX, self.dW, self.dw_s, self.dw_t, self.ws, _stream())

    def saved_views(self):
        """The parts of `saved`: Hs [P, d], s_dst [Q, heads], ms [N, heads, 2]."""
        P, Q, N, d, H = self.g.P, self.g.Q, self.g.N, self.d, self.H
        al = lambda n: (max(n, 1) * 4 + 255) // 256 * 256 // 4
        f32 = self.saved.view(torch.float32)
        hs = f32[: P * d].view(P, d)
        off = al(P * d)
        s_dst = f32[off: off + Q * H].view(Q, H)
        off += al(Q * H)
        return hs, s_dst, f32[off: off + 2 * N * H].view(N, H, 2)

    def grads(self):
        return dict(dX=self.dX, dW=self.dW, dw_s=self.dw_s, dw_t=self.dw_t)


class RgcnLayer:
    def __init__(self, graph, d, norm="in_degree_per_rel", act="none", self_loop=False, dtype="f32", flags=0, d_in=None):
        """d: output width; d_in: input width when it differs."""
        self.g, self.d, self.self_loop = graph, d, self_loop
        k = d_in or d
        code, self.tdt = _tdtype(dtype)
        self.desc = B.make_desc(code, k, d, 1, 0.0,
                                B.RGNN_NORM_IN_DEGREE_PER_REL if norm == "in_degree_per_rel" else B.RGNN_NORM_NONE,
                                B.RGNN_ACT_RELU if act == "relu" else B.RGNN_ACT_NONE, flags)
        f, b, s = B.rgnn_workspace_bytes(graph.handle, B.RGNN_LAYER_RGCN, self.desc)
        self.ws = _buf(max(f, b))
        self.saved = _buf(s)
        N, R = graph.N, graph.R
        self.out = torch.empty(N, d, device="cuda")
        self.dX = torch.empty(N, k, device="cuda")
        self.dW = torch.empty(R, k, d, device="cuda")
        self.dW0 = torch.empty(k, d, device="cuda") if self_loop else None

    def load(self, X, W, W0=None, dOut=None):
        t = self.tdt
        self.X, self.W, self.W0, self.dOut = _dev(X, t), _dev(W, t), _dev(W0, t), _dev(dOut, t)

    def fwd(self):
        B.rgnn_rgcn_fwd(self.g.handle, self.desc, self.X, self.W, self.W0, self.out, self.saved, self.ws, _stream())

    def bwd(self):
        B.rgnn_rgcn_bwd(self.g.handle, self.desc, self.X, self.W, self.W0, self.out, self.saved, self.dOut, self.dX,
                        self.dW, self.dW0, self.ws, _stream())

    def grads(self):
        g = dict(dX=self.dX, dW=self.dW)
        if self.self_loop:
            g["dW0"] = self.dW0
        return g


class HgtLayer:
    def __init__(self, graph, d, heads, with_mu=True, dtype="f32", flags=0):
        self.g, self.d, self.H = graph, d, heads
        code, self.tdt = _tdtype(dtype)
        self.desc = B.make_desc(code, d, d, heads, flags=flags)
        f, b, s = B.rgnn_workspace_bytes(graph.handle, B.RGNN_LAYER_HGT, self.desc)
        self.ws = _buf(max(f, b))
        self.saved = _buf(s)
        N, R, T, dh = graph.N, graph.R, graph.T, d // heads
        e = lambda *shape: torch.empty(*shape, device="cuda")
        self.out, self.dX = e(N, d), e(N, d)
        self.dWk, self.dWq, self.dWv, self.dWo = e(T, d, d), e(T, d, d), e(T, d, d), e(T, d, d)
        self.dWatt, self.dWmsg = e(R, heads, dh, dh), e(R, heads, dh, dh)
        self.dmu = e(R, heads) if with_mu else None

    def load(self, X, Wk, Wq, Wv, Wo, Watt, Wmsg, mu=None, dOut=None):
        (self.X, self.Wk, self.Wq, self.Wv, self.Wo, self.Watt, self.Wmsg, self.mu, self.dOut) = (
            _dev(a, self.tdt) for a in (X, Wk, Wq, Wv, Wo, Watt, Wmsg, mu, dOut))

    def fwd(self):
        B.rgnn_hgt_fwd(self.g.handle, self.desc, self.X, self.Wk, self.Wq, self.Wv, self.Wo, self.Watt, self.Wmsg,
                       self.mu, self.out, self.saved, self.ws, _stream())

    def bwd(self):
        B.rgnn_hgt_bwd(self.g.handle, self.desc, self.X, self.Wk, self.Wq, self.Wv, self.Wo, self.Watt, self.Wmsg,
                       self.mu, self.out, self.saved, self.dOut, self.dX, self.dWk, self.dWq, self.dWv, self.dWo,
                       self.dWatt, self.dWmsg, self.dmu, self.ws, _stream())

    def grads(self):
        g = dict(dX=self.dX, dWk=self.dWk, dWq=self.dWq, dWv=self.dWv, dWo=self.dWo, dWatt=self.dWatt,
                 dWmsg=self.dWmsg)
        if self.dmu is not None:
            g["dmu"] = self.dmu
        return g
