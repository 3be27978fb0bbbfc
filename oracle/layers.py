"""ctypes front end of the C oracle (oracle/rgnn_oracle.c).

All floating-point inputs are converted to float64 (exactly, from fp32 or from
bf16-rounded fp32) and all results are float64.  Edges are COO arrays in any
order.  Test infrastructure only.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.LIB if os.path.exists(_build.LIB) else _build.build()
        _lib = C.CDLL(path)
        _lib.oracle_num_threads.restype = C.c_int
    return _lib


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def _f(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float64)


def _i(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.int32)


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


_NORM = {"none": 0, "in_degree_per_rel": 1, None: 0, 0: 0, 1: 1}
_ACT = {"none": 0, "relu": 1, None: 0, 0: 0, 1: 1}


def rgcn_fwd(N, src, dst, rel, X, W, W0=None, norm="in_degree_per_rel", act="none"):
    src, dst, rel, X, W, W0 = _i(src), _i(dst), _i(rel), _f(X), _f(W), _f(W0)
    R, d_in, d_out = W.shape
    out = np.empty((N, d_out))
    lib().oracle_rgcn_fwd(C.c_int64(N), C.c_int64(len(src)), C.c_int32(R), C.c_int32(d_in), C.c_int32(d_out),
                          _p(src), _p(dst), _p(rel), _p(X), _p(W), _p(W0),
                          C.c_int32(_NORM[norm]), C.c_int32(_ACT[act]), _p(out))
    return out


def rgcn_bwd(N, src, dst, rel, X, W, W0, dOut, norm="in_degree_per_rel", act="none", out=None):
    src, dst, rel, X, W, W0, dOut = _i(src), _i(dst), _i(rel), _f(X), _f(W), _f(W0), _f(dOut)
    R, d_in, d_out = W.shape
    if out is None:
        out = rgcn_fwd(N, src, dst, rel, X, W, W0, norm, act)
    out = _f(out)
    dX = np.empty((N, d_in))
    dW = np.empty_like(W)
    dW0 = None if W0 is None else np.empty_like(W0)
    lib().oracle_rgcn_bwd(C.c_int64(N), C.c_int64(len(src)), C.c_int32(R), C.c_int32(d_in), C.c_int32(d_out),
                          _p(src), _p(dst), _p(rel), _p(X), _p(W), _p(W0),
                          C.c_int32(_NORM[norm]), C.c_int32(_ACT[act]), _p(out), _p(dOut),
                          _p(dX), _p(dW), _p(dW0))
    return dict(dX=dX, dW=dW, dW0=dW0)


def rgat_fwd(N, src, dst, rel, X, W, w_s, w_t, slope=0.2, want_alpha=False):
    src, dst, rel, X, W, w_s, w_t = _i(src), _i(dst), _i(rel), _f(X), _f(W), _f(w_s), _f(w_t)
    R, d_in, d_out = W.shape
    E = len(src)
    out = np.empty((N, d_out))
    alpha = np.zeros(E) if want_alpha else None
    z = np.zeros(E) if want_alpha else None
    lib().oracle_rgat_fwd(C.c_int64(N), C.c_int64(E), C.c_int32(R), C.c_int32(d_in), C.c_int32(d_out),
                          _p(src), _p(dst), _p(rel), _p(X), _p(W), _p(w_s), _p(w_t), C.c_double(slope),
                          _p(out), _p(alpha), _p(z))
    return (out, alpha, z) if want_alpha else out


def rgat_bwd(N, src, dst, rel, X, W, w_s, w_t, dOut, slope=0.2):
    src, dst, rel, X, W, w_s, w_t, dOut = _i(src), _i(dst), _i(rel), _f(X), _f(W), _f(w_s), _f(w_t), _f(dOut)
    R, d_in, d_out = W.shape
    dX = np.empty((N, d_in))
    dW = np.empty_like(W)
    dws = np.empty_like(w_s)
    dwt = np.empty_like(w_t)
    lib().oracle_rgat_bwd(C.c_int64(N), C.c_int64(len(src)), C.c_int32(R), C.c_int32(d_in), C.c_int32(d_out),
                          _p(src), _p(dst), _p(rel), _p(X), _p(W), _p(w_s), _p(w_t), C.c_double(slope),
                          _p(dOut), _p(dX), _p(dW), _p(dws), _p(dwt))
    return dict(dX=dX, dW=dW, dw_s=dws, dw_t=dwt)


def _head_slices(d_out, heads):
    if heads < 1 or d_out % heads:
        raise ValueError("heads must divide d_out")
    dh = d_out // heads
    return [slice(h * dh, (h + 1) * dh) for h in range(heads)]


def rgat_heads_fwd(N, src, dst, rel, X, W, w_s, w_t, heads, slope=0.2, want_alpha=False):
    """Multi-head RGAT: head h is the single-head layer of the listing on the column slice h of
    W, w_s, w_t (its own logits, its own softmax, its own messages); the outputs are concatenated.
    alpha, z: [E, heads]."""
    W, w_s, w_t = _f(W), _f(w_s), _f(w_t)
    out = np.empty((N, W.shape[2]))
    alpha = np.zeros((len(src), heads))
    z = np.zeros((len(src), heads))
    for h, sl in enumerate(_head_slices(W.shape[2], heads)):
        o, a, zz = rgat_fwd(N, src, dst, rel, X, W[:, :, sl], w_s[:, sl], w_t[:, sl], slope, want_alpha=True)
        out[:, sl], alpha[:, h], z[:, h] = o, a, zz
    return (out, alpha, z) if want_alpha else out


def rgat_heads_bwd(N, src, dst, rel, X, W, w_s, w_t, dOut, heads, slope=0.2):
    """Gradients of the concatenation: each head's parameter slices get that head's gradients, dX is
    the sum over the heads (every head reads the whole X)."""
    X, W, w_s, w_t, dOut = _f(X), _f(W), _f(w_s), _f(w_t), _f(dOut)
    g = dict(dX=np.zeros_like(X), dW=np.empty_like(W), dw_s=np.empty_like(w_s), dw_t=np.empty_like(w_t))
    for sl in _head_slices(W.shape[2], heads):
        gh = rgat_bwd(N, src, dst, rel, X, W[:, :, sl], w_s[:, sl], w_t[:, sl], dOut[:, sl], slope)
        g["dX"] += gh["dX"]
        g["dW"][:, :, sl], g["dw_s"][:, sl], g["dw_t"][:, sl] = gh["dW"], gh["dw_s"], gh["dw_t"]
    return g


def hgt_fwd(N, src, dst, rel, ntype, X, Wk, Wq, Wv, Wo, Watt, Wmsg, mu=None, want_alpha=False):
    src, dst, rel, ntype = _i(src), _i(dst), _i(rel), _i(ntype)
    X, Wk, Wq, Wv, Wo, Watt, Wmsg, mu = map(_f, (X, Wk, Wq, Wv, Wo, Watt, Wmsg, mu))
    T, d, _ = Wk.shape
    R, H = Watt.shape[:2]
    E = len(src)
    out = np.empty((N, d))
    alpha = np.zeros((E, H)) if want_alpha else None
    lib().oracle_hgt_fwd(C.c_int64(N), C.c_int64(E), C.c_int32(T), C.c_int32(R), C.c_int32(d), C.c_int32(H),
                         _p(src), _p(dst), _p(rel), _p(ntype), _p(X), _p(Wk), _p(Wq), _p(Wv), _p(Wo),
                         _p(Watt), _p(Wmsg), _p(mu), _p(out), _p(alpha))
    return (out, alpha) if want_alpha else out


def hgt_bwd(N, src, dst, rel, ntype, X, Wk, Wq, Wv, Wo, Watt, Wmsg, mu, dOut):
    src, dst, rel, ntype = _i(src), _i(dst), _i(rel), _i(ntype)
    X, Wk, Wq, Wv, Wo, Watt, Wmsg, mu, dOut = map(_f, (X, Wk, Wq, Wv, Wo, Watt, Wmsg, mu, dOut))
    T, d, _ = Wk.shape
    R, H = Watt.shape[:2]
    g = dict(dX=np.empty((N, d)), dWk=np.empty_like(Wk), dWq=np.empty_like(Wq), dWv=np.empty_like(Wv),
             dWo=np.empty_like(Wo), dWatt=np.empty_like(Watt), dWmsg=np.empty_like(Wmsg),
             dmu=None if mu is None else np.empty_like(mu))
    lib().oracle_hgt_bwd(C.c_int64(N), C.c_int64(len(src)), C.c_int32(T), C.c_int32(R), C.c_int32(d), C.c_int32(H),
                         _p(src), _p(dst), _p(rel), _p(ntype), _p(X), _p(Wk), _p(Wq), _p(Wv), _p(Wo),
                         _p(Watt), _p(Wmsg), _p(mu), _p(dOut),
                         _p(g["dX"]), _p(g["dWk"]), _p(g["dWq"]), _p(g["dWv"]), _p(g["dWo"]),
                         _p(g["dWatt"]), _p(g["dWmsg"]), _p(g["dmu"]))
    return g
