"""Thin ctypes binding of the C ABI in include/rgnn.h.

Argument marshalling only: every step of a layer runs in the HIP library.
PyTorch is used by callers for device memory and streams; this module just
takes raw device pointers (ints), torch tensors (via data_ptr()) or, for
rgnn_graph_create with mem=HOST, numpy int32 arrays.  There is no fallback:
if the library is missing or a call fails, an exception is raised.
"""
import ctypes as C
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "librgnn.so")

RGNN_OK = 0
RGNN_F32, RGNN_BF16 = 0, 1
RGNN_LAYER_RGCN, RGNN_LAYER_RGAT, RGNN_LAYER_HGT = 0, 1, 2
RGNN_NORM_NONE, RGNN_NORM_IN_DEGREE_PER_REL = 0, 1
RGNN_ACT_NONE, RGNN_ACT_RELU = 0, 1
RGNN_FLAG_EDGE_PARALLEL_AGGREGATION = 1
RGNN_FLAG_NO_BATCHED_WALKS = 2
RGNN_FLAG_NO_ROW_SELECT = 4
RGNN_FLAG_NO_WEIGHT_FOLDING = 8
RGNN_FLAG_SEPARATE_SOFTMAX = 16
RGNN_FLAG_ACCUMULATE = 32
RGNN_MEM_HOST, RGNN_MEM_DEVICE = 0, 1
RGNN_COO, RGNN_CSR_DST = 0, 1
RGNN_STATIC_SCRATCH_BYTES = 64 << 20

INDEX_NAMES = ["in_ptr", "in_src", "in_rel", "in_eid", "in_pair", "in_run", "in_cnt", "pair_ptr", "pair_src",
               "pair_rel", "run_ptr", "run_dst", "run_rel", "dst_run_ptr", "relrun_ptr", "relrun_idx", "out_ptr",
               "out_epos", "out_dst", "srcpair_ptr", "srcpair_idx", "ntype_ptr", "ntype_perm", "relrun_dst", "in_pair_tag",
               "pair_sel_dst", "rel_src_type"]

EXPORTS = ["rgnn_last_error", "rgnn_graph_create", "rgnn_graph_destroy", "rgnn_graph_info", "rgnn_graph_export",
           "rgnn_workspace_bytes", "rgnn_rgcn_fwd", "rgnn_rgcn_bwd", "rgnn_rgat_fwd", "rgnn_rgat_bwd",
           "rgnn_hgt_fwd", "rgnn_hgt_bwd", "rgnn_profile_start", "rgnn_profile_stop", "rgnn_profile_select", "rgnn_rgat_fwd_static", "rgnn_schedule"]


class RgnnError(RuntimeError):
    def __init__(self, status, msg):
        super().__init__(f"rgnn status {status}: {msg}")
        self.status = status


class GraphInfo(C.Structure):
    _fields_ = [("num_nodes", C.c_int64), ("num_edges", C.c_int64), ("num_pairs", C.c_int64),
                ("num_runs", C.c_int64), ("max_in_degree", C.c_int64), ("max_pair_out_degree", C.c_int64),
                ("index_bytes", C.c_int64), ("num_rels", C.c_int32), ("num_ntypes", C.c_int32),
                ("num_single_pairs", C.c_int64)]


class LayerDesc(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("d_in", C.c_int32), ("d_out", C.c_int32), ("heads", C.c_int32),
                ("slope", C.c_float), ("norm", C.c_int32), ("activation", C.c_int32), ("flags", C.c_uint32)]


class Schedule(C.Structure):
    _fields_ = [(k, C.c_int32) for k in (
        "item_len", "tile_chunks", "wide_chunks", "rows_bf16", "row_select", "hgt_folded", "fused_softmax", "ws_in_lds",
        "edge_parallel", "dst_batched_single", "dst_batched_short", "pair_walk_multi_only", "pair_batched_single",
        "pair_batched_short")]

    def as_dict(self):
        return {k: int(getattr(self, k)) for k, _ in self._fields_}


_lib = None


def lib():
    """Load librgnn.so (built beforehand by build.py / __graft_entry__.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2412_04747_amd.build` first")
        _lib = C.CDLL(LIB_PATH)
        _lib.rgnn_last_error.restype = C.c_char_p
        for name in EXPORTS[1:]:
            getattr(_lib, name).restype = C.c_int
    return _lib


def _check(status):
    if status != RGNN_OK:
        raise RgnnError(status, lib().rgnn_last_error().decode())


def _ptr(x):
    """Raw pointer of None / int / numpy array / torch tensor."""
    if x is None:
        return C.c_void_p(None)
    if isinstance(x, int):
        return C.c_void_p(x)
    if isinstance(x, np.ndarray):
        return C.c_void_p(x.ctypes.data)
    return C.c_void_p(x.data_ptr())      # torch tensor


def make_desc(dtype=RGNN_F32, d_in=64, d_out=64, heads=1, slope=0.2, norm=RGNN_NORM_NONE,
              activation=RGNN_ACT_NONE, flags=0):
    return LayerDesc(dtype, d_in, d_out, heads, slope, norm, activation, flags)


def rgnn_graph_create(num_nodes, num_ntypes, num_rels, num_edges, fmt, a, b, rel, ntype=None,
                      rel_src_ntype=None, rel_dst_ntype=None, mem=RGNN_MEM_HOST):
    g = C.c_void_p()
    _check(lib().rgnn_graph_create(C.byref(g), C.c_int64(num_nodes), C.c_int32(num_ntypes), C.c_int32(num_rels),
                                   C.c_int64(num_edges), C.c_int32(fmt), _ptr(a), _ptr(b), _ptr(rel), _ptr(ntype),
                                   _ptr(rel_src_ntype), _ptr(rel_dst_ntype), C.c_int32(mem)))
    return g


def rgnn_graph_destroy(g):
    _check(lib().rgnn_graph_destroy(g))


def rgnn_graph_info(g):
    info = GraphInfo()
    _check(lib().rgnn_graph_info(g, C.byref(info)))
    return info


def rgnn_graph_export(g, which, length):
    out = np.empty(length, np.int32)
    _check(lib().rgnn_graph_export(g, C.c_int32(which), _ptr(out), C.c_size_t(out.nbytes)))
    return out


def rgnn_workspace_bytes(g, layer, desc):
    f, b, s = C.c_size_t(), C.c_size_t(), C.c_size_t()
    _check(lib().rgnn_workspace_bytes(g, C.c_int32(layer), C.byref(desc), C.byref(f), C.byref(b), C.byref(s)))
    return f.value, b.value, s.value


def rgnn_schedule(g, layer, desc):
    """The schedule / layout choices of a layer configuration on a graph, as a dict."""
    out = Schedule()
    _check(lib().rgnn_schedule(g, C.c_int32(layer), C.byref(desc), C.byref(out)))
    return out.as_dict()


def rgnn_rgcn_fwd(g, desc, X, W, W0, out, saved, workspace, stream=None):
    _check(lib().rgnn_rgcn_fwd(g, C.byref(desc), _ptr(X), _ptr(W), _ptr(W0), _ptr(out), _ptr(saved),
                               _ptr(workspace), _ptr(stream)))


def rgnn_rgcn_bwd(g, desc, X, W, W0, out, saved, dOut, dX, dW, dW0, workspace, stream=None):
    _check(lib().rgnn_rgcn_bwd(g, C.byref(desc), _ptr(X), _ptr(W), _ptr(W0), _ptr(out), _ptr(saved), _ptr(dOut),
                               _ptr(dX), _ptr(dW), _ptr(dW0), _ptr(workspace), _ptr(stream)))


def rgnn_rgat_fwd(g, desc, X, W, w_s, w_t, out, saved, workspace, stream=None):
    _check(lib().rgnn_rgat_fwd(g, C.byref(desc), _ptr(X), _ptr(W), _ptr(w_s), _ptr(w_t), _ptr(out), _ptr(saved),
                               _ptr(workspace), _ptr(stream)))


def rgnn_rgat_fwd_static(g, desc, X, W, w_s, w_t, out, saved, stream=None):
    _check(lib().rgnn_rgat_fwd_static(g, C.byref(desc), _ptr(X), _ptr(W), _ptr(w_s), _ptr(w_t), _ptr(out),
                                      _ptr(saved), _ptr(stream)))


def rgnn_rgat_bwd(g, desc, X, W, w_s, w_t, out, saved, dOut, dX, dW, dw_s, dw_t, workspace, stream=None):
    _check(lib().rgnn_rgat_bwd(g, C.byref(desc), _ptr(X), _ptr(W), _ptr(w_s), _ptr(w_t), _ptr(out), _ptr(saved),
                               _ptr(dOut), _ptr(dX), _ptr(dW), _ptr(dw_s), _ptr(dw_t), _ptr(workspace),
                               _ptr(stream)))


def rgnn_hgt_fwd(g, desc, X, Wk, Wq, Wv, Wo, Watt, Wmsg, mu, out, saved, workspace, stream=None):
    _check(lib().rgnn_hgt_fwd(g, C.byref(desc), _ptr(X), _ptr(Wk), _ptr(Wq), _ptr(Wv), _ptr(Wo), _ptr(Watt),
                              _ptr(Wmsg), _ptr(mu), _ptr(out), _ptr(saved), _ptr(workspace), _ptr(stream)))


def rgnn_hgt_bwd(g, desc, X, Wk, Wq, Wv, Wo, Watt, Wmsg, mu, out, saved, dOut, dX, dWk, dWq, dWv, dWo, dWatt,
                 dWmsg, dmu, workspace, stream=None):
    _check(lib().rgnn_hgt_bwd(g, C.byref(desc), _ptr(X), _ptr(Wk), _ptr(Wq), _ptr(Wv), _ptr(Wo), _ptr(Watt),
                              _ptr(Wmsg), _ptr(mu), _ptr(out), _ptr(saved), _ptr(dOut), _ptr(dX), _ptr(dWk),
                              _ptr(dWq), _ptr(dWv), _ptr(dWo), _ptr(dWatt), _ptr(dWmsg), _ptr(dmu),
                              _ptr(workspace), _ptr(stream)))


def rgnn_profile_select(name=None):
    _check(lib().rgnn_profile_select(name.encode() if name else None))


def rgnn_profile_start():
    _check(lib().rgnn_profile_start())


def rgnn_profile_stop():
    """-> {kernel name: (launches, total milliseconds)} in first-launch order."""
    buf = C.create_string_buffer(1 << 16)
    _check(lib().rgnn_profile_stop(buf, C.c_size_t(len(buf))))
    rep = {}
    for line in buf.value.decode().splitlines():
        name, n, ms = line.split()
        rep[name] = (int(n), float(ms))
    return rep
