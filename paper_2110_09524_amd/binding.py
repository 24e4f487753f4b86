"""ctypes binding of libgnnfused.so: argument marshalling only.

Every function mirrors one entry point of include/gnn_fused.h and takes torch
tensors that live on the GPU (torch is used for device memory and streams, no
arithmetic happens here).  If the shared library is missing the import fails
loudly: there is no CPU or PyTorch fallback.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("GNNFUSED_LIB") or os.path.join(_HERE, "libgnnfused.so")

GNN_NUM_BUCKETS = 33
STATUS_NAMES = {0: "GNN_OK", 1: "GNN_ERR_INVALID_ARG", 2: "GNN_ERR_BAD_GRAPH",
                3: "GNN_ERR_WORKSPACE", 4: "GNN_ERR_UNSUPPORTED", 5: "GNN_ERR_HIP"}

EXPORTS = [
    "gnn_last_error", "gnn_graph_create", "gnn_graph_destroy", "gnn_graph_get_csc",
    "gnn_graph_get_buckets", "gnn_graph_get_blocked", "gnn_graph_get_launch_groups", "gnn_release_cached_memory", "gnn_config_set", "gnn_linear_fwd", "gnn_gat_workspace_bytes", "gnn_gat_fwd",
    "gnn_gat_bwd", "gnn_gat_bwd_noalloc", "gnn_gat_blocked_kernel_name", "gnn_gat_stash_layout", "gnn_gat_stash_alpha", "gnn_gat_bwd_stashed", "gnn_edgeconv_workspace_bytes", "gnn_edgeconv_fwd", "gnn_edgeconv_bwd",
    "gnn_gmm_workspace_bytes", "gnn_gmm_fwd", "gnn_gmm_bwd", "gnn_gmm_tune", "gnn_gmm_tune_bwd",
    "gnn_gmmp_workspace_bytes", "gnn_gmmp_fwd", "gnn_gmmp_bwd", "gnn_pseudo_proj_workspace_bytes",
    "gnn_pseudo_proj_fwd", "gnn_pseudo_proj_bwd", "gnn_monet_workspace_bytes", "gnn_monet_fwd", "gnn_monet_bwd",
    "gnn_gcn_workspace_bytes", "gnn_gcn_fwd", "gnn_gcn_bwd", "gnn_gcn_tune", "gnn_gcn_blocked_kernel_name",
    "gnn_edge_weights_create", "gnn_edge_weights_destroy", "gnn_gcn_edge_fwd", "gnn_gcn_edge_bwd",
    "gnn_bias_act_fwd", "gnn_bias_act_workspace_bytes", "gnn_bias_act_bwd", "gnn_softmax_xent_workspace_bytes",
    "gnn_softmax_xent", "gnn_sgd_update", "gnn_knn_graph", "gnn_prof_enable",
    "gnn_prof_collect", "gnn_prof_reset", "gnn_prof_count", "gnn_prof_get",
]


class GnnError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {text}")
        self.status = status


def load_library(path: str = LIB_PATH) -> C.CDLL:
    if not os.path.exists(path):
        raise ImportError(
            f"{path} is missing: build it with `python -m paper_2110_09524_amd.build` "
            "(there is no fallback path)")
    lib = C.CDLL(path)
    vp, i32, i64, f32, sz = C.c_void_p, C.c_int, C.c_int64, C.c_float, C.c_size_t
    lib.gnn_last_error.restype = C.c_char_p
    lib.gnn_last_error.argtypes = []
    lib.gnn_graph_create.argtypes = [C.c_int32, i64, vp, vp, vp, C.POINTER(vp)]
    lib.gnn_graph_destroy.argtypes = [vp]
    lib.gnn_graph_get_csc.argtypes = [vp, vp, vp, vp, vp]
    lib.gnn_graph_get_buckets.argtypes = [vp, i32, vp, vp, vp, vp]
    lib.gnn_graph_get_blocked.argtypes = [vp, i32, C.POINTER(C.c_int32), C.POINTER(C.c_int32), vp, vp, vp]
    lib.gnn_graph_get_launch_groups.argtypes = [vp, i32, i32, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
    lib.gnn_config_set.argtypes = [C.c_char_p, i64]
    lib.gnn_release_cached_memory.argtypes = []
    lib.gnn_linear_fwd.argtypes = [i64, i32, i32, vp, vp, vp, vp]
    lib.gnn_gat_workspace_bytes.restype = sz
    lib.gnn_gat_workspace_bytes.argtypes = [vp, i32, i32, i32]
    lib.gnn_gat_fwd.argtypes = [vp, i32, i32, i32, f32] + [vp] * 12 + [vp, sz, vp]
    lib.gnn_gat_bwd.argtypes = [vp, i32, i32, i32, f32] + [vp] * 17 + [vp, sz, vp]
    lib.gnn_gat_bwd_noalloc.argtypes = [vp, i32, i32, i32, f32] + [vp] * 17 + [vp]
    lib.gnn_gat_blocked_kernel_name.argtypes = [vp, i32, i32, i32, C.c_char_p, sz]
    lib.gnn_gcn_blocked_kernel_name.argtypes = [vp, i32, i32, C.c_char_p, sz]
    lib.gnn_gat_stash_alpha.argtypes = [vp, i32, i32, f32] + [vp] * 5 + [vp]
    lib.gnn_gat_stash_layout.argtypes = [vp, i32, i32]
    lib.gnn_gat_stash_layout.restype = i32
    lib.gnn_gat_bwd_stashed.argtypes = [vp, i32, i32, i32, f32] + [vp] * 18 + [vp, sz, vp]
    lib.gnn_edgeconv_workspace_bytes.restype = sz
    lib.gnn_edgeconv_workspace_bytes.argtypes = [vp, i32, i32]
    lib.gnn_edgeconv_fwd.argtypes = [vp, i32, i32] + [vp] * 6 + [vp, sz, vp]
    lib.gnn_edgeconv_bwd.argtypes = [vp, i32, i32] + [vp] * 8 + [vp, sz, vp]
    lib.gnn_gmm_workspace_bytes.restype = sz
    lib.gnn_gmm_workspace_bytes.argtypes = [vp, i32, i32, i32]
    lib.gnn_gmm_fwd.argtypes = [vp, i32, i32, i32] + [vp] * 7 + [vp, sz, vp]
    lib.gnn_gmm_bwd.argtypes = [vp, i32, i32, i32] + [vp] * 11 + [vp, sz, vp]
    lib.gnn_gmm_tune.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp, vp, C.POINTER(C.c_float)]
    lib.gnn_gmm_tune_bwd.argtypes = [vp, i32, i32, i32, vp, vp, vp, vp, vp, vp, C.c_size_t, vp, C.POINTER(C.c_float)]
    lib.gnn_gmmp_workspace_bytes.restype = sz
    lib.gnn_gmmp_workspace_bytes.argtypes = [vp, i32, i32, i32]
    lib.gnn_gmmp_fwd.argtypes = [vp, i32, i32, i32, i32] + [vp] * 7 + [vp]
    lib.gnn_gmmp_bwd.argtypes = [vp, i32, i32, i32, i32] + [vp] * 13 + [vp, sz, vp]
    lib.gnn_pseudo_proj_workspace_bytes.restype = sz
    lib.gnn_pseudo_proj_workspace_bytes.argtypes = [vp]
    lib.gnn_monet_workspace_bytes.restype = sz
    lib.gnn_monet_workspace_bytes.argtypes = [vp, i32, i32, i32]
    lib.gnn_monet_fwd.argtypes = [vp, i32, i32, i32, i32] + [vp] * 9 + [vp]
    lib.gnn_monet_bwd.argtypes = [vp, i32, i32, i32, i32] + [vp] * 15 + [vp, sz, vp]
    lib.gnn_pseudo_proj_fwd.argtypes = [vp, i32, vp, vp, vp, vp, vp, vp]
    lib.gnn_pseudo_proj_bwd.argtypes = [vp, i32, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.gnn_gcn_workspace_bytes.restype = sz
    lib.gnn_gcn_workspace_bytes.argtypes = [vp, i32, i32]
    lib.gnn_gcn_fwd.argtypes = [vp, i32, i32] + [vp] * 6 + [vp]
    lib.gnn_gcn_bwd.argtypes = [vp, i32, i32] + [vp] * 7 + [vp, sz, vp]
    lib.gnn_gcn_tune.argtypes = [vp, i32, vp, sz, vp, C.POINTER(C.c_float)]
    lib.gnn_edge_weights_create.argtypes = [vp, vp, vp, C.POINTER(vp)]
    lib.gnn_edge_weights_destroy.argtypes = [vp]
    lib.gnn_gcn_edge_fwd.argtypes = [vp, vp, i32, i32] + [vp] * 4 + [vp]
    lib.gnn_gcn_edge_bwd.argtypes = [vp, vp, i32, i32] + [vp] * 5 + [vp, sz, vp]
    lib.gnn_bias_act_fwd.argtypes = [i64, i32, i32, f32, vp, vp, vp, vp]
    lib.gnn_bias_act_workspace_bytes.restype = sz
    lib.gnn_bias_act_workspace_bytes.argtypes = [i64, i32]
    lib.gnn_bias_act_bwd.argtypes = [i64, i32, i32, f32, vp, vp, vp, vp, vp, sz, vp]
    lib.gnn_softmax_xent_workspace_bytes.restype = sz
    lib.gnn_softmax_xent_workspace_bytes.argtypes = [i64]
    lib.gnn_softmax_xent.argtypes = [i64, i32, i64, vp, vp, vp, vp, vp, sz, vp]
    lib.gnn_sgd_update.argtypes = [i64, f32, vp, vp, vp]
    lib.gnn_knn_graph.argtypes = [i32, i32, i32, i32, vp, vp, vp, vp]
    lib.gnn_prof_enable.argtypes = [i32]
    lib.gnn_prof_collect.argtypes = []
    lib.gnn_prof_reset.argtypes = []
    lib.gnn_prof_count.argtypes = []
    lib.gnn_prof_get.argtypes = [i32, C.POINTER(C.c_char_p), C.POINTER(C.c_double), C.POINTER(i64)]
    for name in EXPORTS:
        fn = getattr(lib, name)
        if name not in ("gnn_last_error", "gnn_gat_workspace_bytes", "gnn_edgeconv_workspace_bytes",
                        "gnn_gmm_workspace_bytes", "gnn_gcn_workspace_bytes", "gnn_prof_count",
                        "gnn_bias_act_workspace_bytes", "gnn_softmax_xent_workspace_bytes",
                        "gnn_gmmp_workspace_bytes", "gnn_pseudo_proj_workspace_bytes", "gnn_monet_workspace_bytes"):
            fn.restype = C.c_int
    return lib


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        _lib = load_library()
    return _lib


def _check(status: int):
    if status != 0:
        raise GnnError(status, lib().gnn_last_error().decode())


def _ptr(t, dtype=None):
    if t is None:
        return None
    if not isinstance(t, torch.Tensor):
        raise TypeError("expected a torch tensor")
    if not t.is_cuda:
        raise ValueError("tensor must live on the GPU")
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"expected {dtype}, got {t.dtype}")
    return C.c_void_p(t.data_ptr())


def _f(t):
    return _ptr(t, torch.float32)


def _i(t):
    return _ptr(t, torch.int32)


def _stream(stream=None):
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


class Graph:
    """Handle of gnn_graph_create.  Keeps the borrowed CSR tensors alive."""

    def __init__(self, indptr: torch.Tensor, indices: torch.Tensor, stream=None):
        self.indptr, self.indices = indptr, indices
        self.n = indptr.numel() - 1
        self.nnz = indices.numel()
        self.device = indptr.device
        h = C.c_void_p()
        _check(lib().gnn_graph_create(self.n, self.nnz, _i(indptr), _i(indices) if self.nnz else None,
                                      _stream(stream), C.byref(h)))
        self._h = h

    def close(self):
        if getattr(self, "_h", None):
            lib().gnn_graph_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def handle(self):
        return self._h

    def csc(self, stream=None):
        ip = torch.empty(self.n + 1, dtype=torch.int32, device=self.device)
        ix = torch.empty(self.nnz, dtype=torch.int32, device=self.device)
        eid = torch.empty(self.nnz, dtype=torch.int32, device=self.device)
        _check(lib().gnn_graph_get_csc(self._h, _i(ip), _i(ix), _i(eid), _stream(stream)))
        return ip, ix, eid

    def blocked(self, side: int, stream=None):
        """(num_blocks, block_cols, bptr, bcol); the tensors are None when num_blocks == 1."""
        nb, bc = C.c_int32(), C.c_int32()
        _check(lib().gnn_graph_get_blocked(self._h, side, C.byref(nb), C.byref(bc), None, None,
                                           _stream(stream)))
        if nb.value <= 1:
            return nb.value, bc.value, None, None
        bptr = torch.empty(nb.value * self.n + 1, dtype=torch.int32, device=self.device)
        bcol = torch.empty(self.nnz, dtype=torch.int32, device=self.device)
        _check(lib().gnn_graph_get_blocked(self._h, side, C.byref(nb), C.byref(bc), _i(bptr), _i(bcol),
                                           _stream(stream)))
        return nb.value, bc.value, bptr, bcol

    def launch_groups(self, side: int, sums: int):
        """Block boundaries of the launches of a column-blocked kernel that keeps `sums` running sums
        per row: group j covers blocks result[j] .. result[j + 1] - 1 ([] without blocked lists)."""
        cnt = C.c_int32()
        _check(lib().gnn_graph_get_launch_groups(self._h, side, sums, None, C.byref(cnt)))
        if cnt.value == 0:
            return []
        buf = (C.c_int32 * (cnt.value + 1))()
        _check(lib().gnn_graph_get_launch_groups(self._h, side, sums, buf, C.byref(cnt)))
        return list(buf)

    def buckets(self, side: int, stream=None):
        b = torch.empty(self.n, dtype=torch.int32, device=self.device)
        o = torch.empty(self.n, dtype=torch.int32, device=self.device)
        off = torch.empty(GNN_NUM_BUCKETS + 1, dtype=torch.int32, device=self.device)
        _check(lib().gnn_graph_get_buckets(self._h, side, _i(b), _i(o), _i(off), _stream(stream)))
        return b, o, off


def gnn_config_set(key: str, value: int):
    _check(lib().gnn_config_set(key.encode(), int(value)))


def gnn_linear_fwd(x, w, y, stream=None):
    n, fin = x.shape
    _check(lib().gnn_linear_fwd(n, fin, w.shape[1], _f(x), _f(w), _f(y), _stream(stream)))


def _ws_args(ws):
    if ws is None:
        return None, 0
    return C.c_void_p(ws.data_ptr()), ws.numel() * ws.element_size()


def gnn_gat_workspace_bytes(g: Graph, fin, heads, f) -> int:
    return int(lib().gnn_gat_workspace_bytes(g.handle, fin, heads, f))


def gnn_gat_fwd(g: Graph, fin, heads, f, slope, x, w, a_l, a_r, z, el, er, m, d, out, t=None,
                sg=None, ws=None, stream=None):
    wp, wb = _ws_args(ws)
    _check(lib().gnn_gat_fwd(g.handle, fin, heads, f, slope, _f(x), _f(w), _f(a_l), _f(a_r), _f(z),
                             _f(el), _f(er), _f(m), _f(d), _f(out), _f(t), _f(sg), wp, wb,
                             _stream(stream)))


def gnn_gat_bwd(g: Graph, fin, heads, f, slope, x, w, a_l, a_r, z, el, er, m, d, out, t, sg, gout,
                gx, gw, ga_l, ga_r, ws, stream=None):
    wp, wb = _ws_args(ws)
    _check(lib().gnn_gat_bwd(g.handle, fin, heads, f, slope, _f(x), _f(w), _f(a_l), _f(a_r), _f(z),
                             _f(el), _f(er), _f(m), _f(d), _f(out), _f(t), _f(sg), _f(gout), _f(gx),
                             _f(gw), _f(ga_l), _f(ga_r), wp, wb, _stream(stream)))


def gnn_gat_blocked_kernel_name(g: Graph, heads, f, mode) -> str:
    buf = C.create_string_buffer(128)
    _check(lib().gnn_gat_blocked_kernel_name(g.handle, heads, f, mode, buf, 128))
    return buf.value.decode()


def gnn_gcn_blocked_kernel_name(g: Graph, fout, weighted=False) -> str:
    buf = C.create_string_buffer(128)
    _check(lib().gnn_gcn_blocked_kernel_name(g.handle, fout, int(bool(weighted)), buf, 128))
    return buf.value.decode()


NOALLOC_SCRATCH_BYTES = 64 << 20   # GNN_NOALLOC_SCRATCH_BYTES of the header


def gnn_gat_bwd_noalloc(g: Graph, fin, heads, f, slope, x, w, a_l, a_r, z, el, er, m, d, out, t, sg, gout,
                        gx, gw, ga_l, ga_r, stream=None):
    _check(lib().gnn_gat_bwd_noalloc(g.handle, fin, heads, f, slope, _f(x), _f(w), _f(a_l), _f(a_r), _f(z),
                                     _f(el), _f(er), _f(m), _f(d), _f(out), _f(t), _f(sg), _f(gout), _f(gx),
                                     _f(gw), _f(ga_l), _f(ga_r), _stream(stream)))


def gnn_gat_stash_layout(g: Graph, heads, f) -> int:
    return int(lib().gnn_gat_stash_layout(g.handle, heads, f))


def gnn_gat_stash_alpha(g: Graph, heads, f, slope, el, er, m, d, alpha_t, stream=None):
    _check(lib().gnn_gat_stash_alpha(g.handle, heads, f, slope, _f(el), _f(er), _f(m), _f(d), _f(alpha_t),
                                     _stream(stream)))


def gnn_gat_bwd_stashed(g: Graph, fin, heads, f, slope, x, w, a_l, a_r, z, el, er, m, d, out, t, sg, alpha_t,
                        gout, gx, gw, ga_l, ga_r, ws, stream=None):
    wp, wb = _ws_args(ws)
    _check(lib().gnn_gat_bwd_stashed(g.handle, fin, heads, f, slope, _f(x), _f(w), _f(a_l), _f(a_r), _f(z),
                                     _f(el), _f(er), _f(m), _f(d), _f(out), _f(t), _f(sg), _f(alpha_t),
                                     _f(gout), _f(gx), _f(gw), _f(ga_l), _f(ga_r), wp, wb, _stream(stream)))


def gnn_edgeconv_workspace_bytes(g: Graph, fin, fout) -> int:
    return int(lib().gnn_edgeconv_workspace_bytes(g.handle, fin, fout))


def gnn_edgeconv_fwd(g: Graph, fin, fout, x, theta, phi, pq, out, argmax, ws=None, stream=None):
    wp, wb = _ws_args(ws)
    _check(lib().gnn_edgeconv_fwd(g.handle, fin, fout, _f(x), _f(theta), _f(phi), _f(pq), _f(out),
                                  _i(argmax), wp, wb, _stream(stream)))


def gnn_edgeconv_bwd(g: Graph, fin, fout, x, theta, phi, argmax, gout, gx, gtheta, gphi, ws,
                     stream=None):
    wp, wb = _ws_args(ws)
    _check(lib().gnn_edgeconv_bwd(g.handle, fin, fout, _f(x), _f(theta), _f(phi), _i(argmax), _f(gout),
                                  _f(gx), _f(gtheta), _f(gphi), wp, wb, _stream(stream)))


def gnn_gcn_workspace_bytes(g: Graph, fin, fout) -> int:
    return int(lib().gnn_gcn_workspace_bytes(g.handle, fin, fout))


def gnn_gcn_fwd(g: Graph, fin, fout, x, w, c_src, c_dst, zs, out, stream=None):
    _check(lib().gnn_gcn_fwd(g.handle, fin, fout, _f(x), _f(w), _f(c_src), _f(c_dst), _f(zs), _f(out),
                             _stream(stream)))


def gnn_gcn_bwd(g: Graph, fin, fout, x, w, c_src, c_dst, gout, gx, gw, ws, stream=None):
    wp, wb = _ws_args(ws)
    _check(lib().gnn_gcn_bwd(g.handle, fin, fout, _f(x), _f(w), _f(c_src), _f(c_dst), _f(gout), _f(gx),
                             _f(gw), wp, wb, _stream(stream)))


class EdgeWeights:
    """Handle of gnn_edge_weights_create: a static scalar per edge ([nnz], CSR order) copied into
    every order the kernels walk.  Keeps its graph alive; close it before the graph."""

    def __init__(self, g: Graph, edge_w: torch.Tensor, stream=None):
        self.graph = g
        h = C.c_void_p()
        _check(lib().gnn_edge_weights_create(g.handle, _f(edge_w) if g.nnz else None, _stream(stream), C.byref(h)))
        self._h = h

    def close(self):
        if getattr(self, "_h", None):
            lib().gnn_edge_weights_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def handle(self):
        return self._h


def gnn_gcn_edge_fwd(g: Graph, ew: EdgeWeights, fin, fout, x, w, z, out, stream=None):
    _check(lib().gnn_gcn_edge_fwd(g.handle, ew.handle, fin, fout, _f(x), _f(w), _f(z), _f(out), _stream(stream)))


def gnn_gcn_edge_bwd(g: Graph, ew: EdgeWeights, fin, fout, x, w, gout, gx, gw, ws, stream=None):
    wp, wb = _ws_args(ws)
    _check(lib().gnn_gcn_edge_bwd(g.handle, ew.handle, fin, fout, _f(x), _f(w), _f(gout), _f(gx), _f(gw), wp, wb,
                                  _stream(stream)))


def gnn_gcn_tune(g: Graph, fout, ws, stream=None):
    """Returns the four measured times (ms): in-edge side vertex-/edge-balanced, out-edge side likewise."""
    wp, wb = _ws_args(ws)
    ms = (C.c_float * 4)()
    _check(lib().gnn_gcn_tune(g.handle, fout, wp, wb, _stream(stream), ms))
    return [float(v) for v in ms]


def gnn_gmm_tune(g: Graph, fout, k, hk, c, mu, inv_sigma, out, stream=None):
    """Returns the two measured times (ms): vertex-balanced, edge-balanced forward aggregation."""
    ms = (C.c_float * 2)()
    _check(lib().gnn_gmm_tune(g.handle, fout, k, _f(hk), _f(c), _f(mu), _f(inv_sigma), _f(out), _stream(stream), ms))
    return [float(v) for v in ms]


def gnn_gmm_tune_bwd(g: Graph, fin, fout, k, hk, c, mu, inv_sigma, gout, ws, stream=None):
    """Returns the four measured times (ms): destination side vertex-/edge-balanced, source side likewise."""
    wp, wb = _ws_args(ws)
    ms = (C.c_float * 4)()
    _check(lib().gnn_gmm_tune_bwd(g.handle, fin, fout, k, _f(hk), _f(c), _f(mu), _f(inv_sigma), _f(gout), wp, wb,
                                  _stream(stream), ms))
    return [float(v) for v in ms]


def gnn_gmmp_workspace_bytes(g: Graph, fin, fout, k) -> int:
    return int(lib().gnn_gmmp_workspace_bytes(g.handle, fin, fout, k))


def gnn_gmmp_fwd(g: Graph, fin, fout, k, r, x, w_fc, pseudo, mu, inv_sigma, hk, out, stream=None):
    _check(lib().gnn_gmmp_fwd(g.handle, fin, fout, k, r, _f(x), _f(w_fc), _f(pseudo), _f(mu), _f(inv_sigma),
                              _f(hk), _f(out), _stream(stream)))


def gnn_gmmp_bwd(g: Graph, fin, fout, k, r, x, w_fc, pseudo, mu, inv_sigma, hk, gout, gx, gw_fc, gmu, ginv_sigma,
                 gpseudo, ws, stream=None, pseudo_t=None):
    wp, wb = _ws_args(ws)
    _check(lib().gnn_gmmp_bwd(g.handle, fin, fout, k, r, _f(x), _f(w_fc), _f(pseudo), _f(mu), _f(inv_sigma),
                              _f(hk), _f(gout), _f(gx), _f(gw_fc), _f(gmu), _f(ginv_sigma), _f(gpseudo),
                              _f(pseudo_t), wp, wb, _stream(stream)))


def gnn_pseudo_proj_workspace_bytes(g: Graph) -> int:
    return int(lib().gnn_pseudo_proj_workspace_bytes(g.handle))


def gnn_pseudo_proj_fwd(g: Graph, r, c, proj_w, proj_b, pseudo, stream=None, pseudo_t=None):
    _check(lib().gnn_pseudo_proj_fwd(g.handle, r, _f(c), _f(proj_w), _f(proj_b), _f(pseudo), _f(pseudo_t),
                                     _stream(stream)))


def gnn_pseudo_proj_bwd(g: Graph, r, c, pseudo, gpseudo, gproj_w, gproj_b, ws, stream=None):
    wp, wb = _ws_args(ws)
    _check(lib().gnn_pseudo_proj_bwd(g.handle, r, _f(c), _f(pseudo), _f(gpseudo), _f(gproj_w), _f(gproj_b), wp, wb,
                                     _stream(stream)))


def gnn_monet_workspace_bytes(g: Graph, fin, fout, k) -> int:
    return int(lib().gnn_monet_workspace_bytes(g.handle, fin, fout, k))


def gnn_monet_fwd(g: Graph, fin, fout, k, r, x, w_fc, c, proj_w, proj_b, mu, inv_sigma, hk, out, stream=None):
    _check(lib().gnn_monet_fwd(g.handle, fin, fout, k, r, _f(x), _f(w_fc), _f(c), _f(proj_w), _f(proj_b), _f(mu),
                               _f(inv_sigma), _f(hk), _f(out), _stream(stream)))


def gnn_monet_bwd(g: Graph, fin, fout, k, r, x, w_fc, c, proj_w, proj_b, mu, inv_sigma, hk, gout, gx, gw_fc, gmu,
                  ginv_sigma, gproj_w, gproj_b, ws, stream=None):
    wp, wb = _ws_args(ws)
    _check(lib().gnn_monet_bwd(g.handle, fin, fout, k, r, _f(x), _f(w_fc), _f(c), _f(proj_w), _f(proj_b), _f(mu),
                               _f(inv_sigma), _f(hk), _f(gout), _f(gx), _f(gw_fc), _f(gmu), _f(ginv_sigma),
                               _f(gproj_w), _f(gproj_b), wp, wb, _stream(stream)))


def gnn_release_cached_memory():
    _check(lib().gnn_release_cached_memory())


ACTS = {"identity": 0, "relu": 1, "elu": 2, "leaky": 3}


def gnn_bias_act_fwd(n, f, act, slope, x, bias, out, stream=None):
    _check(lib().gnn_bias_act_fwd(n, f, ACTS[act], slope, _f(x), _f(bias), _f(out), _stream(stream)))


def gnn_bias_act_workspace_bytes(n, f) -> int:
    return int(lib().gnn_bias_act_workspace_bytes(n, f))


def gnn_bias_act_bwd(n, f, act, slope, y, gout, gin, gbias, ws=None, stream=None):
    wp, wb = _ws_args(ws)
    _check(lib().gnn_bias_act_bwd(n, f, ACTS[act], slope, _f(y), _f(gout), _f(gin), _f(gbias), wp, wb,
                                  _stream(stream)))


def gnn_softmax_xent_workspace_bytes(n) -> int:
    return int(lib().gnn_softmax_xent_workspace_bytes(n))


def gnn_softmax_xent(n, c, n_labelled, logits, labels, loss, glogits, ws, stream=None):
    wp, wb = _ws_args(ws)
    _check(lib().gnn_softmax_xent(n, c, n_labelled, _f(logits), _i(labels), _f(loss), _f(glogits), wp, wb,
                                  _stream(stream)))


def gnn_sgd_update(lr, grad, param, stream=None):
    assert grad.numel() == param.numel()
    _check(lib().gnn_sgd_update(param.numel(), lr, _f(grad), _f(param), _stream(stream)))


def gnn_knn_graph(clouds, points, dim, k, coords, indptr, indices, stream=None):
    _check(lib().gnn_knn_graph(clouds, points, dim, k, _f(coords), _i(indptr), _i(indices), _stream(stream)))


def gnn_gmm_workspace_bytes(g: Graph, fin, fout, k) -> int:
    return int(lib().gnn_gmm_workspace_bytes(g.handle, fin, fout, k))


def gnn_gmm_fwd(g: Graph, fin, fout, k, x, w_fc, c, mu, inv_sigma, hk, out, ws=None, stream=None):
    wp, wb = _ws_args(ws)
    _check(lib().gnn_gmm_fwd(g.handle, fin, fout, k, _f(x), _f(w_fc), _f(c), _f(mu), _f(inv_sigma),
                             _f(hk), _f(out), wp, wb, _stream(stream)))


def gnn_gmm_bwd(g: Graph, fin, fout, k, x, w_fc, c, mu, inv_sigma, hk, gout, gx, gw_fc, gmu,
                ginv_sigma, ws, stream=None):
    wp, wb = _ws_args(ws)
    _check(lib().gnn_gmm_bwd(g.handle, fin, fout, k, _f(x), _f(w_fc), _f(c), _f(mu), _f(inv_sigma),
                             _f(hk), _f(gout), _f(gx), _f(gw_fc), _f(gmu), _f(ginv_sigma), wp, wb,
                             _stream(stream)))


def gnn_prof_enable(on: bool):
    _check(lib().gnn_prof_enable(1 if on else 0))


def gnn_prof_reset():
    _check(lib().gnn_prof_reset())


def gnn_prof_report() -> dict:
    """{kernel name: (total_ms, launches)} of everything timed since the last reset."""
    _check(lib().gnn_prof_collect())
    res = {}
    for i in range(lib().gnn_prof_count()):
        name, ms, cnt = C.c_char_p(), C.c_double(), C.c_int64()
        _check(lib().gnn_prof_get(i, C.byref(name), C.byref(ms), C.byref(cnt)))
        res[name.value.decode()] = (ms.value, cnt.value)
    return res
