"""ctypes binding of libhgnn.so: argument marshalling only.

Every function mirrors a C entry point of include/hgnn.h with the same name.
PyTorch tensors are used as device memory (their `data_ptr()` is passed) and for
the current stream; no step of the path is computed here.  There is no fallback:
if the shared library has not been built, importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhgnn.so")

HGNN_OK = 0
HGNN_F32, HGNN_BF16 = 0, 1
STATUS_NAMES = {0: "HGNN_OK", -1: "HGNN_EINVAL", -2: "HGNN_ENOMEM", -3: "HGNN_EHIP",
                -4: "HGNN_EOVERFLOW", -5: "HGNN_ENOTREADY", -6: "HGNN_EUNSUPPORTED"}


class HgnnError(RuntimeError):
    def __init__(self, status, msg):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {msg}")
        self.status = status


class Schema(C.Structure):
    _fields_ = [("num_types", C.c_int32), ("num_rels", C.c_int32),
                ("rel_src_type", C.POINTER(C.c_int32)), ("rel_dst_type", C.POINTER(C.c_int32)),
                ("heads", C.c_int32), ("agg", C.c_int32), ("fuse", C.c_int32), ("dtype", C.c_int32)]


class CooLayer(C.Structure):
    _fields_ = [("num_edges", C.c_int64), ("edge_index", C.c_void_p), ("index_is_i64", C.c_int32),
                ("edge_type", C.c_void_p), ("edge_id", C.c_void_p), ("global_edge_type", C.c_void_p),
                ("num_global_edges", C.c_int64), ("n_src", C.c_void_p), ("n_dst", C.c_void_p),
                ("transpose_types", C.c_void_p)]


class CsrView(C.Structure):
    _fields_ = [("rows", C.c_int64), ("edges", C.c_int64), ("src_rows", C.c_int64), ("transpose_edges", C.c_int64)] + \
               [(k, C.POINTER(C.c_int32)) for k in
                ("rel_row_off", "rel_edge_off", "rowptr", "colidx", "perm", "cptr", "crow", "cperm")]


class HostGraph(C.Structure):
    _fields_ = [("num_nodes", C.POINTER(C.c_int64)), ("in_indptr", C.POINTER(C.c_void_p)),
                ("in_nbr", C.POINTER(C.c_void_p)), ("edge_off", C.POINTER(C.c_int64))]


MAX_TYPES = 32


class MinibatchView(C.Structure):
    _fields_ = [("n_src", C.c_int64 * MAX_TYPES), ("n_dst", C.c_int64 * MAX_TYPES), ("num_edges", C.c_int64),
                ("edge_index", C.POINTER(C.c_int64)), ("edge_id", C.POINTER(C.c_int64))]


class AdamParams(C.Structure):
    _fields_ = [("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float), ("step", C.c_int64)]


class LayerParams(C.Structure):
    _fields_ = [("in_dim", C.POINTER(C.c_int32)), ("out_dim", C.c_int32), ("relu", C.c_int32),
                ("w_rel", C.POINTER(C.c_void_p)), ("w_root", C.POINTER(C.c_void_p)),
                ("bias", C.POINTER(C.c_void_p)), ("input_grad", C.POINTER(C.c_int32)),
                ("w_type", C.POINTER(C.c_void_p)), ("a_src", C.POINTER(C.c_void_p)), ("a_dst", C.POINTER(C.c_void_p)),
                ("w_sem", C.c_void_p), ("b_sem", C.c_void_p), ("q_sem", C.c_void_p)]


class LayerGrads(C.Structure):
    _fields_ = [("dw_rel", C.POINTER(C.c_void_p)), ("dw_root", C.POINTER(C.c_void_p)),
                ("dbias", C.POINTER(C.c_void_p)),
                ("dw_type", C.POINTER(C.c_void_p)), ("da_src", C.POINTER(C.c_void_p)), ("da_dst", C.POINTER(C.c_void_p)),
                ("dw_sem", C.c_void_p), ("db_sem", C.c_void_p), ("dq_sem", C.c_void_p)]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(hipcc, gfx950) first; there is no CPU fallback")
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    sig = {
        "hgnn_create": [C.POINTER(vp), C.POINTER(Schema), C.c_int, C.c_int, C.c_int],
        "hgnn_merge_features": [vp, vp, C.POINTER(vp), C.POINTER(i32), C.POINTER(vp), C.POINTER(i64), vp,
                                C.POINTER(i32), C.POINTER(i64)],
        "hgnn_merge_features_index_first": [vp, vp, C.POINTER(vp), C.POINTER(i32), C.POINTER(vp), C.POINTER(i64), C.POINTER(vp), vp],
        "hgnn_select_type_first": [vp, vp, vp, C.POINTER(i32), C.POINTER(vp), C.POINTER(i64), vp, C.POINTER(i32), C.POINTER(i64)],
        "hgnn_build_semantic_csr": [vp, i32, C.POINTER(CooLayer), C.POINTER(vp)],
        "hgnn_build_semantic_csr_device": [vp, vp, i32, C.POINTER(CooLayer), C.POINTER(vp), C.POINTER(C.c_float)],
        "hgnn_set_edge_types": [vp, vp, i64],
        "hgnn_set_build_permutation": [vp, i32],
        "hgnn_graph_wait": [vp, vp],
        "hgnn_sampler_create": [vp, C.POINTER(HostGraph), C.POINTER(vp)],
        "hgnn_sample_and_build": [vp, vp, i32, vp, i64, i32, C.POINTER(i32), C.c_uint64, C.POINTER(vp), C.POINTER(vp)],
        "hgnn_graph_ids": [vp, vp, C.POINTER(i64), C.POINTER(vp), C.POINTER(vp)],
        "hgnn_graph_minibatch_view": [vp, vp, i32, C.POINTER(MinibatchView)],
        "hgnn_graph_wait_stream": [vp, vp, vp],
        "hgnn_graph_host_view": [vp, vp, i32, C.POINTER(CsrView)],
        "hgnn_layer_workspace_bytes": [vp, vp, i32, C.POINTER(LayerParams), C.POINTER(C.c_size_t),
                                       C.POINTER(C.c_size_t)],
        "hgnn_layer_fwd": [vp, vp, vp, i32, C.POINTER(LayerParams), vp, vp, vp, C.c_size_t, vp, C.c_size_t],
        "hgnn_layer_fwd_gather": [vp, vp, vp, i32, C.POINTER(LayerParams), C.POINTER(vp), C.POINTER(vp), vp, vp, vp, C.c_size_t, vp,
                                  C.c_size_t],
        "hgnn_layer_bwd_gather": [vp, vp, vp, i32, C.POINTER(LayerParams), vp, vp, vp, vp, vp, C.POINTER(LayerGrads),
                                  vp, C.c_size_t],
        "hgnn_layer_fwd_static": [vp, vp, vp, i32, C.POINTER(LayerParams), vp, vp, vp, C.c_size_t],
        "hgnn_layer_fwd_naive": [vp, vp, vp, i32, C.POINTER(LayerParams), vp, vp, vp, C.c_size_t, vp, C.c_size_t,
                                 C.POINTER(i32)],
        "hgnn_layer_fwd_two_step": [vp, vp, vp, i32, C.POINTER(LayerParams), vp, vp, vp, C.c_size_t, vp, C.c_size_t,
                                    vp, C.c_size_t, C.POINTER(i32)],
        "hgnn_layer_bwd": [vp, vp, vp, i32, C.POINTER(LayerParams), vp, vp, vp, vp, vp, C.POINTER(LayerGrads),
                           vp, C.c_size_t],
        "hgnn_layer_bwd_naive": [vp, vp, vp, i32, C.POINTER(LayerParams), vp, vp, vp, vp, vp, C.POINTER(LayerGrads),
                                 vp, C.c_size_t, C.POINTER(i32)],
        "hgnn_layer_launch_count": [vp, vp, i32, C.POINTER(LayerParams), C.POINTER(i32), C.POINTER(i32)],
        "hgnn_softmax_xent": [vp, vp, vp, vp, i64, i32, vp, vp],
        "hgnn_adam_update": [vp, vp, i32, C.POINTER(vp), C.POINTER(vp), C.POINTER(vp), C.POINTER(vp), C.POINTER(vp),
                             C.POINTER(i64), C.POINTER(AdamParams)],
        "hgnn_adam_update_rows": [vp, vp, vp, vp, vp, vp, i32, vp, i64, vp, C.POINTER(AdamParams)],
        "hgnn_probe_select": [vp, i32, i32],
        "hgnn_probe_read": [vp, i32, i32, C.POINTER(C.c_double), C.POINTER(i64)],
    }
    for name, args in sig.items():
        f = getattr(lib, name)
        f.argtypes = args
        f.restype = C.c_int
    lib.hgnn_destroy.argtypes = [vp]; lib.hgnn_destroy.restype = None
    lib.hgnn_graph_release.argtypes = [vp, vp]; lib.hgnn_graph_release.restype = None
    lib.hgnn_sampler_destroy.argtypes = [vp, vp]; lib.hgnn_sampler_destroy.restype = None
    lib.hgnn_last_error.argtypes = []; lib.hgnn_last_error.restype = C.c_char_p
    return lib


lib = _load()

EXPORTS = ["hgnn_create", "hgnn_destroy", "hgnn_last_error", "hgnn_merge_features", "hgnn_merge_features_index_first", "hgnn_select_type_first", "hgnn_build_semantic_csr_device", "hgnn_layer_fwd_gather", "hgnn_layer_bwd_gather", "hgnn_set_edge_types",
           "hgnn_build_semantic_csr", "hgnn_sampler_create", "hgnn_sampler_destroy", "hgnn_sample_and_build",
           "hgnn_graph_ids", "hgnn_graph_minibatch_view", "hgnn_graph_wait_stream",
           "hgnn_set_build_permutation", "hgnn_graph_wait", "hgnn_graph_host_view", "hgnn_graph_release", "hgnn_layer_workspace_bytes",
           "hgnn_layer_fwd", "hgnn_layer_fwd_static", "hgnn_layer_bwd", "hgnn_layer_fwd_naive", "hgnn_layer_bwd_naive", "hgnn_layer_fwd_two_step", "hgnn_layer_launch_count",
           "hgnn_softmax_xent", "hgnn_adam_update", "hgnn_adam_update_rows", "hgnn_probe_select", "hgnn_probe_read"]

KERNEL_IDS = dict(merge=0, transpose_w=1, spmm_fwd=2, gemm_fwd=3, zero_grads=4, relu_bias_bwd=5, gemm_dw=6,
                  gemm_da=7, spmm_bwd=8, xent=9)


def _check(st):
    if st != HGNN_OK:
        raise HgnnError(st, lib.hgnn_last_error().decode())


def _ptr(t) -> Optional[int]:
    """Device pointer of a torch tensor (None -> NULL)."""
    return None if t is None else t.data_ptr()


def _stream_ptr(device=None):
    """HIP stream PyTorch currently uses on `device` (an explicit index keeps torch from probing the
    environment on every call)."""
    import torch
    return torch.cuda.current_stream(device).cuda_stream


class Graph:
    """Handle of one mini-batch's index arrays; keeps the host inputs alive while the build runs."""

    def __init__(self, ctx, handle, keep):
        self.ctx, self.handle, self._keep = ctx, handle, keep

    def wait(self):
        _check(lib.hgnn_graph_wait(self.ctx.handle, self.handle))
        self._keep = None

    def host_view(self, layer):
        v = CsrView()
        _check(lib.hgnn_graph_host_view(self.ctx.handle, self.handle, layer, C.byref(v)))
        R = self.ctx.num_rels
        out = dict(rows=v.rows, edges=v.edges, src_rows=v.src_rows, transpose_edges=v.transpose_edges)
        for k, n in (("rel_row_off", R + 1), ("rel_edge_off", R + 1), ("rowptr", v.rows + 1), ("colidx", v.edges),
                     ("perm", v.edges), ("cptr", v.src_rows + 1), ("crow", v.transpose_edges), ("cperm", v.transpose_edges)):
            if k in ("perm", "cperm") and not getattr(v, k):   # built without the permutations
                out[k] = None
                continue
            out[k] = np.ctypeslib.as_array(getattr(v, k), shape=(n,)).copy() if n > 0 else np.zeros(0, np.int32)
        return out

    def num_edges(self, layer) -> int:
        """Edges of the layer's merged CSR (waits for the build)."""
        v = CsrView()
        _check(lib.hgnn_graph_host_view(self.ctx.handle, self.handle, layer, C.byref(v)))
        return int(v.edges)

    # ---- graphs made by hgnn_sample_and_build ----
    def ids(self, device=False):
        """(n_rows per type, host id arrays per type[, device pointers per type]) of the first layer's source rows;
        blocks until the sampling has finished (with device=True: until the build has)."""
        T = self.ctx.num_types
        n = (C.c_int64 * T)()
        hp, dp = (C.c_void_p * T)(), (C.c_void_p * T)()
        _check(lib.hgnn_graph_ids(self.ctx.handle, self.handle, n, hp, dp if device else None))
        host = [np.ctypeslib.as_array(C.cast(hp[t], C.POINTER(C.c_int64)), shape=(n[t],)).copy() if n[t] else
                np.zeros(0, np.int64) for t in range(T)]
        return (list(n), host, [dp[t] or 0 for t in range(T)]) if device else (list(n), host)

    def minibatch_view(self, layer, arrays=True):
        v = MinibatchView()
        _check(lib.hgnn_graph_minibatch_view(self.ctx.handle, self.handle, layer, C.byref(v)))
        T, E = self.ctx.num_types, v.num_edges
        out = dict(n_src=list(v.n_src[:T]), n_dst=list(v.n_dst[:T]))
        if arrays:
            out["edge_index"] = np.ctypeslib.as_array(v.edge_index, shape=(2, E)).copy() if E else np.zeros((2, 0), np.int64)
            out["edge_id"] = np.ctypeslib.as_array(v.edge_id, shape=(E,)).copy() if E else np.zeros(0, np.int64)
        return out

    def wait_stream(self):
        _check(lib.hgnn_graph_wait_stream(self.ctx.handle, self.handle, _stream_ptr(self.ctx.device)))

    def release(self):
        if self.handle is not None:
            lib.hgnn_graph_release(self.ctx.handle, self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.release()
        except Exception:
            pass


class Sampler:
    def __init__(self, ctx, handle, keep):
        self.ctx, self.handle, self._keep = ctx, handle, keep

    def close(self):
        if self.handle is not None:
            lib.hgnn_sampler_destroy(self.ctx.handle, self.handle)
            self.handle = None


class Layer:
    """Marshalled hgnn_layer_params (+ optional gradient table) for one layer; holds the tensors."""

    def __init__(self, ctx, in_dim, out_dim, relu, w_rel, w_root, bias, dw_rel=None, dw_root=None, dbias=None,
                 input_grad=None, attn=None, dattn=None):
        """attn / dattn: dicts of tensors (w_type [T], a_src [R], a_dst [R], w_sem, b_sem, q_sem) and of their
        fp32 gradient buffers (dw_type, da_src, da_dst, dw_sem, db_sem, dq_sem) for the attention variant."""
        T, R = ctx.num_types, ctx.num_rels
        self.tensors = (w_rel, w_root, bias, dw_rel, dw_root, dbias, attn, dattn)
        nullv, nulli = C.POINTER(C.c_void_p)(), C.POINTER(C.c_int32)()

        def arr(ts, n):
            return (C.c_void_p * n)(*[_ptr(w) for w in ts]) if ts is not None else None

        self._in_dim = (C.c_int32 * T)(*in_dim)
        self._w_rel, self._w_root, self._bias = arr(w_rel, R), arr(w_root, T), arr(bias, T)
        self._input_grad = (C.c_int32 * T)(*[int(x) for x in input_grad]) if input_grad is not None else None
        a = attn or {}
        self._w_type, self._a_src, self._a_dst = arr(a.get("w_type"), T), arr(a.get("a_src"), R), arr(a.get("a_dst"), R)
        self.params = LayerParams(self._in_dim, out_dim, int(relu),
                                  self._w_rel if self._w_rel is not None else nullv,
                                  self._w_root if self._w_root is not None else nullv,
                                  self._bias if self._bias is not None else nullv,
                                  self._input_grad if self._input_grad is not None else nulli,
                                  self._w_type if self._w_type is not None else nullv,
                                  self._a_src if self._a_src is not None else nullv,
                                  self._a_dst if self._a_dst is not None else nullv,
                                  _ptr(a.get("w_sem")), _ptr(a.get("b_sem")), _ptr(a.get("q_sem")))
        self.in_dim, self.out_dim, self.relu = list(in_dim), out_dim, bool(relu)
        self.grads = None
        if dw_rel is not None or dattn is not None:
            d = dattn or {}
            self._dw_rel, self._dw_root, self._dbias = arr(dw_rel, R), arr(dw_root, T), arr(dbias, T)
            self._dw_type, self._da_src, self._da_dst = arr(d.get("dw_type"), T), arr(d.get("da_src"), R), arr(d.get("da_dst"), R)
            self.grads = LayerGrads(self._dw_rel if self._dw_rel is not None else nullv,
                                    self._dw_root if self._dw_root is not None else nullv,
                                    self._dbias if self._dbias is not None else nullv,
                                    self._dw_type if self._dw_type is not None else nullv,
                                    self._da_src if self._da_src is not None else nullv,
                                    self._da_dst if self._da_dst is not None else nullv,
                                    _ptr(d.get("dw_sem")), _ptr(d.get("db_sem")), _ptr(d.get("dq_sem")))


class Context:
    def __init__(self, rel_src: Sequence[int], rel_dst: Sequence[int], num_types: int, dtype: str = "f32",
                 device: int = 0, host_threads: int = 0, concurrent_builds: int = 0, heads: int = 1,
                 attention: bool = False):
        """attention=True: per-relation edge attention with `heads` heads and semantic-attention fusion
        (HGNN_AGG_ATTN / HGNN_FUSE_SEMATTN) instead of mean aggregation with sum fusion."""
        R = len(rel_src)
        self._rs = (C.c_int32 * R)(*rel_src)
        self._rd = (C.c_int32 * R)(*rel_dst)
        sch = Schema(num_types, R, self._rs, self._rd, heads, 1 if attention else 0, 1 if attention else 0,
                     HGNN_BF16 if dtype == "bf16" else HGNN_F32)
        h = C.c_void_p()
        _check(lib.hgnn_create(C.byref(h), C.byref(sch), device, host_threads, concurrent_builds))
        self.handle, self.num_types, self.num_rels, self.dtype = h, num_types, R, dtype
        self.device = device if device >= 0 else None
        self.rel_src, self.rel_dst = list(rel_src), list(rel_dst)

    def close(self):
        if self.handle is not None:
            lib.hgnn_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- hgnn_merge_features ----
    def hgnn_merge_features(self, stores, ids, x_merged, feat_dim=None, n_rows=None):
        """n_rows: rows taken from the front of every id list (default: all of them)."""
        T = self.num_types
        feat_dim = [s.shape[1] for s in stores] if feat_dim is None else feat_dim
        st = (C.c_void_p * T)(*[_ptr(s) for s in stores])
        idp = (C.c_void_p * T)(*[(_ptr(i) if i is not None and i.numel() > 0 else None) for i in ids])
        fd = (C.c_int32 * T)(*feat_dim)
        nr = (C.c_int64 * T)(*([(0 if i is None else i.numel()) for i in ids] if n_rows is None else n_rows))
        row_off = (C.c_int32 * (T + 1))()
        elem_off = (C.c_int64 * (T + 1))()
        _check(lib.hgnn_merge_features(self.handle, _stream_ptr(self.device), st, fd, idp, nr, _ptr(x_merged), row_off, elem_off))
        return np.array(row_off[:], dtype=np.int32), np.array(elem_off[:], dtype=np.int64)

    def hgnn_merge_features_index_first(self, stores, ids, pos, x_interleaved, feat_dim=None):
        """pos: per type a device int32 tensor, the interleaved-buffer row of each of the type's rows."""
        T = self.num_types
        feat_dim = [s.shape[1] for s in stores] if feat_dim is None else feat_dim
        st = (C.c_void_p * T)(*[_ptr(s) for s in stores])
        idp = (C.c_void_p * T)(*[(_ptr(i) if i is not None and i.numel() > 0 else None) for i in ids])
        pp = (C.c_void_p * T)(*[(_ptr(q) if q is not None and q.numel() > 0 else None) for q in pos])
        fd = (C.c_int32 * T)(*feat_dim)
        nr = (C.c_int64 * T)(*[(0 if i is None else i.numel()) for i in ids])
        _check(lib.hgnn_merge_features_index_first(self.handle, _stream_ptr(self.device), st, fd, idp, nr, pp, _ptr(x_interleaved)))

    def hgnn_select_type_first(self, x_interleaved, pos, x_merged, feat_dim):
        T = self.num_types
        pp = (C.c_void_p * T)(*[(_ptr(q) if q is not None and q.numel() > 0 else None) for q in pos])
        fd = (C.c_int32 * T)(*feat_dim)
        nr = (C.c_int64 * T)(*[(0 if q is None else q.numel()) for q in pos])
        row_off = (C.c_int32 * (T + 1))()
        elem_off = (C.c_int64 * (T + 1))()
        _check(lib.hgnn_select_type_first(self.handle, _stream_ptr(self.device), _ptr(x_interleaved), fd, pp, nr, _ptr(x_merged),
                                          row_off, elem_off))
        return np.array(row_off[:], dtype=np.int32), np.array(elem_off[:], dtype=np.int64)

    # ---- parameter update ----
    class AdamList:
        """Marshalled tensor lists of hgnn_adam_update (built once, reused every step)."""

        def __init__(self, params, masters, grads, ms, vs):
            n = len(params)
            self.keep = (params, masters, grads, ms, vs)
            arr = lambda ts: (C.c_void_p * n)(*[_ptr(t) for t in ts])
            self.n = n
            self.param, self.grad, self.m, self.v = arr(params), arr(grads), arr(ms), arr(vs)
            self.master = arr(masters) if masters is not None else None
            self.numel = (C.c_int64 * n)(*[p.numel() for p in params])

    def hgnn_adam_update(self, lst, lr, beta1, beta2, eps, step):
        hp = AdamParams(lr, beta1, beta2, eps, step)
        _check(lib.hgnn_adam_update(self.handle, _stream_ptr(self.device), lst.n, lst.param, lst.master, lst.grad, lst.m, lst.v,
                                    lst.numel, C.byref(hp)))

    def hgnn_adam_update_rows(self, store, master, m, v, ids, grad_rows, lr, beta1, beta2, eps, step):
        """ids: device int64 tensor (or any object with data_ptr() / numel()); grad_rows: [len(ids) x F] rows."""
        hp = AdamParams(lr, beta1, beta2, eps, step)
        _check(lib.hgnn_adam_update_rows(self.handle, _stream_ptr(self.device), _ptr(store), _ptr(master), _ptr(m), _ptr(v),
                                         store.shape[1], _ptr(ids), ids.numel(), _ptr(grad_rows), C.byref(hp)))

    # ---- sampling in the loop ----
    def hgnn_sampler_create(self, num_nodes, in_indptr, in_nbr, edge_off):
        """Host arrays of the whole graph (kept alive by the returned object)."""
        R, T = self.num_rels, self.num_types
        nn = np.ascontiguousarray(num_nodes, dtype=np.int64)
        eo = np.ascontiguousarray(edge_off, dtype=np.int64)
        ptrs = [np.ascontiguousarray(p, dtype=np.int64) for p in in_indptr]
        nbrs = [np.ascontiguousarray(p, dtype=np.int32) for p in in_nbr]
        assert len(nn) == T and len(eo) == R + 1 and len(ptrs) == R and len(nbrs) == R
        pa = (C.c_void_p * R)(*[p.ctypes.data for p in ptrs])
        na = (C.c_void_p * R)(*[p.ctypes.data for p in nbrs])
        hg = HostGraph(nn.ctypes.data_as(C.POINTER(C.c_int64)), pa, na, eo.ctypes.data_as(C.POINTER(C.c_int64)))
        h = C.c_void_p()
        _check(lib.hgnn_sampler_create(self.handle, C.byref(hg), C.byref(h)))
        return Sampler(self, h, (nn, eo, ptrs, nbrs, pa, na))

    def hgnn_sample_and_build(self, sampler, target_type, targets, fanouts, seed, transpose_types=None) -> Graph:
        tg = np.ascontiguousarray(targets, dtype=np.int64)
        L = len(fanouts)
        fo = (C.c_int32 * L)(*[int(f) for f in fanouts])
        keep, tp = [], None
        if transpose_types is not None:
            tp = (C.c_void_p * L)()
            for l, tt in enumerate(transpose_types):
                if tt is not None:
                    a = np.ascontiguousarray(tt, dtype=np.int32)
                    keep.append(a)
                    tp[l] = a.ctypes.data
        h = C.c_void_p()
        _check(lib.hgnn_sample_and_build(self.handle, sampler.handle, int(target_type), tg.ctypes.data, tg.shape[0], L, fo,
                                         C.c_uint64(int(seed) & (2 ** 64 - 1)), tp, C.byref(h)))
        return Graph(self, h, None)

    # ---- hgnn_build_semantic_csr ----
    def hgnn_set_edge_types(self, global_edge_type):
        t = np.ascontiguousarray(global_edge_type, dtype=np.int32)
        _check(lib.hgnn_set_edge_types(self.handle, t.ctypes.data, t.shape[0]))

    def hgnn_set_build_permutation(self, enabled: bool):
        _check(lib.hgnn_set_build_permutation(self.handle, 1 if enabled else 0))

    def hgnn_build_semantic_csr(self, blocks, global_edge_type=None, use_edge_id=False, transpose_types=None, on_device=False) -> Graph:
        """blocks: objects with n_src, n_dst, edge_index (2 x E, int64 or int32), edge_type / edge_id.
        use_edge_id with global_edge_type None: the table registered with hgnn_set_edge_types is used.
        transpose_types: per layer, None or a 0/1 list per vertex type (hgnn_coo_layer.transpose_types)."""
        n = len(blocks)
        arr = (CooLayer * n)()
        keep = []
        for i, b in enumerate(blocks):
            ei = np.ascontiguousarray(b.edge_index)
            assert ei.dtype in (np.int64, np.int32) and ei.ndim == 2 and ei.shape[0] == 2
            ns = np.ascontiguousarray(b.n_src, dtype=np.int64)
            nd = np.ascontiguousarray(b.n_dst, dtype=np.int64)
            keep += [ei, ns, nd]
            arr[i].num_edges = ei.shape[1]
            arr[i].edge_index = ei.ctypes.data
            arr[i].index_is_i64 = 1 if ei.dtype == np.int64 else 0
            if use_edge_id:
                eid = np.ascontiguousarray(b.edge_id, dtype=np.int64)
                keep.append(eid)
                arr[i].edge_type = None
                arr[i].edge_id = eid.ctypes.data
                if global_edge_type is not None:
                    get = np.ascontiguousarray(global_edge_type, dtype=np.int32)
                    keep.append(get)
                    arr[i].global_edge_type = get.ctypes.data
                    arr[i].num_global_edges = get.shape[0]
            else:
                et = np.ascontiguousarray(b.edge_type, dtype=np.int32)
                keep.append(et)
                arr[i].edge_type = et.ctypes.data
            arr[i].n_src = ns.ctypes.data
            arr[i].n_dst = nd.ctypes.data
            tt = None if transpose_types is None else transpose_types[i]
            if tt is not None:
                tta = np.ascontiguousarray(tt, dtype=np.int32)
                keep.append(tta)
                arr[i].transpose_types = tta.ctypes.data
        h = C.c_void_p()
        if on_device:
            ms = C.c_float()
            _check(lib.hgnn_build_semantic_csr_device(self.handle, _stream_ptr(self.device), n, arr, C.byref(h), C.byref(ms)))
            gr = Graph(self, h, keep)
            gr.build_gpu_ms = ms.value
            return gr
        _check(lib.hgnn_build_semantic_csr(self.handle, n, arr, C.byref(h)))
        return Graph(self, h, keep)

    def hgnn_build_semantic_csr_device(self, blocks, global_edge_type=None, use_edge_id=False, transpose_types=None) -> Graph:
        """The same build by device kernels on the current stream; the graph carries build_gpu_ms."""
        return self.hgnn_build_semantic_csr(blocks, global_edge_type, use_edge_id, transpose_types, on_device=True)

    # ---- layer calls ----
    def hgnn_layer_workspace_bytes(self, graph: Graph, layer: int, lp: Layer):
        a, b = C.c_size_t(), C.c_size_t()
        _check(lib.hgnn_layer_workspace_bytes(self.handle, graph.handle, layer, C.byref(lp.params), C.byref(a), C.byref(b)))
        return a.value, b.value

    def hgnn_layer_fwd(self, graph, layer, lp, x_merged, h_out, saved, scratch):
        _check(lib.hgnn_layer_fwd(self.handle, _stream_ptr(self.device), graph.handle, layer, C.byref(lp.params), _ptr(x_merged),
                                  _ptr(h_out), _ptr(saved), saved.numel() * saved.element_size(), _ptr(scratch),
                                  scratch.numel() * scratch.element_size()))

    def hgnn_layer_fwd_gather(self, graph, layer, lp, stores, ids, x_dst, h_out, saved, scratch):
        T = self.num_types
        st = (C.c_void_p * T)(*[_ptr(s) for s in stores])
        idp = (C.c_void_p * T)(*[(_ptr(i) if i is not None and i.numel() > 0 else None) for i in ids])
        _check(lib.hgnn_layer_fwd_gather(self.handle, _stream_ptr(self.device), graph.handle, layer, C.byref(lp.params), st, idp,
                                         _ptr(x_dst), _ptr(h_out), _ptr(saved), saved.numel() * saved.element_size(),
                                         _ptr(scratch), scratch.numel() * scratch.element_size()))

    def hgnn_layer_bwd_gather(self, graph, layer, lp, x_dst, h_out, saved, grad_h, grad_x_merged, scratch):
        _check(lib.hgnn_layer_bwd_gather(self.handle, _stream_ptr(self.device), graph.handle, layer, C.byref(lp.params), _ptr(x_dst),
                                         _ptr(h_out), _ptr(saved), _ptr(grad_h), _ptr(grad_x_merged), C.byref(lp.grads),
                                         _ptr(scratch), scratch.numel() * scratch.element_size()))

    def hgnn_layer_fwd_static(self, graph, layer, lp, x_merged, h_out, saved):
        _check(lib.hgnn_layer_fwd_static(self.handle, _stream_ptr(self.device), graph.handle, layer, C.byref(lp.params),
                                         _ptr(x_merged), _ptr(h_out), _ptr(saved), saved.numel() * saved.element_size()))

    def hgnn_layer_fwd_naive(self, graph, layer, lp, x_merged, h_out, saved, scratch) -> int:
        n = C.c_int32()
        _check(lib.hgnn_layer_fwd_naive(self.handle, _stream_ptr(self.device), graph.handle, layer, C.byref(lp.params),
                                        _ptr(x_merged), _ptr(h_out), _ptr(saved), saved.numel() * saved.element_size(),
                                        _ptr(scratch), scratch.numel() * scratch.element_size(), C.byref(n)))
        return n.value

    def hgnn_layer_fwd_two_step(self, graph, layer, lp, x_merged, h_out, saved, scratch, feature_cat) -> int:
        n = C.c_int32()
        _check(lib.hgnn_layer_fwd_two_step(self.handle, _stream_ptr(self.device), graph.handle, layer, C.byref(lp.params),
                                           _ptr(x_merged), _ptr(h_out), _ptr(saved), saved.numel() * saved.element_size(),
                                           _ptr(scratch), scratch.numel() * scratch.element_size(), _ptr(feature_cat),
                                           feature_cat.numel() * feature_cat.element_size(), C.byref(n)))
        return n.value

    def hgnn_layer_bwd(self, graph, layer, lp, x_merged, h_out, saved, grad_h, grad_x_merged, scratch):
        _check(lib.hgnn_layer_bwd(self.handle, _stream_ptr(self.device), graph.handle, layer, C.byref(lp.params), _ptr(x_merged),
                                  _ptr(h_out), _ptr(saved), _ptr(grad_h), _ptr(grad_x_merged), C.byref(lp.grads),
                                  _ptr(scratch), scratch.numel() * scratch.element_size()))

    def hgnn_layer_bwd_naive(self, graph, layer, lp, x_merged, h_out, saved, grad_h, grad_x_merged, scratch) -> int:
        n = C.c_int32()
        _check(lib.hgnn_layer_bwd_naive(self.handle, _stream_ptr(self.device), graph.handle, layer, C.byref(lp.params),
                                        _ptr(x_merged), _ptr(h_out), _ptr(saved), _ptr(grad_h), _ptr(grad_x_merged),
                                        C.byref(lp.grads), _ptr(scratch), scratch.numel() * scratch.element_size(), C.byref(n)))
        return n.value

    def hgnn_layer_launch_count(self, graph, layer, lp):
        a, b = C.c_int32(), C.c_int32()
        _check(lib.hgnn_layer_launch_count(self.handle, graph.handle, layer, C.byref(lp.params), C.byref(a), C.byref(b)))
        return a.value, b.value

    def hgnn_probe_select(self, kernel: int, layer: int = -1):
        _check(lib.hgnn_probe_select(self.handle, kernel, layer))

    def hgnn_probe_read(self, kernel: int, layer: int = -1):
        ms, n = C.c_double(), C.c_int64()
        _check(lib.hgnn_probe_read(self.handle, kernel, layer, C.byref(ms), C.byref(n)))
        return ms.value, n.value

    def hgnn_softmax_xent(self, logits, labels, loss, grad_logits):
        rows, classes = logits.shape
        _check(lib.hgnn_softmax_xent(self.handle, _stream_ptr(self.device), _ptr(logits), _ptr(labels), rows, classes,
                                     _ptr(loss), _ptr(grad_logits)))
