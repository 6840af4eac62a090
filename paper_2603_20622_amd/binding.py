"""ctypes binding of libnrt.so: argument marshalling only.

Every function has the name of the C entry point it calls (include/nrt.h).  PyTorch is used for device
memory (workspaces, inputs, outputs are torch tensors on cuda:0) and for the current stream; no step of
the hot path runs in Python or in torch ops.  If the library is missing the import of this module's
`lib()` fails loudly: there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
import time
from typing import List, Optional

import torch

NRT_MAX_LAYERS = 4
NRT_OK, NRT_ERR_INVALID_ARG, NRT_ERR_BAD_BATCH, NRT_ERR_STATE, NRT_ERR_OOM, NRT_ERR_DEVICE, NRT_ERR_UNSUPPORTED = range(7)
STATUS_NAMES = ["NRT_OK", "NRT_ERR_INVALID_ARG", "NRT_ERR_BAD_BATCH", "NRT_ERR_STATE", "NRT_ERR_OOM",
                "NRT_ERR_DEVICE", "NRT_ERR_UNSUPPORTED"]

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libnrt.so")

c_fp = ctypes.c_void_p


class nrt_model_desc(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("n_layers", ctypes.c_int32),
                ("dims", ctypes.c_int32 * (NRT_MAX_LAYERS + 1)),
                ("heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("gin_eps", ctypes.c_float), ("leaky_slope", ctypes.c_float),
                ("W", (c_fp * 2) * NRT_MAX_LAYERS), ("b", (c_fp * 2) * NRT_MAX_LAYERS),
                ("att_src", c_fp * NRT_MAX_LAYERS), ("att_dst", c_fp * NRT_MAX_LAYERS),
                ("agnn_beta", ctypes.c_float * NRT_MAX_LAYERS), ("monet_kernels", ctypes.c_int32),
                ("monet_mu", c_fp * NRT_MAX_LAYERS), ("monet_prec", c_fp * NRT_MAX_LAYERS), ("agg_only", ctypes.c_int32),
                ("n_relations", ctypes.c_int32), ("aggregate_first", ctypes.c_int32)]


class nrt_batch(ctypes.Structure):
    _fields_ = [("n_ins", ctypes.c_int64), ("ins_src", c_fp), ("ins_dst", c_fp), ("ins_w", c_fp),
                ("n_del", ctypes.c_int64), ("del_src", c_fp), ("del_dst", c_fp),
                ("n_feat", ctypes.c_int64), ("feat_ids", c_fp), ("feat_rows", c_fp)]


class nrt_layer_stats(ctypes.Structure):
    _fields_ = [("n_src", ctypes.c_int64), ("n_affected", ctypes.c_int64), ("n_items", ctypes.c_int64),
                ("n_in_edges", ctypes.c_int64), ("n_pairs", ctypes.c_int64),
                ("ms_expand", ctypes.c_float), ("ms_compact", ctypes.c_float), ("ms_items", ctypes.c_float),
                ("ms_gather", ctypes.c_float), ("ms_combine", ctypes.c_float), ("ms_update", ctypes.c_float)]


class nrt_stats(ctypes.Structure):
    _fields_ = [("n_layers", ctypes.c_int32), ("layer", nrt_layer_stats * NRT_MAX_LAYERS),
                ("ms_ingest", ctypes.c_float), ("ms_total", ctypes.c_float), ("n_launches", ctypes.c_int64)]


class NrtError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__("%s: %s" % (STATUS_NAMES[status] if 0 <= status < len(STATUS_NAMES) else status, message))
        self.status = status


EXPORTS = ["nrt_graph_workspace_bytes", "nrt_graph_create", "nrt_graph_destroy", "nrt_graph_num_edges",
           "nrt_graph_export_csc", "nrt_graph_export_csc_static", "nrt_cache_workspace_bytes", "nrt_cache_init", "nrt_cache_destroy",
           "nrt_apply_batch", "nrt_get_layer", "nrt_get_aggregate", "nrt_get_layer_affected", "nrt_set_profiling",
           "nrt_set_mode", "nrt_set_lazy", "nrt_query", "nrt_apply_batch_query", "nrt_get_stats", "nrt_measure_stream", "nrt_last_error", "nrt_version"]

_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libnrt.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
        L = ctypes.CDLL(LIB_PATH)
        i32, i64, sz = ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
        P = ctypes.POINTER
        L.nrt_graph_workspace_bytes.argtypes = [i64, i64, i32, P(sz)]
        L.nrt_graph_create.argtypes = [i64, i64, i64, i32, c_fp, c_fp, c_fp, c_fp, c_fp, c_fp, c_fp, sz, c_fp, P(c_fp)]
        L.nrt_graph_destroy.argtypes = [c_fp]
        L.nrt_graph_destroy.restype = None
        L.nrt_graph_num_edges.argtypes = [c_fp, P(i64)]
        L.nrt_graph_export_csc.argtypes = [c_fp, c_fp, c_fp, c_fp, i64, c_fp]
        L.nrt_graph_export_csc_static.argtypes = [c_fp, c_fp, c_fp, c_fp, i64, c_fp]
        L.nrt_cache_workspace_bytes.argtypes = [c_fp, P(nrt_model_desc), i64, i64, P(sz)]
        L.nrt_cache_init.argtypes = [c_fp, P(nrt_model_desc), c_fp, i64, i64, c_fp, sz, c_fp, P(c_fp)]
        L.nrt_cache_destroy.argtypes = [c_fp]
        L.nrt_cache_destroy.restype = None
        L.nrt_apply_batch.argtypes = [c_fp, P(nrt_batch), c_fp, c_fp, i64, P(i64), c_fp]
        L.nrt_get_layer.argtypes = [c_fp, i32, P(c_fp), P(i64), P(i64)]
        L.nrt_get_aggregate.argtypes = [c_fp, i32, P(c_fp), P(i64), P(i64)]
        L.nrt_get_layer_affected.argtypes = [c_fp, i32, P(c_fp), P(i64)]
        L.nrt_set_profiling.argtypes = [c_fp, i32]
        L.nrt_set_mode.argtypes = [c_fp, i32]
        L.nrt_set_lazy.argtypes = [c_fp, i32, c_fp]
        L.nrt_query.argtypes = [c_fp, c_fp, i64, c_fp, P(i64), c_fp]
        L.nrt_apply_batch_query.argtypes = [c_fp, P(nrt_batch), c_fp, i64, P(i64), c_fp, i64, c_fp, P(i64), P(i64), c_fp]
        L.nrt_get_stats.argtypes = [c_fp, P(nrt_stats)]
        L.nrt_measure_stream.argtypes = [i32, c_fp, c_fp, i64, i32, c_fp, P(ctypes.c_float)]
        L.nrt_last_error.restype = ctypes.c_char_p
        L.nrt_version.restype = ctypes.c_char_p
        _lib = L
    return _lib


def _check(st: int):
    if st != NRT_OK:
        raise NrtError(st, lib().nrt_last_error().decode())


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous()
    return ctypes.c_void_p(t.data_ptr()) if t.numel() else None


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _workspace(nbytes: int) -> torch.Tensor:
    t = torch.empty(nbytes + 256, dtype=torch.uint8, device="cuda")
    shift = (-t.data_ptr()) % 256
    return t[shift:shift + nbytes]


def _view(ptr: int, shape, dtype, owner) -> torch.Tensor:
    """Tensor view of device memory inside `owner` (a workspace tensor) at address ptr."""
    esize = torch.empty(0, dtype=dtype).element_size()
    off = ptr - owner.data_ptr()
    n = 1
    for d in shape:
        n *= d
    assert 0 <= off and off + n * esize <= owner.numel()
    return owner[off:off + n * esize].view(dtype).view(*shape)


# ---------------------------------------------------------------------------- same-named entry points
def nrt_graph_workspace_bytes(n: int, e_capacity: int, weighted: bool) -> int:
    out = ctypes.c_size_t()
    _check(lib().nrt_graph_workspace_bytes(n, e_capacity, int(weighted), ctypes.byref(out)))
    return out.value


class Graph:
    def __init__(self, handle, ws, n, weighted):
        self.handle, self.ws, self.n, self.weighted = handle, ws, n, weighted

    def __del__(self):
        if getattr(self, "handle", None):
            lib().nrt_graph_destroy(self.handle)
            self.handle = None


def nrt_graph_create(n: int, e: int, e_capacity: int, csr=None, csc=None) -> Graph:
    """csr / csc = (indptr int64, indices int32, weights float32 or None) cuda tensors."""
    weighted = any(t is not None and t[2] is not None for t in (csr, csc))
    ws = _workspace(nrt_graph_workspace_bytes(n, e_capacity, weighted))
    a = csr if csr is not None else (None, None, None)
    b = csc if csc is not None else (None, None, None)
    h = ctypes.c_void_p()
    _check(lib().nrt_graph_create(n, e, e_capacity, int(weighted), _ptr(a[0]), _ptr(a[1]), _ptr(a[2]),
                                  _ptr(b[0]), _ptr(b[1]), _ptr(b[2]), ctypes.c_void_p(ws.data_ptr()), ws.numel(),
                                  _stream(), ctypes.byref(h)))
    return Graph(h, ws, n, weighted)


def nrt_graph_num_edges(g: Graph) -> int:
    out = ctypes.c_int64()
    _check(lib().nrt_graph_num_edges(g.handle, ctypes.byref(out)))
    return out.value


def nrt_graph_export_csc(g: Graph):
    e = nrt_graph_num_edges(g)
    indptr = torch.empty(g.n + 1, dtype=torch.int64, device="cuda")
    indices = torch.empty(max(e, 1), dtype=torch.int32, device="cuda")
    w = torch.empty(max(e, 1), dtype=torch.float32, device="cuda") if g.weighted else None
    _check(lib().nrt_graph_export_csc(g.handle, _ptr(indptr), _ptr(indices), _ptr(w), max(e, 1), _stream()))
    return indptr, indices[:e], None if w is None else w[:e]


def nrt_graph_export_csc_static(g: Graph, indptr: torch.Tensor, indices: torch.Tensor, weights: Optional[torch.Tensor]) -> None:
    """The export into buffers the caller already holds; the call itself allocates nothing."""
    _check(lib().nrt_graph_export_csc_static(g.handle, _ptr(indptr), _ptr(indices), _ptr(weights), indices.numel(), _stream()))


def make_desc(spec, dev_params) -> nrt_model_desc:
    """spec: object with kind, dims, heads, head_dim, gin_eps, leaky_slope; dev_params: cuda tensors."""
    d = nrt_model_desc()
    d.kind = spec.kind
    d.n_layers = len(spec.dims) - 1
    for i, v in enumerate(spec.dims):
        d.dims[i] = v
    d.heads, d.head_dim = spec.heads, spec.head_dim
    d.gin_eps, d.leaky_slope = spec.gin_eps, spec.leaky_slope
    for l in range(d.n_layers):
        d.agnn_beta[l] = float(getattr(spec, "agnn_beta", 1.0))
    d.agg_only = int(bool(getattr(spec, "agg_only", False)))
    d.monet_kernels = int(getattr(spec, "monet_kernels", 0))
    d.n_relations = int(getattr(spec, "n_relations", 0))
    d.aggregate_first = int(bool(getattr(spec, "aggregate_first", False)))
    for l, (mu, prec) in enumerate(zip(dev_params.get("monet_mu", []), dev_params.get("monet_prec", []))):
        if mu is not None:
            d.monet_mu[l], d.monet_prec[l] = mu.data_ptr(), prec.data_ptr()
    for l in range(d.n_layers):
        for j, W in enumerate(dev_params["W"][l]):
            d.W[l][j] = W.data_ptr()
        for j, b in enumerate(dev_params["b"][l]):
            d.b[l][j] = b.data_ptr() if b is not None else None
        if dev_params["att_src"][l] is not None:
            d.att_src[l] = dev_params["att_src"][l].data_ptr()
            d.att_dst[l] = dev_params["att_dst"][l].data_ptr()
    return d


def nrt_cache_workspace_bytes(g: Graph, desc: nrt_model_desc, max_batch_edges: int, max_batch_feats: int) -> int:
    out = ctypes.c_size_t()
    _check(lib().nrt_cache_workspace_bytes(g.handle, ctypes.byref(desc), max_batch_edges, max_batch_feats,
                                           ctypes.byref(out)))
    return out.value


class Cache:
    def __init__(self, handle, ws, graph, desc):
        self.handle, self.ws, self.graph, self.desc = handle, ws, graph, desc
        self.n_layers = desc.n_layers
        self.d_out = desc.dims[desc.n_layers]

    def __del__(self):
        if getattr(self, "handle", None):
            lib().nrt_cache_destroy(self.handle)
            self.handle = None


def nrt_cache_init(g: Graph, desc: nrt_model_desc, features: torch.Tensor, max_batch_edges: int,
                   max_batch_feats: int) -> Cache:
    ws = _workspace(nrt_cache_workspace_bytes(g, desc, max_batch_edges, max_batch_feats))
    h = ctypes.c_void_p()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    _check(lib().nrt_cache_init(g.handle, ctypes.byref(desc), _ptr(features), max_batch_edges, max_batch_feats,
                                ctypes.c_void_p(ws.data_ptr()), ws.numel(), _stream(), ctypes.byref(h)))
    c = Cache(h, ws, g, desc)
    c.init_ms = (time.perf_counter() - t0) * 1e3      # the call synchronises the stream before it returns
    return c


def make_batch(ins_src=None, ins_dst=None, ins_w=None, del_src=None, del_dst=None, feat_ids=None,
               feat_rows=None) -> nrt_batch:
    b = nrt_batch()
    b.n_ins = 0 if ins_src is None else ins_src.numel()
    b.ins_src, b.ins_dst, b.ins_w = _ptr(ins_src), _ptr(ins_dst), _ptr(ins_w)
    b.n_del = 0 if del_src is None else del_src.numel()
    b.del_src, b.del_dst = _ptr(del_src), _ptr(del_dst)
    b.n_feat = 0 if feat_ids is None else feat_ids.numel()
    b.feat_ids, b.feat_rows = _ptr(feat_ids), _ptr(feat_rows)
    return b


def nrt_apply_batch(c: Cache, batch: nrt_batch, affected_ids: torch.Tensor, affected_rows: Optional[torch.Tensor]) -> int:
    n = ctypes.c_int64(0)
    cap = affected_ids.numel()
    _check(lib().nrt_apply_batch(c.handle, ctypes.byref(batch), _ptr(affected_ids), _ptr(affected_rows), cap,
                                 ctypes.byref(n), _stream()))
    return n.value


def nrt_get_layer(c: Cache, layer: int) -> torch.Tensor:
    p, n, ld = ctypes.c_void_p(), ctypes.c_int64(), ctypes.c_int64()
    _check(lib().nrt_get_layer(c.handle, layer, ctypes.byref(p), ctypes.byref(n), ctypes.byref(ld)))
    return _view(p.value, (n.value, ld.value), torch.float32, c.ws)


def nrt_get_aggregate(c: Cache, layer: int) -> torch.Tensor:
    p, n, ld = ctypes.c_void_p(), ctypes.c_int64(), ctypes.c_int64()
    _check(lib().nrt_get_aggregate(c.handle, layer, ctypes.byref(p), ctypes.byref(n), ctypes.byref(ld)))
    return _view(p.value, (n.value, ld.value), torch.float32, c.ws)


def nrt_get_layer_affected(c: Cache, layer: int) -> torch.Tensor:
    p, n = ctypes.c_void_p(), ctypes.c_int64()
    _check(lib().nrt_get_layer_affected(c.handle, layer, ctypes.byref(p), ctypes.byref(n)))
    if n.value == 0:
        return torch.empty(0, dtype=torch.int32, device="cuda")
    return _view(p.value, (n.value,), torch.int32, c.ws)


NRT_MODE_INCREMENTAL, NRT_MODE_RECOMPUTE, NRT_MODE_FULL, NRT_MODE_AUTO = 0, 1, 2, 3


def nrt_set_mode(c: Cache, mode: int) -> None:
    _check(lib().nrt_set_mode(c.handle, int(mode)))


def nrt_set_lazy(c: Cache, on: bool) -> None:
    _check(lib().nrt_set_lazy(c.handle, int(on), _stream()))


def nrt_query(c: Cache, query_ids: torch.Tensor, rows: torch.Tensor) -> int:
    """rows[i] = final-layer embedding of query_ids[i]; returns the number of vertices recomputed for it."""
    n = ctypes.c_int64(0)
    _check(lib().nrt_query(c.handle, _ptr(query_ids), int(query_ids.numel()), _ptr(rows), ctypes.byref(n), _stream()))
    return int(n.value)


def nrt_apply_batch_query(c: Cache, batch: nrt_batch, affected_ids: torch.Tensor, query_ids: torch.Tensor, rows: torch.Tensor):
    """(n_affected, n_updated, n_recomputed); rows[i] = final-layer embedding of query_ids[i] after the batch."""
    na, nu, nr = ctypes.c_int64(0), ctypes.c_int64(0), ctypes.c_int64(0)
    _check(lib().nrt_apply_batch_query(c.handle, ctypes.byref(batch), _ptr(affected_ids), affected_ids.numel(), ctypes.byref(na),
                                       _ptr(query_ids), int(query_ids.numel()), _ptr(rows), ctypes.byref(nu), ctypes.byref(nr),
                                       _stream()))
    return int(na.value), int(nu.value), int(nr.value)


def nrt_set_profiling(c: Cache, on: bool) -> None:
    _check(lib().nrt_set_profiling(c.handle, int(on)))


def nrt_get_stats(c: Cache) -> nrt_stats:
    s = nrt_stats()
    _check(lib().nrt_get_stats(c.handle, ctypes.byref(s)))
    return s


def nrt_measure_stream(kind: int, b: torch.Tensor, a: torch.Tensor, reps: int = 10) -> float:
    """Average milliseconds of one streaming pass over a (kind 0: copy into b, kind 1: read only)."""
    ms = ctypes.c_float(0.0)
    _check(lib().nrt_measure_stream(int(kind), _ptr(b), _ptr(a), int(a.numel()), int(reps), _stream(), ctypes.byref(ms)))
    return float(ms.value)
