"""Convenience wrapper used by tests, the smoke check and the benchmark: moves numpy inputs to the device
and calls the C ABI through the binding.  No arithmetic of the method happens here."""
from __future__ import annotations

from typing import List, Optional

import numpy as np
import torch

from . import binding as nb
from . import workloads as wl


def _dev(a, dtype=None):
    if a is None:
        return None
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


class DeviceBatch:
    """A batch resident in device memory plus the nrt_batch struct that points at it."""

    def __init__(self, b: wl.Batch):
        self.ins_src, self.ins_dst = _dev(b.ins_src), _dev(b.ins_dst)
        self.ins_w = _dev(b.ins_w)
        self.del_src, self.del_dst = _dev(b.del_src), _dev(b.del_dst)
        self.feat_ids, self.feat_rows = _dev(b.feat_ids), _dev(b.feat_rows)
        self.n_edge_updates = b.n_edge_updates
        self.struct = nb.make_batch(self.ins_src, self.ins_dst, self.ins_w, self.del_src, self.del_dst,
                                    self.feat_ids, self.feat_rows)


class Session:
    def __init__(self, spec: wl.ModelSpec, params: wl.Params, n: int, src, dst, w, x, e_capacity: Optional[int] = None,
                 max_batch_edges: int = 1 << 16, max_batch_feats: int = 1 << 12, give="both"):
        self.spec, self.n = spec, n
        e = int(len(src))
        e_capacity = e_capacity if e_capacity is not None else e + e // 8 + 4 * max_batch_edges + 1024
        csr = csc = None
        if give in ("both", "csr"):
            ip, ix, ww = wl.to_csr(n, np.asarray(src), np.asarray(dst), w)
            csr = (_dev(ip), _dev(ix), _dev(ww))
        if give in ("both", "csc"):
            ip, ix, ww = wl.to_csr(n, np.asarray(dst), np.asarray(src), w)
            csc = (_dev(ip), _dev(ix), _dev(ww))
        self.graph = nb.nrt_graph_create(n, e, e_capacity, csr, csc)
        del csr, csc
        self.dev_params = {
            "W": [[_dev(W) for W in Ws] for Ws in params.W],
            "b": [[_dev(b) for b in bs] for bs in params.b],
            "att_src": [_dev(a) for a in params.att_src],
            "att_dst": [_dev(a) for a in params.att_dst],
            "monet_mu": [_dev(a) for a in getattr(params, "monet_mu", [])],
            "monet_prec": [_dev(a) for a in getattr(params, "monet_prec", [])],
        }
        self.desc = nb.make_desc(spec, self.dev_params)
        xd = _dev(x, torch.float32)
        self.cache = nb.nrt_cache_init(self.graph, self.desc, xd, max_batch_edges, max_batch_feats)
        del xd
        self.ids = torch.empty(n, dtype=torch.int32, device="cuda")
        self.rows = torch.empty((n, spec.dims[-1]), dtype=torch.float32, device="cuda")

    def apply(self, batch, want_rows: bool = True) -> int:
        db = batch if isinstance(batch, DeviceBatch) else DeviceBatch(batch)
        return nb.nrt_apply_batch(self.cache, db.struct, self.ids, self.rows if want_rows else None)

    def layer(self, l: int) -> torch.Tensor:
        return nb.nrt_get_layer(self.cache, l)

    def aggregate(self, l: int) -> torch.Tensor:
        return nb.nrt_get_aggregate(self.cache, l)

    def affected(self, l: int) -> np.ndarray:
        return nb.nrt_get_layer_affected(self.cache, l).cpu().numpy()

    def stats(self):
        return nb.nrt_get_stats(self.cache)

    def mode(self, mode: int):
        nb.nrt_set_mode(self.cache, mode)

    def lazy(self, on: bool):
        nb.nrt_set_lazy(self.cache, on)

    def query(self, ids: np.ndarray):
        """(rows, n_recomputed) for the queried vertex ids."""
        q = _dev(np.asarray(ids, dtype=np.int32))
        rows = torch.empty((len(ids), self.spec.dims[-1]), dtype=torch.float32, device="cuda")
        n = nb.nrt_query(self.cache, q, rows)
        return rows, n

    def apply_query(self, batch, ids: np.ndarray):
        """A batch and a query in one call (on-demand mode): (rows, n_affected, n_updated, n_recomputed)."""
        db = batch if isinstance(batch, DeviceBatch) else DeviceBatch(batch)
        q = _dev(np.asarray(ids, dtype=np.int32))
        rows = torch.empty((len(ids), self.spec.dims[-1]), dtype=torch.float32, device="cuda")
        na, nu, nr = nb.nrt_apply_batch_query(self.cache, db.struct, self.ids, q, rows)
        return rows, na, nu, nr

    def profiling(self, on: bool):
        nb.nrt_set_profiling(self.cache, on)

    def close(self):
        self.cache = None
        self.graph = None
