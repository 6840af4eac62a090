"""Seeded synthetic inputs: R-MAT graphs, features, model parameters, update batches.

This module only draws random inputs and keeps an edge set consistent while a
stream of batches is generated.  It holds none of the method's arithmetic (no
aggregation, no normalisation, no dense update), so both the CPU oracle's tests
and the GPU path's tests may use it without sharing any computation.

The graphs stand in for the power-law real graphs of the paper's evaluation
(Table III, Section V "Datasets and workloads"): R-MAT with (a,b,c,d) =
(0.57, 0.19, 0.19, 0.05), simple and directed, vertex ids shuffled so hubs are
not at consecutive ids.  Batches are hybrid insert/delete workloads sized as a
number of edges, as in the paper's workload description.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

GCN, SAGE_MEAN, GIN, GAT, COMMNET, PINSAGE, AGNN, MONET, GGCN, RGCN, RGAT = 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11
KIND_NAMES = {GCN: "gcn", SAGE_MEAN: "sage_mean", GIN: "gin", GAT: "gat", COMMNET: "commnet", PINSAGE: "pinsage", AGNN: "agnn", MONET: "monet", GGCN: "ggcn",
              RGCN: "rgcn", RGAT: "rgat"}
RELATIONAL = (RGCN, RGAT)           # typed edges: the edge weight array holds the relation id of every edge


@dataclass
class ModelSpec:
    """Shape of an L-layer GNN.  dims = [d_0, ..., d_L] (GAT: heads*head_dim for l>=1; RGAT: head_dim for l>=1)."""
    kind: int
    dims: List[int]
    heads: int = 1
    head_dim: int = 0
    gin_eps: float = 0.1
    leaky_slope: float = 0.2
    weighted: bool = False
    agnn_beta: float = 1.0          # A-GNN: the scalar in front of the cosine (the same at every layer)
    monet_kernels: int = 0          # MoNet: Gaussian kernels per layer (the width of its aggregate)
    agg_only: bool = False          # GCN: keep only the aggregates of hidden layers (storage option of the cache)
    n_relations: int = 0            # RGCN, RGAT: number of edge types (relation ids are 0 .. n_relations-1)
    aggregate_first: bool = False   # GCN, GIN, GraphSAGE, CommNet: never apply a layer's weights before its aggregation

    @property
    def n_layers(self) -> int:
        return len(self.dims) - 1


@dataclass
class Params:
    """Model parameters, fp32, row-major [in][out]."""
    W: List[List[np.ndarray]] = field(default_factory=list)      # W[l] = [Wa] or [Wa, Wb] (GIN)
    b: List[List[Optional[np.ndarray]]] = field(default_factory=list)
    att_src: List[Optional[np.ndarray]] = field(default_factory=list)   # GAT [heads][head_dim]
    att_dst: List[Optional[np.ndarray]] = field(default_factory=list)
    monet_mu: List[Optional[np.ndarray]] = field(default_factory=list)     # MoNet [kernels][d_in] means
    monet_prec: List[Optional[np.ndarray]] = field(default_factory=list)   # MoNet [kernels][d_in] diagonal precisions


@dataclass
class Batch:
    ins_src: np.ndarray
    ins_dst: np.ndarray
    ins_w: Optional[np.ndarray]
    del_src: np.ndarray
    del_dst: np.ndarray
    feat_ids: np.ndarray
    feat_rows: np.ndarray

    @property
    def n_edge_updates(self) -> int:
        return int(self.ins_src.size + self.del_src.size)


def _rmat_draw(rng: np.random.Generator, scale: int, m: int, abcd=(0.57, 0.19, 0.19, 0.05)):
    """m R-MAT (src, dst) draws on a 2^scale grid; quadrant a = (0,0), b = (0,1), c = (1,0), d = (1,1)."""
    a, b, c, _ = abcd
    src = np.zeros(m, dtype=np.int64)
    dst = np.zeros(m, dtype=np.int64)
    for _bit in range(scale):
        r = rng.random(m)
        sbit = r >= (a + b)
        dbit = ((r >= a) & (r < a + b)) | (r >= a + b + c)
        src = (src << 1) | sbit
        dst = (dst << 1) | dbit
    return src, dst


class EdgeSampler:
    """Draws candidate edges either R-MAT distributed (through a fixed id shuffle) or uniform."""

    def __init__(self, n: int, perm: Optional[np.ndarray], uniform: bool):
        self.n = n
        self.scale = max(1, int(np.ceil(np.log2(n))))
        self.perm = perm
        self.uniform = uniform

    def draw(self, rng: np.random.Generator, m: int):
        if self.uniform:
            s = rng.integers(0, self.n, size=m, dtype=np.int64)
            d = rng.integers(0, self.n, size=m, dtype=np.int64)
        else:
            s, d = _rmat_draw(rng, self.scale, m)
            ok = (s < self.n) & (d < self.n)
            s, d = s[ok], d[ok]
            if self.perm is not None:
                s, d = self.perm[s], self.perm[d]
        ok = s != d
        return s[ok], d[ok]


def rmat_graph(n: int, e: int, seed: int = 0, shuffle: bool = True):
    """Exactly e distinct directed edges, no self-loops.  Returns (src int32, dst int32, sampler)."""
    rng = np.random.default_rng([seed, 11])
    perm = rng.permutation(n).astype(np.int64) if shuffle else None
    sampler = EdgeSampler(n, perm, uniform=False)
    keys = np.empty(0, dtype=np.int64)
    while keys.size < e:
        need = e - keys.size
        s, d = sampler.draw(rng, int(need * 1.3) + 1024)
        keys = np.unique(np.concatenate([keys, s * n + d]))
    if keys.size > e:                       # drop a seeded random surplus, keep the rest sorted
        drop = rng.choice(keys.size, size=keys.size - e, replace=False)
        mask = np.ones(keys.size, dtype=bool)
        mask[drop] = False
        keys = keys[mask]
    return (keys // n).astype(np.int32), (keys % n).astype(np.int32), sampler


def features(n: int, d: int, seed: int = 0) -> np.ndarray:
    return np.random.default_rng([seed, 23]).standard_normal((n, d), dtype=np.float32)


def edge_weights(e: int, seed: int = 0) -> np.ndarray:
    return np.random.default_rng([seed, 31]).random(e, dtype=np.float32)


def relation_ids(e: int, n_relations: int, seed: int = 0) -> np.ndarray:
    """One relation id per edge, as the float32 edge weight array carries it; skewed like real typed graphs
    (relation r is about twice as frequent as relation r+1)."""
    p = 0.5 ** np.arange(n_relations)
    return np.random.default_rng([seed, 37]).choice(n_relations, size=e, p=p / p.sum()).astype(np.float32)


def _glorot(rng, fan_in: int, fan_out: int, shape) -> np.ndarray:
    lim = np.sqrt(6.0 / (fan_in + fan_out))
    return rng.uniform(-lim, lim, size=shape).astype(np.float32)


def make_params(spec: ModelSpec, seed: int = 0, bias: bool = False) -> Params:
    """Glorot-uniform matrices; biases zero (or small random when bias=True, for tests)."""
    rng = np.random.default_rng([seed, 47])
    p = Params()
    for l in range(1, spec.n_layers + 1):
        din, dout = spec.dims[l - 1], spec.dims[l]
        kin = 2 * din if spec.kind in (SAGE_MEAN, COMMNET, PINSAGE) else din
        if spec.kind == MONET:
            kin = spec.monet_kernels
        Ws = [_glorot(rng, kin, dout, (kin, dout))]
        if spec.kind == GIN:
            Ws.append(_glorot(rng, dout, dout, (dout, dout)))
        if spec.kind == PINSAGE:
            Ws.append(_glorot(rng, din, din, (din, din)))
        if spec.kind == GGCN:                                   # [W_1; W_2], the gate's two projections
            Ws.append(_glorot(rng, 2 * din, din, (2 * din, din)))
        if spec.kind == RGCN:                                   # W[0] = W_o; W[1] = [W_0 | ... | W_{R-1}], one column block per relation
            Ws.append(_glorot(rng, din, dout, (din, spec.n_relations * dout)))
        if spec.kind == RGAT:                                   # W[0] = [W_0 | ... | W_{R-1}], each d_in x head_dim
            Ws = [_glorot(rng, din, spec.head_dim, (din, spec.n_relations * spec.head_dim))]
        bs: List[Optional[np.ndarray]] = []
        for i, W in enumerate(Ws):
            width = dout if spec.kind == RGAT else W.shape[1]
            with_bias = bias and not (spec.kind == RGCN and i == 1)     # relation messages carry no bias
            bs.append(rng.uniform(-0.1, 0.1, size=width).astype(np.float32) if with_bias else None)
        p.W.append(Ws)
        p.b.append(bs)
        if spec.kind == MONET:
            # means spread like the inputs, precisions small enough that a kernel answers to more than one point
            p.monet_mu.append(rng.standard_normal((spec.monet_kernels, din)).astype(np.float32))
            p.monet_prec.append((rng.uniform(0.2, 2.0, size=(spec.monet_kernels, din)) / din).astype(np.float32))
        else:
            p.monet_mu.append(None)
            p.monet_prec.append(None)
        if spec.kind in (GAT, RGAT):
            groups = spec.heads if spec.kind == GAT else spec.n_relations
            p.att_src.append(_glorot(rng, 2 * spec.head_dim, 1, (groups, spec.head_dim)))
            p.att_dst.append(_glorot(rng, 2 * spec.head_dim, 1, (groups, spec.head_dim)))
        else:
            p.att_src.append(None)
            p.att_dst.append(None)
    return p


class BatchStream:
    """Keeps the current edge set (sorted int64 keys src*n+dst, with weights) and draws
    conflict-free batches: inserts are new edges, deletes are current edges, the two are
    disjoint, feature replacements hit distinct vertices."""

    def __init__(self, n: int, src: np.ndarray, dst: np.ndarray, w: Optional[np.ndarray],
                 sampler: EdgeSampler, d0: int, seed: int = 0, n_relations: int = 0):
        self.n = n
        self.n_relations = n_relations          # > 0: w holds relation ids and inserted edges draw one
        keys = src.astype(np.int64) * n + dst.astype(np.int64)
        order = np.argsort(keys, kind="stable")
        self.keys = keys[order]
        self.w = None if w is None else w[order].astype(np.float32)
        self.sampler = sampler
        self.d0 = d0
        self.seed = seed
        self.k = 0

    def edges(self):
        return ((self.keys // self.n).astype(np.int32), (self.keys % self.n).astype(np.int32),
                None if self.w is None else self.w.copy())

    def next_batch(self, n_ins: int, n_del: int, n_feat: int = 0) -> Batch:
        rng = np.random.default_rng([self.seed, 1000 + self.k])
        self.k += 1
        n_del = min(n_del, self.keys.size)
        del_pos = np.sort(rng.choice(self.keys.size, size=n_del, replace=False)) if n_del else \
            np.empty(0, dtype=np.int64)
        del_keys = self.keys[del_pos]
        ins_keys = np.empty(0, dtype=np.int64)
        # rejection sampling only ends while enough absent pairs are left; refuse what would spin for ever or nearly so
        free = self.n * (self.n - 1) - self.keys.size
        if n_ins > free // 2:
            raise ValueError("cannot draw %d new edges: only %d absent pairs are left" % (n_ins, free))
        while ins_keys.size < n_ins:
            s, d = self.sampler.draw(rng, int((n_ins - ins_keys.size) * 1.5) + 64)
            cand = s * self.n + d
            pos = np.searchsorted(self.keys, cand)
            pos[pos >= self.keys.size] = self.keys.size - 1
            fresh = cand[self.keys[pos] != cand] if self.keys.size else cand
            merged = np.concatenate([ins_keys, fresh])
            _, first = np.unique(merged, return_index=True)
            ins_keys = merged[np.sort(first)]            # keep draw order, drop duplicates
        ins_keys = ins_keys[:n_ins]
        ins_w = rng.random(n_ins, dtype=np.float32) if self.w is not None else None
        if self.w is not None and self.n_relations:
            ins_w = rng.integers(0, self.n_relations, size=n_ins).astype(np.float32)
        feat_ids = rng.choice(self.n, size=n_feat, replace=False).astype(np.int32) if n_feat else \
            np.empty(0, dtype=np.int32)
        feat_rows = rng.standard_normal((n_feat, self.d0), dtype=np.float32)
        # shuffle delete order so the lists are not sorted by key
        dperm = rng.permutation(n_del)
        del_keys = del_keys[dperm]
        # advance the tracked edge set
        keep = np.ones(self.keys.size, dtype=bool)
        keep[del_pos] = False
        keys = self.keys[keep]
        w = None if self.w is None else self.w[keep]
        if n_ins:
            order = np.argsort(ins_keys, kind="stable")
            ik = ins_keys[order]
            at = np.searchsorted(keys, ik)
            keys = np.insert(keys, at, ik)
            if w is not None:
                w = np.insert(w, at, ins_w[order])
        self.keys, self.w = keys, w
        return Batch((ins_keys // self.n).astype(np.int32), (ins_keys % self.n).astype(np.int32), ins_w,
                     (del_keys // self.n).astype(np.int32), (del_keys % self.n).astype(np.int32),
                     feat_ids, feat_rows)


def empty_batch(d0: int, weighted: bool = False) -> Batch:
    z = np.empty(0, dtype=np.int32)
    return Batch(z, z.copy(), np.empty(0, np.float32) if weighted else None, z.copy(), z.copy(),
                 z.copy(), np.empty((0, d0), dtype=np.float32))


def to_csr(n: int, keyrow: np.ndarray, other: np.ndarray, w: Optional[np.ndarray]):
    """Group (keyrow -> other) pairs by keyrow: indptr int64[n+1], indices int32, weights (layout only)."""
    order = np.argsort(keyrow, kind="stable")
    indptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(np.bincount(keyrow, minlength=n), out=indptr[1:])
    return indptr, other[order].astype(np.int32), None if w is None else w[order].astype(np.float32)


@dataclass
class Workload:
    name: str
    spec: ModelSpec
    n: int
    e: int
    n_ins: int
    n_del: int
    n_feat: int
    n_batches: int
    uniform_inserts: bool = False


def config(i: int, scale: float = 1.0) -> Workload:
    """The five benchmark configurations; scale<1 shrinks vertices/edges/batch for quick tests."""
    def s(x, lo=1):
        return max(lo, int(round(x * scale)))
    if i == 0:
        return Workload("cfg1_gcn2_10k", ModelSpec(GCN, [64, 64, 16]), s(10_000, 64), s(100_000, 256),
                        s(100), s(100), 0, 1, uniform_inserts=True)
    if i == 1:
        return Workload("cfg2_sage2_1m", ModelSpec(SAGE_MEAN, [128, 128, 64]), s(1_000_000, 64),
                        s(20_000_000, 256), s(500), s(500), s(100), 100)
    if i == 2:
        return Workload("cfg3_gcn3_4m", ModelSpec(GCN, [128, 256, 256, 64]), s(4_000_000, 64),
                        s(100_000_000, 256), s(7_000), s(3_000), 0, 20)
    if i == 3:
        return Workload("cfg4_gin3_10m", ModelSpec(GIN, [128, 256, 256, 128], weighted=True),
                        s(10_000_000, 64), s(200_000_000, 256), s(5_000), s(5_000), s(1_000), 20)
    if i == 4:
        return Workload("cfg5_gat2_2m", ModelSpec(GAT, [128, 256, 256], heads=4, head_dim=64),
                        s(2_000_000, 64), s(50_000_000, 256), s(25_000), s(25_000), 0, 20)
    raise ValueError(i)


def build(wl: Workload, seed: int = 0):
    """Graph, features, parameters and a batch stream for a workload."""
    src, dst, sampler = rmat_graph(wl.n, wl.e, seed)
    w = edge_weights(wl.e, seed) if wl.spec.weighted else None
    if wl.spec.kind in RELATIONAL:
        w = relation_ids(wl.e, wl.spec.n_relations, seed)
    x = features(wl.n, wl.spec.dims[0], seed)
    params = make_params(wl.spec, seed)
    ins_sampler = EdgeSampler(wl.n, sampler.perm, uniform=wl.uniform_inserts)
    stream = BatchStream(wl.n, src, dst, w, ins_sampler, wl.spec.dims[0], seed,
                         wl.spec.n_relations if wl.spec.kind in RELATIONAL else 0)
    return src, dst, w, x, params, stream
