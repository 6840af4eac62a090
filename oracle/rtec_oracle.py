"""CPU fp64 oracle for runtime embedding computation on a streaming graph.

TEST INFRASTRUCTURE ONLY.  Only tests, the smoke check and the benchmark's CPU-baseline leg
may import this module; the product path never does, and this module imports nothing from
the product package.  It shares no code with the HIP kernels.

What it computes.  The paper's Theorem 1 states that the incremental layer (Algorithm 1)
returns the same embeddings as a full-neighbour recomputation over the updated
neighbourhoods.  The oracle is therefore that plain definition: apply the batch to the edge
set and the feature matrix, then run the ordinary L-layer message-aggregate-update forward
(Eq. 1) over all vertices and all in-edges of the post-update snapshot, in float64 (fp32
inputs are widened exactly).  No caches, no deltas, no frontier logic in the numeric part.

The affected sets (integer, compared bit-exactly) follow the computation-graph construction
of Algorithm 4 and its description in Section IV: per hop, the affected edges are the updated
edges plus the out-edges of the previous hop's affected vertices, and their destinations are
the next hop's affected vertices.

Readings taken where the paper is silent or garbled (the GPU path takes the same ones):
  * Algorithm 4 as printed empties V_curr and never refills it; the text says the destinations
    form the next layer's affected set, which is what is done here.
  * GCN on a directed graph uses one degree vector d_x = in-degree(x) + 1 (self-loop counted)
    for both ends of Eq. 2.  A vertex whose in-degree changed therefore sends a different
    message along all its out-edges ("updates propagate to all incident edges of a
    neighbor", Section III-C related work), so every destination of an updated edge is a
    source of change at every layer.
  * Every configured model has a self term (GCN/GAT self-loop, SAGE concat-self, GIN
    (1+eps) x_v, CommNet W_1 h_v, PinSAGE concat-self), so a vertex affected at layer l-1 is affected at layer l.
  * Hidden layers are activated (Table II "update" column), the last layer is linear.
  * GraphSAGE-mean: y_v = [x_v || mean_{u in N(v)} x_u] W, the mean of an empty neighbourhood is 0.
  * GIN: t_v = (1+eps) x_v + sum_u w_uv x_u;  y_v = ReLU(t_v Wa + ba) Wb + bb.
  * CommNet: y_v = x_v W_1 + (sum_{u in N(v)} x_u) W_2 as in its Table II row; hidden layers are activated
    like those of the other models (the row prints no activation; without one the layers would collapse
    into a single linear map).
  * PinSAGE: the importance alpha_uv of its Table II row is the edge weight (1 on an unweighted graph), sigma is
    ReLU, Q is square (the message keeps the width of h), and the mean divides by the neighbour count as the
    row's count context says (not by the sum of the weights).
  * A-GNN: a_v = sum_{u in N(v)} w cos(h_v, h_u) h_u exactly as its Table II row prints it (no softmax, no
    self-loop); the cosine with a zero row is 0; a vertex affected at layer l-1 is affected at layer l because
    its own row enters every one of its messages.
  * MoNet: its Table II row prints exp(1/2 (h_u - w_u)^t W_j (h_u - w_u)) with f_nn = 1 and update ReLU(W a_v).
    Read as the Gaussian mixture kernels of MoNet evaluated on the source row: J kernels per layer with mean mu_j
    and a diagonal precision, g_j(h_u) = exp(-1/2 sum_k prec_jk (h_uk - mu_jk)^2) (the sign of the exponent is lost
    in the printed row), the aggregate is the J-vector of summed responses and W maps J to the layer width.  No
    self term in the row; a vertex affected at layer l-1 stays affected at layer l (the structural rule of all
    models here), its row then simply does not change unless an in-neighbour did.
  * G-GCN: the sigma of its message is the logistic function (a gate in (0, 1), as in gated graph ConvNets), applied
    element by element to W_1 h_u + W_2 h_v, both matrices square; the sigma of its update is the ReLU of the
    other models; no self term in the row.
  * GAT: z = x W viewed [heads][head_dim]; e_uv = LeakyReLU(a_dst . z_v + a_src . z_u)
    (destination first, as in Eq. 3); softmax over N(v) U {v}; heads concatenated; ELU on
    hidden layers.
  * RGCN, RGAT (typed edges): every edge <u,v> carries one relation id r(u,v) in 0..R-1, held in the edge weight
    array; an ordered pair of vertices has at most one edge, hence one relation.
  * RGCN: its Table II row: message W_r h_u, count context, a_v = (1/|N(v)|) sum_u W_{r(u,v)} h_u with the count
    taken over all in-neighbours (the row prints one nct_v, not one per relation), update sigma(W_o h_v + a_v);
    a bias is added before sigma; an empty neighbourhood gives a_v = 0.
  * RGAT: its Table II row: per relation r a projection z^r = W_r h, attention parameters a_r and a softmax group of
    its own (the row's context is indexed by the relation of the edge), a_v = sum_u alpha_uv z^{r(u,v)}_u summed over
    all in-edges, update sigma(a_v).  Logit, LeakyReLU, ELU and destination-first order as in the GAT reading; as
    there, every softmax group also holds v itself (under that relation's projection), so no group is empty and a
    vertex affected at layer l-1 stays affected at layer l.
  * A batch is a set applied atomically: inserted edges must be absent, deleted edges present.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional, Sequence

import numpy as np
from scipy.special import expit

GCN, SAGE_MEAN, GIN, GAT, COMMNET, PINSAGE, AGNN, MONET, GGCN, RGCN, RGAT = 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "librtec_oracle.so")
_lib = None


def build_library(force: bool = False) -> str:
    """Compile rtec_oracle.c with gcc (OpenMP)."""
    src = os.path.join(_HERE, "rtec_oracle.c")
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-o", _LIB_PATH, src, "-lm"])
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        build_library()
        _lib = ctypes.CDLL(_LIB_PATH)
        i64, p = ctypes.c_int64, ctypes.c_void_p
        _lib.orc_in_sum.argtypes = [i64, i64, p, p, p, i64, p, p]
        _lib.orc_in_sum.restype = ctypes.c_int
        _lib.orc_gat_attend.argtypes = [i64, i64, p, p, i64, i64, p, p, p, ctypes.c_double, p]
        _lib.orc_gat_attend.restype = ctypes.c_int
        _lib.orc_num_threads.restype = ctypes.c_int
    return _lib


def num_threads() -> int:
    return int(_load().orc_num_threads())


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def in_sum(n: int, src: np.ndarray, dst: np.ndarray, coef: Optional[np.ndarray], payload: np.ndarray) -> np.ndarray:
    """a_v = sum_{<u,v>} coef_uv p_u  (sum aggregation of Eq. 1)."""
    src = np.ascontiguousarray(src, dtype=np.int32)
    dst = np.ascontiguousarray(dst, dtype=np.int32)
    payload = np.ascontiguousarray(payload, dtype=np.float64)
    coef = None if coef is None else np.ascontiguousarray(coef, dtype=np.float64)
    out = np.empty((n, payload.shape[1]), dtype=np.float64)
    rc = _load().orc_in_sum(n, src.size, _ptr(src), _ptr(dst), _ptr(coef), payload.shape[1], _ptr(payload), _ptr(out))
    if rc:
        raise MemoryError("orc_in_sum")
    return out


def gat_attend(n, src, dst, heads, hd, z, a_s, a_d, slope) -> np.ndarray:
    src = np.ascontiguousarray(src, dtype=np.int32)
    dst = np.ascontiguousarray(dst, dtype=np.int32)
    z = np.ascontiguousarray(z, dtype=np.float64)
    a_s = np.ascontiguousarray(a_s, dtype=np.float64)
    a_d = np.ascontiguousarray(a_d, dtype=np.float64)
    out = np.empty_like(z)
    rc = _load().orc_gat_attend(n, src.size, _ptr(src), _ptr(dst), heads, hd, _ptr(z), _ptr(a_s), _ptr(a_d),
                                float(slope), _ptr(out))
    if rc:
        raise MemoryError("orc_gat_attend")
    return out


# ----------------------------------------------------------------------------- batch application
def apply_batch(n: int, src, dst, w, x, batch):
    """Post-update snapshot (src, dst, w, x) of a batch applied as sets (Section IV-B: an inserted
    element adds a message, a deleted one cancels it).  Raises ValueError on a batch that inserts a
    present edge, deletes an absent one, repeats an entry or names a vertex out of range."""
    src = np.asarray(src, dtype=np.int64)
    dst = np.asarray(dst, dtype=np.int64)
    keys = src * n + dst
    ins_s, ins_d = np.asarray(batch.ins_src, np.int64), np.asarray(batch.ins_dst, np.int64)
    del_s, del_d = np.asarray(batch.del_src, np.int64), np.asarray(batch.del_dst, np.int64)
    for a in (ins_s, ins_d, del_s, del_d, np.asarray(batch.feat_ids, np.int64)):
        if a.size and (a.min() < 0 or a.max() >= n):
            raise ValueError("vertex id out of range")
    if np.any(ins_s == ins_d) or np.any(del_s == del_d):
        raise ValueError("self-loop in batch")
    ins_k, del_k = ins_s * n + ins_d, del_s * n + del_d
    if np.unique(ins_k).size != ins_k.size or np.unique(del_k).size != del_k.size:
        raise ValueError("duplicate edge in batch")
    if np.unique(batch.feat_ids).size != len(batch.feat_ids):
        raise ValueError("duplicate feature id in batch")
    if np.isin(ins_k, keys).any():
        raise ValueError("inserted edge already present")
    if not np.isin(del_k, keys).all():
        raise ValueError("deleted edge not present")
    keep = ~np.isin(keys, del_k)
    new_src = np.concatenate([src[keep], ins_s]).astype(np.int32)
    new_dst = np.concatenate([dst[keep], ins_d]).astype(np.int32)
    new_w = None
    if w is not None:
        new_w = np.concatenate([np.asarray(w, np.float32)[keep], np.asarray(batch.ins_w, np.float32)])
    new_x = np.array(x, dtype=np.float32, copy=True)
    if len(batch.feat_ids):
        new_x[np.asarray(batch.feat_ids, np.int64)] = np.asarray(batch.feat_rows, np.float32)
    return new_src, new_dst, new_w, new_x


# ----------------------------------------------------------------------------- full forward
def _act_relu(y):
    return np.maximum(y, 0.0)


def _elu(y):
    return np.where(y > 0, y, np.expm1(np.minimum(y, 0.0)))


def _f64(a):
    return None if a is None else np.asarray(a, dtype=np.float64)


def layer(spec, params, l: int, n: int, src, dst, w, x: np.ndarray) -> np.ndarray:
    """One message-aggregate-update layer (Eq. 1) over the whole graph.  l is 1-based; x = h^{l-1} fp64."""
    L = spec.n_layers
    W = [_f64(m) for m in params.W[l - 1]]
    b = [_f64(v) for v in params.b[l - 1]]
    last = (l == L)
    if spec.kind == GCN:
        # Eq. 2 with d = in-degree + 1 and the self-loop as one more neighbour.
        deg = np.bincount(dst, minlength=n).astype(np.float64) + 1.0
        p = x / np.sqrt(deg)[:, None]
        a = (in_sum(n, src, dst, None, p) + p) / np.sqrt(deg)[:, None]
        y = a @ W[0]
        if b[0] is not None:
            y = y + b[0]
    elif spec.kind == SAGE_MEAN:
        # Table II GraphSAGE row: sum, then divide by the neighbour count; update on [x_v || mean].
        cnt = np.bincount(dst, minlength=n).astype(np.float64)
        s = in_sum(n, src, dst, None, x)
        mean = np.where(cnt[:, None] > 0, s / np.maximum(cnt, 1.0)[:, None], 0.0)
        y = np.concatenate([x, mean], axis=1) @ W[0]
        if b[0] is not None:
            y = y + b[0]
    elif spec.kind == COMMNET:
        # Table II CommNet row: message 1 * h_u, plain sum, update W_1 h_v + W_2 a_v (W[0] holds W_1 above W_2).
        s = in_sum(n, src, dst, None, x)
        y = x @ W[0][: x.shape[1]] + s @ W[0][x.shape[1]:]
        if b[0] is not None:
            y = y + b[0]
    elif spec.kind == PINSAGE:
        # Table II PinSAGE row: message alpha_uv * sigma(Q h_u + q), count context, mean, update on [x_v || a_v].
        m = _act_relu(x @ W[1] + (0.0 if b[1] is None else b[1]))
        cnt = np.bincount(dst, minlength=n).astype(np.float64)
        s = in_sum(n, src, dst, _f64(w), m)
        mean = np.where(cnt[:, None] > 0, s / np.maximum(cnt, 1.0)[:, None], 0.0)
        y = np.concatenate([x, mean], axis=1) @ W[0]
        if b[0] is not None:
            y = y + b[0]
    elif spec.kind == AGNN:
        # Table II A-GNN row: message w * cos(h_v, h_u) * h_u, plain sum, update sigma(W a_v).
        nrm = np.sqrt((x * x).sum(axis=1))
        unit = np.where(nrm[:, None] > 0, x / np.where(nrm > 0, nrm, 1.0)[:, None], 0.0)
        cos = (unit[dst] * unit[src]).sum(axis=1)
        a = in_sum(n, src, dst, float(spec.agnn_beta) * cos, x)
        y = a @ W[0]
        if b[0] is not None:
            y = y + b[0]
    elif spec.kind == MONET:
        # Table II MoNet row: message = the Gaussian kernel responses of the source row, f_nn = 1, plain sum.
        mu, prec = _f64(params.monet_mu[l - 1]), _f64(params.monet_prec[l - 1])
        diff = x[:, None, :] - mu[None, :, :]
        g = np.exp(-0.5 * (prec[None, :, :] * diff * diff).sum(axis=2))
        a = in_sum(n, src, dst, None, g)
        y = a @ W[0]
        if b[0] is not None:
            y = y + b[0]
    elif spec.kind == GGCN:
        # Table II G-GCN row: message sigma(W_1 h_u + W_2 h_v) * h_u element by element, plain sum, update sigma(W a_v).
        d = x.shape[1]
        p1, p2 = x @ W[1][:d], x @ W[1][d:]
        gate = expit(p1[src] + p2[dst])
        a = np.zeros((n, d))
        np.add.at(a, dst, gate * x[src])
        y = a @ W[0]
        if b[0] is not None:
            y = y + b[0]
    elif spec.kind == GIN:
        # Fig. 4: message f(x) = x (times the edge weight), sum aggregation, MLP update.
        s = in_sum(n, src, dst, _f64(w), x)
        t = (1.0 + float(spec.gin_eps)) * x + s
        hmid = t @ W[0]
        if b[0] is not None:
            hmid = hmid + b[0]
        y = _act_relu(hmid) @ W[1]
        if b[1] is not None:
            y = y + b[1]
    elif spec.kind == RGCN:
        # Table II RGCN row: message W_r h_u, sum, divide by the neighbour count, update sigma(W_o h_v + a_v).
        R, dout = spec.n_relations, W[0].shape[1]
        rel = np.asarray(w).astype(np.int64)
        cnt = np.bincount(dst, minlength=n).astype(np.float64)
        s = np.zeros((n, dout))
        for r in range(R):
            sel = rel == r
            s += in_sum(n, src[sel], dst[sel], None, x @ W[1][:, r * dout:(r + 1) * dout])
        a = np.where(cnt[:, None] > 0, s / np.maximum(cnt, 1.0)[:, None], 0.0)
        y = x @ W[0] + a
        if b[0] is not None:
            y = y + b[0]
    elif spec.kind == RGAT:
        # Table II RGAT row: one attention softmax per relation (Eq. 3-4 on the edges of that relation), outputs summed.
        R, hd = spec.n_relations, spec.head_dim
        rel = np.asarray(w).astype(np.int64)
        y = np.zeros((n, hd))
        for r in range(R):
            sel = rel == r
            z = x @ W[0][:, r * hd:(r + 1) * hd]
            a_s = z @ _f64(params.att_src[l - 1])[r]
            a_d = z @ _f64(params.att_dst[l - 1])[r]
            y += gat_attend(n, src[sel], dst[sel], 1, hd, z, a_s[:, None], a_d[:, None], spec.leaky_slope)
        if b[0] is not None:
            y = y + b[0]
        return y if last else _elu(y)
    elif spec.kind == GAT:
        # Eq. 3-4 / Algorithm 2.
        H, hd = spec.heads, spec.head_dim
        z = x @ W[0]
        zv = z.reshape(n, H, hd)
        a_s = np.einsum("nhc,hc->nh", zv, _f64(params.att_src[l - 1]))
        a_d = np.einsum("nhc,hc->nh", zv, _f64(params.att_dst[l - 1]))
        y = gat_attend(n, src, dst, H, hd, z, a_s, a_d, spec.leaky_slope)
        if b[0] is not None:
            y = y + b[0]
        return y if last else _elu(y)
    else:
        raise ValueError("unknown model kind")
    return y if last else _act_relu(y)


def forward(spec, params, n: int, src, dst, w, x) -> List[np.ndarray]:
    """All layer outputs [h^1, ..., h^L] (float64) of the full-neighbour forward on one snapshot."""
    src = np.ascontiguousarray(src, dtype=np.int32)
    dst = np.ascontiguousarray(dst, dtype=np.int32)
    h = np.asarray(x, dtype=np.float64)
    outs = []
    for l in range(1, spec.n_layers + 1):
        h = layer(spec, params, l, n, src, dst, w, h)
        outs.append(h)
    return outs


# ----------------------------------------------------------------------------- affected sets
def affected_sets(spec, n: int, new_src, new_dst, batch) -> List[np.ndarray]:
    """[A_1, ..., A_L]: sorted int32 ids of the vertices whose layer-l embedding may change.

    Algorithm 4: at each hop the affected edges are the updated edges plus the out-edges of the
    vertices affected at the previous hop; the destinations are the next hop's affected vertices.
    Because each model has a self term, an affected vertex stays affected at the next layer.  For GCN
    a destination of an updated edge changes degree, hence its outgoing messages, at every layer.
    """
    new_src = np.asarray(new_src, dtype=np.int64)
    new_dst = np.asarray(new_dst, dtype=np.int64)
    d_dst = np.zeros(n, dtype=bool)
    d_dst[np.asarray(batch.ins_dst, np.int64)] = True
    d_dst[np.asarray(batch.del_dst, np.int64)] = True
    prev = np.zeros(n, dtype=bool)
    prev[np.asarray(batch.feat_ids, np.int64)] = True
    out = []
    for _l in range(1, spec.n_layers + 1):
        sources = prev | d_dst if spec.kind == GCN else prev.copy()
        cur = d_dst | sources
        cur[new_dst[sources[new_src]]] = True
        out.append(np.flatnonzero(cur).astype(np.int32))
        prev = cur
    return out
