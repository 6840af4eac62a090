"""Pins for the CPU oracle: things other than the oracle itself that fix its values.

  * brute force: a per-vertex recursive evaluation of the message-aggregate-update layer (Eq. 1)
    from hand-written adjacency lists, in Python floats, for all eleven models;
  * the dense-matrix closed forms the models reduce to (normalised adjacency products);
  * closed forms on special graphs / parameters (cycle, constant features, zero attention,
    two-term softmax, star hub);
  * the sum identity of the GIN example of Fig. 4 / Section III-C with worked numbers;
  * affected sets against hand-enumerated lists and boolean reachability powers (Algorithm 4);
  * invariants: empty batch, insert-then-delete, value-changed subset of affected.
"""
import math
import os

import numpy as np
import pytest

from paper_2603_20622_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
ALL_KINDS = [wl.GCN, wl.SAGE_MEAN, wl.GIN, wl.GAT, wl.COMMNET, wl.PINSAGE, wl.AGNN, wl.MONET, wl.GGCN, wl.RGCN, wl.RGAT]


# ------------------------------------------------------------------ brute force from adjacency lists
def _lin(vec, W, b=None):
    out = []
    for j in range(len(W[0])):
        s = 0.0 if b is None else float(b[j])
        for i in range(len(vec)):
            s += vec[i] * float(W[i][j])
        out.append(s)
    return out


def brute_embedding(spec, params, in_nbrs, x, v, l):
    """h_v^l by direct recursion on Eq. 1; in_nbrs[v] = list of (u, w_uv)."""
    if l == 0:
        return [float(t) for t in x[v]]
    L = spec.n_layers
    W, b = params.W[l - 1], params.b[l - 1]
    hv = brute_embedding(spec, params, in_nbrs, x, v, l - 1)
    hu = {u: brute_embedding(spec, params, in_nbrs, x, u, l - 1) for u, _ in in_nbrs[v]}
    d = len(hv)
    if spec.kind == wl.GCN:
        dv = len(in_nbrs[v]) + 1
        a = [hv[k] / math.sqrt(dv * dv) for k in range(d)]
        for u, _ in in_nbrs[v]:
            du = len(in_nbrs[u]) + 1
            for k in range(d):
                a[k] += hu[u][k] / math.sqrt(du * dv)
        y = _lin(a, W[0], b[0])
        act = "relu"
    elif spec.kind == wl.SAGE_MEAN:
        m = [0.0] * d
        for u, _ in in_nbrs[v]:
            for k in range(d):
                m[k] += hu[u][k] / len(in_nbrs[v])
        y = _lin(hv + m, W[0], b[0])
        act = "relu"
    elif spec.kind == wl.PINSAGE:
        m = [0.0] * d
        for u, w in in_nbrs[v]:
            mu = [max(q, 0.0) for q in _lin(hu[u], W[1], b[1])]
            for k in range(d):
                m[k] += float(w) * mu[k] / len(in_nbrs[v])
        y = _lin(hv + m, W[0], b[0])
        act = "relu"
    elif spec.kind == wl.GGCN:
        a = [0.0] * d
        for u, _ in in_nbrs[v]:
            g1 = _lin(hu[u], W[1][:d])
            g2 = _lin(hv, W[1][d:])
            for k in range(d):
                a[k] += hu[u][k] / (1.0 + math.exp(-(g1[k] + g2[k])))
        y = _lin(a, W[0], b[0])
        act = "relu"
    elif spec.kind == wl.MONET:
        mu, prec = params.monet_mu[l - 1], params.monet_prec[l - 1]
        a = [0.0] * spec.monet_kernels
        for u, _ in in_nbrs[v]:
            for j in range(spec.monet_kernels):
                q = sum(float(prec[j][k]) * (hu[u][k] - float(mu[j][k])) ** 2 for k in range(d))
                a[j] += math.exp(-0.5 * q)
        y = _lin(a, W[0], b[0])
        act = "relu"
    elif spec.kind == wl.AGNN:
        a = [0.0] * d
        nv = math.sqrt(sum(q * q for q in hv))
        for u, _ in in_nbrs[v]:
            nu = math.sqrt(sum(q * q for q in hu[u]))
            cos = 0.0 if nv == 0 or nu == 0 else sum(hv[k] * hu[u][k] for k in range(d)) / (nv * nu)
            for k in range(d):
                a[k] += spec.agnn_beta * cos * hu[u][k]
        y = _lin(a, W[0], b[0])
        act = "relu"
    elif spec.kind == wl.COMMNET:
        tot = [0.0] * d
        for u, _ in in_nbrs[v]:
            for k in range(d):
                tot[k] += hu[u][k]
        y = _lin(hv + tot, W[0], b[0])
        act = "relu"
    elif spec.kind == wl.RGCN:
        dout = len(W[0][0])
        a = [0.0] * dout
        for u, r in in_nbrs[v]:                                  # the second entry of a pair is the relation id
            Wr = [row[int(r) * dout:(int(r) + 1) * dout] for row in W[1]]
            mu = _lin(hu[u], Wr)
            for k in range(dout):
                a[k] += mu[k] / len(in_nbrs[v])
        own = _lin(hv, W[0], b[0])
        y = [own[k] + a[k] for k in range(dout)]
        act = "relu"
    elif spec.kind == wl.RGAT:
        hd = spec.head_dim
        a_s, a_d = params.att_src[l - 1], params.att_dst[l - 1]
        y = [0.0] * hd
        for r in range(spec.n_relations):
            Wr = [row[r * hd:(r + 1) * hd] for row in W[0]]
            members = [v] + [u for u, rr in in_nbrs[v] if int(rr) == r]
            zs = {u: _lin(hv if u == v else hu[u], Wr) for u in members}
            ad = sum(float(a_d[r][c]) * zs[v][c] for c in range(hd))
            ex = []
            for u in members:
                t = ad + sum(float(a_s[r][c]) * zs[u][c] for c in range(hd))
                ex.append(math.exp(t if t > 0 else spec.leaky_slope * t))
            for c in range(hd):
                y[c] += sum(ex[i] / sum(ex) * zs[u][c] for i, u in enumerate(members))
        if b[0] is not None:
            y = [y[j] + float(b[0][j]) for j in range(hd)]
        act = "elu"
    elif spec.kind == wl.GIN:
        t = [(1.0 + spec.gin_eps) * hv[k] for k in range(d)]
        for u, w in in_nbrs[v]:
            for k in range(d):
                t[k] += float(w) * hu[u][k]
        mid = [max(q, 0.0) for q in _lin(t, W[0], b[0])]
        y = _lin(mid, W[1], b[1])
        act = "relu"
    else:
        H, hd = spec.heads, spec.head_dim
        zs = {u: _lin(hu[u], W[0]) for u in hu}
        zs[v] = _lin(hv, W[0])
        a_s, a_d = params.att_src[l - 1], params.att_dst[l - 1]
        y = []
        for h in range(H):
            sl = slice(h * hd, (h + 1) * hd)
            ad = sum(float(a_d[h][c]) * zs[v][sl][c] for c in range(hd))
            members = [v] + [u for u, _ in in_nbrs[v]]
            logits = []
            for u in members:
                t = ad + sum(float(a_s[h][c]) * zs[u][sl][c] for c in range(hd))
                logits.append(t if t > 0 else spec.leaky_slope * t)
            ex = [math.exp(t) for t in logits]          # raw exp / sum, as Algorithm 2 prints it
            tot = sum(ex)
            for c in range(hd):
                y.append(sum(ex[i] / tot * zs[u][sl][c] for i, u in enumerate(members)))
        if b[0] is not None:
            y = [y[j] + float(b[0][j]) for j in range(len(y))]
        act = "elu"
    if l == L:
        return y
    if act == "relu":
        return [max(q, 0.0) for q in y]
    return [q if q > 0 else math.expm1(q) for q in y]


TINY_EDGES = [(0, 1), (2, 1), (3, 1), (1, 0), (3, 2), (4, 3), (5, 3), (0, 5), (1, 5), (6, 4), (2, 6), (5, 6)]
# vertex 7 is isolated; the graph is asymmetric on purpose (a transposed edge direction changes results)


def _tiny(kind, L, seed, bias=True):
    n = 8
    src = np.array([e[0] for e in TINY_EDGES], dtype=np.int32)
    dst = np.array([e[1] for e in TINY_EDGES], dtype=np.int32)
    rng = np.random.default_rng(seed)
    w = rng.random(src.size, dtype=np.float32) if kind in (wl.GIN, wl.PINSAGE) else None
    if kind in wl.RELATIONAL:
        w = (np.arange(src.size) * 7 % 3).astype(np.float32)        # relation ids 0, 1, 2, all present, mixed per destination
    if kind == wl.GAT:
        dims = [3] + [4] * L
        spec = wl.ModelSpec(kind, dims, heads=2, head_dim=2)
    elif kind == wl.RGAT:
        dims = [3] + [4] * L
        spec = wl.ModelSpec(kind, dims, head_dim=4, weighted=True, n_relations=3)
    elif kind == wl.RGCN:
        dims = [3, 5, 4, 2][: L + 1]
        spec = wl.ModelSpec(kind, dims, weighted=True, n_relations=3)
    else:
        dims = [3, 5, 4, 2][: L + 1]
        spec = wl.ModelSpec(kind, dims, weighted=(kind in (wl.GIN, wl.PINSAGE)), agnn_beta=0.7, monet_kernels=4)
    params = wl.make_params(spec, seed, bias=bias)
    x = rng.standard_normal((n, dims[0])).astype(np.float32)
    return n, src, dst, w, x, spec, params


def _in_lists(n, src, dst, w):
    lists = [[] for _ in range(n)]
    for i in range(len(src)):
        lists[int(dst[i])].append((int(src[i]), 1.0 if w is None else float(w[i])))
    return lists


@pytest.mark.parametrize("kind", ALL_KINDS)
@pytest.mark.parametrize("L", [1, 2, 3])
def test_forward_matches_brute_force(oracle, kind, L):
    n, src, dst, w, x, spec, params = _tiny(kind, L, seed=3 + L)
    outs = oracle.forward(spec, params, n, src, dst, w, x)
    lists = _in_lists(n, src, dst, w)
    for l in range(1, L + 1):
        for v in range(n):
            ref = brute_embedding(spec, params, lists, x, v, l)
            np.testing.assert_allclose(outs[l - 1][v], ref, rtol=1e-11, atol=1e-12)


# ------------------------------------------------------------------ dense-matrix closed forms
def _dense_adj(n, src, dst, w=None):
    A = np.zeros((n, n))                       # A[v, u] = weight of edge u -> v
    for i in range(len(src)):
        A[dst[i], src[i]] = 1.0 if w is None else float(w[i])
    return A


def test_gcn_is_normalised_adjacency_product(oracle):
    n, e = 60, 400
    src, dst, _ = wl.rmat_graph(n, e, seed=5)
    spec = wl.ModelSpec(wl.GCN, [7, 6, 5])
    params = wl.make_params(spec, 1)
    x = wl.features(n, 7, 2)
    A = _dense_adj(n, src, dst) + np.eye(n)
    dinv = 1.0 / np.sqrt(A.sum(axis=1))
    Ahat = dinv[:, None] * A * dinv[None, :]
    h1 = np.maximum(Ahat @ x.astype(np.float64) @ params.W[0][0].astype(np.float64), 0)
    h2 = Ahat @ h1 @ params.W[1][0].astype(np.float64)
    outs = oracle.forward(spec, params, n, src, dst, None, x)
    np.testing.assert_allclose(outs[0], h1, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(outs[1], h2, rtol=1e-11, atol=1e-12)


def test_sage_is_row_normalised_adjacency_product(oracle):
    n, e = 50, 300
    src, dst, _ = wl.rmat_graph(n, e, seed=6)
    spec = wl.ModelSpec(wl.SAGE_MEAN, [4, 6, 3])
    params = wl.make_params(spec, 2)
    x = wl.features(n, 4, 3).astype(np.float64)
    A = _dense_adj(n, src, dst)
    deg = A.sum(axis=1)
    assert (deg == 0).any() and (deg > 0).any()      # both branches of the empty-mean rule are exercised
    P = np.where(deg[:, None] > 0, A / np.maximum(deg, 1)[:, None], 0.0)
    h1 = np.maximum(np.hstack([x, P @ x]) @ params.W[0][0].astype(np.float64), 0)
    h2 = np.hstack([h1, P @ h1]) @ params.W[1][0].astype(np.float64)
    outs = oracle.forward(spec, params, n, src, dst, None, x)
    np.testing.assert_allclose(outs[1], h2, rtol=1e-11, atol=1e-12)


def test_gin_is_weighted_adjacency_product(oracle):
    n, e = 40, 250
    src, dst, _ = wl.rmat_graph(n, e, seed=7)
    w = wl.edge_weights(e, 7)
    spec = wl.ModelSpec(wl.GIN, [5, 6, 4], gin_eps=0.1, weighted=True)
    params = wl.make_params(spec, 3, bias=True)
    x = wl.features(n, 5, 4).astype(np.float64)
    M = _dense_adj(n, src, dst, w) + 1.1 * np.eye(n)
    f = lambda a: a.astype(np.float64)
    h = x
    for l in range(2):
        mid = np.maximum(M @ h @ f(params.W[l][0]) + f(params.b[l][0]), 0)
        h = mid @ f(params.W[l][1]) + f(params.b[l][1])
        if l == 0:
            h = np.maximum(h, 0)
    outs = oracle.forward(spec, params, n, src, dst, w, x)
    np.testing.assert_allclose(outs[1], h, rtol=1e-11, atol=1e-12)


def test_commnet_is_adjacency_product(oracle):
    """Table II CommNet row as matrices: H' = act(H W_1 + A H W_2) with the plain 0/1 adjacency."""
    n, e = 45, 280
    src, dst, _ = wl.rmat_graph(n, e, seed=12)
    spec = wl.ModelSpec(wl.COMMNET, [4, 5, 3])
    params = wl.make_params(spec, 8, bias=True)
    x = wl.features(n, 4, 9).astype(np.float64)
    A = _dense_adj(n, src, dst)
    f = lambda a: a.astype(np.float64)
    W0, W1 = f(params.W[0][0]), f(params.W[1][0])
    h1 = np.maximum(x @ W0[:4] + A @ x @ W0[4:] + f(params.b[0][0]), 0)
    h2 = h1 @ W1[:5] + A @ h1 @ W1[5:] + f(params.b[1][0])
    outs = oracle.forward(spec, params, n, src, dst, None, x)
    np.testing.assert_allclose(outs[0], h1, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(outs[1], h2, rtol=1e-11, atol=1e-12)


def test_commnet_reduces_to_sage_and_gin_on_special_cases(oracle):
    """In-regular graph of degree k: the sum is k times the mean, so CommNet with [W_1; W_2] equals GraphSAGE-mean
    with [W_1; k W_2].  With W_1 = W_2 = W a layer is (x_v + sum_u x_u) W: the first product of a GIN layer with
    eps = 0 and unit edge weights."""
    n, k = 12, 4                                     # a power of two: scaling the fp32 weights by k is exact
    src = np.array([(v + j + 1) % n for v in range(n) for j in range(k)], np.int32)     # v hears v+1..v+k
    dst = np.array([v for v in range(n) for _ in range(k)], np.int32)
    x = wl.features(n, 4, 13)
    com = wl.ModelSpec(wl.COMMNET, [4, 6, 2])
    params = wl.make_params(com, 14, bias=True)
    sage = wl.ModelSpec(wl.SAGE_MEAN, [4, 6, 2])
    scaled = wl.make_params(sage, 14, bias=True)
    for l, d in enumerate([4, 6]):
        scaled.W[l][0] = params.W[l][0].copy()
        scaled.W[l][0][d:] *= k
        scaled.b[l][0] = params.b[l][0].copy()
    got = oracle.forward(com, params, n, src, dst, None, x)
    want = oracle.forward(sage, scaled, n, src, dst, None, x)
    np.testing.assert_allclose(got[1], want[1], rtol=1e-12, atol=1e-13)

    one = wl.ModelSpec(wl.COMMNET, [4, 3])
    p1 = wl.make_params(one, 15)
    p1.W[0][0][4:] = p1.W[0][0][:4]
    out = oracle.forward(one, p1, n, src, dst, None, x)[0]
    t = x.astype(np.float64) + _dense_adj(n, src, dst) @ x.astype(np.float64)
    np.testing.assert_allclose(out, t @ p1.W[0][0][:4].astype(np.float64), rtol=1e-12, atol=1e-13)


def test_pinsage_is_weighted_row_normalised_product(oracle):
    """Table II PinSAGE row as matrices: M = ReLU(H Q + q); A_w = weighted adjacency; a = (A_w M) / count;
    H' = act([H || a] W + b)."""
    n, e = 40, 260
    src, dst, _ = wl.rmat_graph(n, e, seed=16)
    w = wl.edge_weights(e, 16)
    spec = wl.ModelSpec(wl.PINSAGE, [4, 6, 3], weighted=True)
    params = wl.make_params(spec, 17, bias=True)
    x = wl.features(n, 4, 18).astype(np.float64)
    f = lambda a: a.astype(np.float64)
    Aw = _dense_adj(n, src, dst, w)
    cnt = _dense_adj(n, src, dst).sum(axis=1)
    assert (cnt == 0).any()
    h = x
    for l in range(2):
        m = np.maximum(h @ f(params.W[l][1]) + f(params.b[l][1]), 0)
        a = np.where(cnt[:, None] > 0, (Aw @ m) / np.maximum(cnt, 1)[:, None], 0.0)
        h = np.hstack([h, a]) @ f(params.W[l][0]) + f(params.b[l][0])
        if l == 0:
            h = np.maximum(h, 0)
    outs = oracle.forward(spec, params, n, src, dst, w, x)
    np.testing.assert_allclose(outs[1], h, rtol=1e-11, atol=1e-12)


def test_pinsage_with_identity_transform_is_graphsage(oracle):
    """Q = I, q = 0, unit importances, non-negative inputs: the message is h_u itself (ReLU of a non-negative row;
    hidden layers are non-negative after their own ReLU), so the model is GraphSAGE-mean with the same W."""
    n, e = 35, 200
    src, dst, _ = wl.rmat_graph(n, e, seed=19)
    x = np.abs(wl.features(n, 4, 19))
    sage = wl.ModelSpec(wl.SAGE_MEAN, [4, 5, 5, 2])
    ps = wl.make_params(sage, 20, bias=True)
    pin = wl.ModelSpec(wl.PINSAGE, [4, 5, 5, 2])
    pp = wl.make_params(pin, 21, bias=True)
    for l, d in enumerate([4, 5, 5]):
        pp.W[l][0], pp.b[l][0] = ps.W[l][0], ps.b[l][0]
        pp.W[l][1], pp.b[l][1] = np.eye(d, dtype=np.float32), None
    got = oracle.forward(pin, pp, n, src, dst, None, x)
    want = oracle.forward(sage, ps, n, src, dst, None, x)
    for l in range(3):
        np.testing.assert_allclose(got[l], want[l], rtol=1e-12, atol=1e-13)


def test_pinsage_two_edges_by_hand(oracle):
    """Edges 0 -> 2 (weight 0.5) and 1 -> 2 (weight 2), scalar feature, Q = -1, q = 1, W = [3; 4]:
    m_0 = ReLU(1 - 2) = 0, m_1 = ReLU(1 + 3) = 4, a_2 = (0.5*0 + 2*4)/2 = 4, h_2 = 3*5 + 4*4 = 31; h_0 = 3*2."""
    spec = wl.ModelSpec(wl.PINSAGE, [1, 1], weighted=True)
    params = wl.Params(W=[[np.array([[3.0], [4.0]], np.float32), np.array([[-1.0]], np.float32)]],
                       b=[[None, np.array([1.0], np.float32)]], att_src=[None], att_dst=[None])
    x = np.array([[2.0], [-3.0], [5.0]], np.float32)
    out = oracle.forward(spec, params, 3, np.array([0, 1], np.int32), np.array([2, 2], np.int32),
                         np.array([0.5, 2.0], np.float32), x)[0]
    np.testing.assert_allclose(out[:, 0], [6.0, -9.0, 31.0], rtol=1e-14)


def test_agnn_is_cosine_masked_adjacency_product(oracle):
    """Table II A-GNN row as matrices: C = w * (X_hat X_hat^T) masked by the adjacency, a = C X, H' = act(a W + b);
    rows of zeros (they appear after a ReLU) have cosine 0 with everything."""
    n, e = 40, 260
    src, dst, _ = wl.rmat_graph(n, e, seed=22)
    spec = wl.ModelSpec(wl.AGNN, [5, 6, 3], agnn_beta=1.3)
    params = wl.make_params(spec, 23, bias=True)
    x = wl.features(n, 5, 24).astype(np.float64)
    x[3] = 0.0
    f = lambda a: a.astype(np.float64)
    A = _dense_adj(n, src, dst)
    h = x
    for l in range(2):
        nrm = np.linalg.norm(h, axis=1)
        hat = np.divide(h, nrm[:, None], out=np.zeros_like(h), where=nrm[:, None] > 0)
        a = (1.3 * (hat @ hat.T) * A) @ h
        h = a @ f(params.W[l][0]) + f(params.b[l][0])
        if l == 0:
            h = np.maximum(h, 0)
    outs = oracle.forward(spec, params, n, src, dst, None, x.astype(np.float32))
    np.testing.assert_allclose(outs[1], h, rtol=1e-10, atol=1e-12)


def test_agnn_special_directions_by_hand(oracle):
    """Hub 0 with x_0 = (3, 4) hears: 1 with 2*x_0 (cos 1), 2 with (-4, 3) (orthogonal, cos 0), 3 with -x_0 (cos -1),
    4 with (5, 0) (cos 3/5).  w = 2, W = identity:
    a_0 = 2 * [ (6, 8) + 0 - (-3, -4) + 0.6 * (5, 0) ] = 2 * (12, 12) = (24, 24).
    Scaling x_0 by a positive factor leaves a_0 unchanged; vertices without in-neighbours get 0."""
    src = np.array([1, 2, 3, 4], np.int32)
    dst = np.zeros(4, np.int32)
    spec = wl.ModelSpec(wl.AGNN, [2, 2], agnn_beta=2.0)
    params = wl.Params(W=[[np.eye(2, dtype=np.float32)]], b=[[None]], att_src=[None], att_dst=[None])
    x = np.array([[3, 4], [6, 8], [-4, 3], [-3, -4], [5, 0]], np.float32)
    out = oracle.forward(spec, params, 5, src, dst, None, x)[0]
    np.testing.assert_allclose(out[0], [24.0, 24.0], rtol=1e-14)
    np.testing.assert_allclose(out[1:], 0.0, atol=0)
    x2 = x.copy()
    x2[0] *= 8
    np.testing.assert_allclose(oracle.forward(spec, params, 5, src, dst, None, x2)[0][0], [24.0, 24.0], rtol=1e-14)


def test_monet_is_adjacency_product_of_kernel_responses(oracle):
    """Table II MoNet row as matrices: G = exp(-1/2 sum_k prec (h - mu)^2) per vertex and kernel, a = A G, H' = act(a W + b)."""
    n, e = 40, 240
    src, dst, _ = wl.rmat_graph(n, e, seed=25)
    spec = wl.ModelSpec(wl.MONET, [5, 6, 3], monet_kernels=8)
    params = wl.make_params(spec, 26, bias=True)
    x = wl.features(n, 5, 27).astype(np.float64)
    f = lambda a: a.astype(np.float64)
    A = _dense_adj(n, src, dst)
    h = x
    for l in range(2):
        mu, prec = f(params.monet_mu[l]), f(params.monet_prec[l])
        G = np.stack([np.exp(-0.5 * (prec[j] * (h - mu[j]) ** 2).sum(axis=1)) for j in range(8)], axis=1)
        h = A @ G @ f(params.W[l][0]) + f(params.b[l][0])
        if l == 0:
            h = np.maximum(h, 0)
    outs = oracle.forward(spec, params, n, src, dst, None, x.astype(np.float32))
    np.testing.assert_allclose(outs[1], h, rtol=1e-10, atol=1e-12)


def test_monet_special_kernels_by_hand(oracle):
    """Zero precision: every response is 1, the aggregate is the in-degree in every kernel, h_v = indeg(v) * colsum(W).
    One kernel by hand: mu = (1, 2), prec = (2, 0.5); sources (1, 2) -> 1, (2, 2) -> exp(-1), (1, 4) -> exp(-1),
    (3, 0) -> exp(-5);  W = [[10]]."""
    n, e = 30, 150
    src, dst, _ = wl.rmat_graph(n, e, seed=28)
    spec = wl.ModelSpec(wl.MONET, [3, 4], monet_kernels=4)
    params = wl.make_params(spec, 29)
    params.monet_prec[0][:] = 0
    x = wl.features(n, 3, 30)
    out = oracle.forward(spec, params, n, src, dst, None, x)[0]
    indeg = np.bincount(dst, minlength=n).astype(np.float64)
    np.testing.assert_allclose(out, indeg[:, None] * params.W[0][0].astype(np.float64).sum(axis=0)[None, :], rtol=1e-12)

    one = wl.ModelSpec(wl.MONET, [2, 1], monet_kernels=1)
    p1 = wl.Params(W=[[np.array([[10.0]], np.float32)]], b=[[None]], att_src=[None], att_dst=[None],
                   monet_mu=[np.array([[1.0, 2.0]], np.float32)], monet_prec=[np.array([[2.0, 0.5]], np.float32)])
    x1 = np.array([[0, 0], [1, 2], [2, 2], [1, 4], [3, 0]], np.float32)
    s1, d1 = np.array([1, 2, 3, 4], np.int32), np.zeros(4, np.int32)
    got = oracle.forward(one, p1, 5, s1, d1, None, x1)[0]
    np.testing.assert_allclose(got[0, 0], 10 * (1 + 2 * math.exp(-1) + math.exp(-5)), rtol=1e-14)
    np.testing.assert_allclose(got[1:, 0], 0.0, atol=0)


def test_ggcn_is_gated_sum_in_matrix_form(oracle):
    """Table II G-GCN row with dense tensors: gate[v, u, :] = sigmoid(h_u W_1 + h_v W_2) on the edges, a_v = sum_u
    gate[v, u] * h_u, H' = act(a W + b)."""
    n, e = 30, 170
    src, dst, _ = wl.rmat_graph(n, e, seed=31)
    spec = wl.ModelSpec(wl.GGCN, [4, 5, 3])
    params = wl.make_params(spec, 32, bias=True)
    x = wl.features(n, 4, 33).astype(np.float64)
    f = lambda a: a.astype(np.float64)
    A = _dense_adj(n, src, dst)
    h = x
    for l, d in enumerate([4, 5]):
        W12 = f(params.W[l][1])
        gate = 1.0 / (1.0 + np.exp(-((h @ W12[:d])[None, :, :] + (h @ W12[d:])[:, None, :])))     # [v, u, k]
        a = np.einsum("vu,vuk,uk->vk", A, gate, h)
        h = a @ f(params.W[l][0]) + f(params.b[l][0])
        if l == 0:
            h = np.maximum(h, 0)
    outs = oracle.forward(spec, params, n, src, dst, None, x.astype(np.float32))
    np.testing.assert_allclose(outs[1], h, rtol=1e-10, atol=1e-12)


def test_ggcn_zero_gate_weights_halve_commnet_sum(oracle):
    """W_1 = W_2 = 0: every gate is sigmoid(0) = 1/2, so a_v is half the plain neighbour sum.  One edge by hand:
    0 -> 1, x_0 = 2, x_1 = -1, W_1 = 1, W_2 = 3: gate = sigmoid(2 - 3), a_1 = gate * 2, W = 5."""
    n, e = 25, 120
    src, dst, _ = wl.rmat_graph(n, e, seed=34)
    spec = wl.ModelSpec(wl.GGCN, [3, 2])
    params = wl.make_params(spec, 35)
    params.W[0][1][:] = 0
    x = wl.features(n, 3, 36)
    out = oracle.forward(spec, params, n, src, dst, None, x)[0]
    half = 0.5 * (_dense_adj(n, src, dst) @ x.astype(np.float64))
    np.testing.assert_allclose(out, half @ params.W[0][0].astype(np.float64), rtol=1e-12, atol=1e-14)

    one = wl.ModelSpec(wl.GGCN, [1, 1])
    p1 = wl.Params(W=[[np.array([[5.0]], np.float32), np.array([[1.0], [3.0]], np.float32)]], b=[[None, None]],
                   att_src=[None], att_dst=[None])
    got = oracle.forward(one, p1, 2, np.array([0], np.int32), np.array([1], np.int32), None,
                         np.array([[2.0], [-1.0]], np.float32))[0]
    np.testing.assert_allclose(got[:, 0], [0.0, 5 * 2 / (1 + math.exp(1.0))], rtol=1e-14)


def test_rgcn_is_sum_of_relation_adjacency_products(oracle):
    """h = ReLU(X W_o + D^-1 sum_r A_r X W_r + b) with D the in-degree over all relations."""
    n, e, R = 45, 280, 3
    src, dst, _ = wl.rmat_graph(n, e, seed=21)
    rel = wl.relation_ids(e, R, 21)
    assert len(set(rel.tolist())) == R
    spec = wl.ModelSpec(wl.RGCN, [4, 5, 3], weighted=True, n_relations=R)
    params = wl.make_params(spec, 12, bias=True)
    f = lambda a: a.astype(np.float64)
    deg = _dense_adj(n, src, dst).sum(axis=1)
    assert (deg == 0).any()
    h = f(wl.features(n, 4, 12))
    x = h.copy()
    for l in range(2):
        dout = spec.dims[l + 1]
        tot = np.zeros((n, dout))
        for r in range(R):
            Ar = _dense_adj(n, src[rel == r], dst[rel == r])
            tot += Ar @ h @ f(params.W[l][1])[:, r * dout:(r + 1) * dout]
        h = h @ f(params.W[l][0]) + tot / np.maximum(deg, 1)[:, None] + f(params.b[l][0])
        if l == 0:
            h = np.maximum(h, 0)
    outs = oracle.forward(spec, params, n, src, dst, rel, x)
    np.testing.assert_allclose(outs[1], h, rtol=1e-11, atol=1e-12)


def test_rgcn_with_equal_relation_weights_is_graphsage(oracle):
    """When every relation shares one matrix W_r = W_n the relation ids cannot matter and the layer is the
    GraphSAGE-mean layer with the stacked weight [W_o; W_n]."""
    n, e, R = 40, 230, 4
    src, dst, _ = wl.rmat_graph(n, e, seed=22)
    rel = wl.relation_ids(e, R, 22)
    sage = wl.ModelSpec(wl.SAGE_MEAN, [5, 5, 5])
    ps = wl.make_params(sage, 13, bias=True)
    spec = wl.ModelSpec(wl.RGCN, [5, 5, 5], weighted=True, n_relations=R)
    pr = wl.Params(W=[[ps.W[l][0][:5], np.tile(ps.W[l][0][5:], (1, R))] for l in range(2)],
                   b=[[ps.b[l][0], None] for l in range(2)], att_src=[None] * 2, att_dst=[None] * 2,
                   monet_mu=[None] * 2, monet_prec=[None] * 2)
    x = wl.features(n, 5, 13)
    a = oracle.forward(spec, pr, n, src, dst, rel, x)
    b = oracle.forward(sage, ps, n, src, dst, None, x)
    np.testing.assert_allclose(a[1], b[1], rtol=1e-11, atol=1e-12)
    # and a permutation of the relation ids changes nothing then, while it does with distinct matrices
    c = oracle.forward(spec, pr, n, src, dst, (rel + 1) % R, x)
    np.testing.assert_allclose(c[1], a[1], rtol=1e-11, atol=1e-12)
    pd = wl.make_params(spec, 14)
    assert not np.allclose(oracle.forward(spec, pd, n, src, dst, rel, x)[1],
                           oracle.forward(spec, pd, n, src, dst, (rel + 1) % R, x)[1])


def test_rgcn_two_edges_by_hand(oracle):
    """Edges 0 -> 2 (relation 1) and 1 -> 2 (relation 0); width 1; W_o = 3, W_0 = 2, W_1 = -5, bias 0.5.
    h_2 = 3 x_2 + (2 x_1 - 5 x_0) / 2 + 0.5; vertices without in-edges: 3 x + 0.5."""
    spec = wl.ModelSpec(wl.RGCN, [1, 1], weighted=True, n_relations=2)
    params = wl.Params(W=[[np.array([[3.0]], np.float32), np.array([[2.0, -5.0]], np.float32)]],
                       b=[[np.array([0.5], np.float32), None]], att_src=[None], att_dst=[None],
                       monet_mu=[None], monet_prec=[None])
    x = np.array([[0.25], [-1.5], [2.0]], np.float32)
    out = oracle.forward(spec, params, 3, np.array([0, 1], np.int32), np.array([2, 2], np.int32),
                         np.array([1.0, 0.0], np.float32), x)[0]
    np.testing.assert_allclose(out[:, 0], [1.25, -4.0, 6.0 + (2 * -1.5 - 5 * 0.25) / 2 + 0.5], rtol=1e-14)


def test_rgat_with_one_relation_is_single_head_gat(oracle):
    n, e = 30, 150
    src, dst, _ = wl.rmat_graph(n, e, seed=23)
    gat = wl.ModelSpec(wl.GAT, [3, 4, 4], heads=1, head_dim=4)
    pg = wl.make_params(gat, 15, bias=True)
    spec = wl.ModelSpec(wl.RGAT, [3, 4, 4], head_dim=4, weighted=True, n_relations=1)
    x = wl.features(n, 3, 15)
    a = oracle.forward(spec, pg, n, src, dst, np.zeros(e, np.float32), x)
    b = oracle.forward(gat, pg, n, src, dst, None, x)
    np.testing.assert_allclose(a[1], b[1], rtol=1e-11, atol=1e-12)


def test_rgat_zero_attention_is_sum_of_relation_means_with_self(oracle):
    n, e, R = 28, 140, 3
    src, dst, _ = wl.rmat_graph(n, e, seed=24)
    rel = wl.relation_ids(e, R, 24)
    spec = wl.ModelSpec(wl.RGAT, [3, 2], head_dim=2, weighted=True, n_relations=R)
    params = wl.make_params(spec, 16)
    params.att_src[0][:] = 0
    params.att_dst[0][:] = 0
    x = wl.features(n, 3, 16).astype(np.float64)
    expect = np.zeros((n, 2))
    for r in range(R):
        A = _dense_adj(n, src[rel == r], dst[rel == r]) + np.eye(n)
        expect += (A / A.sum(axis=1, keepdims=True)) @ (x @ params.W[0][0].astype(np.float64)[:, 2 * r:2 * r + 2])
    out = oracle.forward(spec, params, n, src, dst, rel, x)[0]
    np.testing.assert_allclose(out, expect, rtol=1e-12, atol=1e-13)


def test_rgat_two_relations_by_hand(oracle):
    """Edges 0 -> 2 (relation 0) and 1 -> 2 (relation 1); width 1; W_0 = 1, W_1 = 2; a_src = (2, 1), a_dst = (-1, 0.5);
    slope 0.2.  Vertex 2 mixes {2, 0} under relation 0 and {2, 1} under relation 1, and the two results add."""
    spec = wl.ModelSpec(wl.RGAT, [1, 1], head_dim=1, weighted=True, n_relations=2, leaky_slope=0.2)
    params = wl.Params(W=[[np.array([[1.0, 2.0]], np.float32)]], b=[[None]],
                       att_src=[np.array([[2.0], [1.0]], np.float32)], att_dst=[np.array([[-1.0], [0.5]], np.float32)],
                       monet_mu=[None], monet_prec=[None])
    x = np.array([[-1.5], [0.75], [0.5]], np.float32)
    out = oracle.forward(spec, params, 3, np.array([0, 1], np.int32), np.array([2, 2], np.int32),
                         np.array([0.0, 1.0], np.float32), x)[0]
    lk = lambda t: t if t > 0 else 0.2 * t
    # relation 0: z = x; logits self L(-0.5 + 1.0), from 0 L(-0.5 - 3.0)
    e_s, e_0 = math.exp(lk(0.5)), math.exp(lk(-3.5))
    r0 = (e_s * 0.5 + e_0 * -1.5) / (e_s + e_0)
    # relation 1: z = 2x; logits self L(0.5*1.0 + 1*1.0), from 1 L(0.5*1.0 + 1*1.5)
    f_s, f_1 = math.exp(lk(1.5)), math.exp(lk(2.0))
    r1 = (f_s * 1.0 + f_1 * 1.5) / (f_s + f_1)
    np.testing.assert_allclose(out[2, 0], r0 + r1, rtol=1e-14)
    np.testing.assert_allclose(out[0, 0], -1.5 + -3.0, rtol=1e-14)     # no in-edges: itself under both relations


def test_commnet_single_edge_by_hand(oracle):
    """Edge 0 -> 1, scalar feature, W_1 = 2, W_2 = -3:  h_0 = 2 x_0,  h_1 = 2 x_1 - 3 x_0."""
    spec = wl.ModelSpec(wl.COMMNET, [1, 1])
    params = wl.Params(W=[[np.array([[2.0], [-3.0]], np.float32)]], b=[[None]], att_src=[None], att_dst=[None])
    x = np.array([[3.0], [5.0]], np.float32)
    out = oracle.forward(spec, params, 2, np.array([0], np.int32), np.array([1], np.int32), None, x)[0]
    np.testing.assert_allclose(out[:, 0], [6.0, 10.0 - 9.0], rtol=1e-14)


# ------------------------------------------------------------------ closed forms on special inputs
def test_gcn_cycle_constant_features(oracle):
    """Directed cycle: every in-degree is 1, d = 2, so a_v = (x + x)/2 = x and h = ReLU(x W)."""
    n = 9
    src = np.arange(n, dtype=np.int32)
    dst = ((np.arange(n) + 1) % n).astype(np.int32)
    spec = wl.ModelSpec(wl.GCN, [3, 4, 2])
    params = wl.make_params(spec, 4)
    row = np.array([0.5, -1.25, 2.0])
    x = np.tile(row, (n, 1)).astype(np.float32)
    outs = oracle.forward(spec, params, n, src, dst, None, x)
    h1 = np.maximum(row @ params.W[0][0].astype(np.float64), 0)
    h2 = h1 @ params.W[1][0].astype(np.float64)
    np.testing.assert_allclose(outs[1], np.tile(h2, (n, 1)), rtol=1e-12, atol=1e-13)


def test_gcn_single_edge_by_hand(oracle):
    """Two vertices, one edge 0 -> 1, scalar feature, W = [[2]]:
    d_0 = 1, d_1 = 2;  a_0 = x0/1;  a_1 = x0/sqrt(1*2) + x1/2."""
    spec = wl.ModelSpec(wl.GCN, [1, 1])
    params = wl.Params(W=[[np.array([[2.0]], np.float32)]], b=[[None]], att_src=[None], att_dst=[None])
    x = np.array([[3.0], [5.0]], np.float32)
    out = oracle.forward(spec, params, 2, np.array([0], np.int32), np.array([1], np.int32), None, x)[0]
    np.testing.assert_allclose(out[:, 0], [6.0, 2 * (3 / math.sqrt(2) + 2.5)], rtol=1e-14)


def test_sage_constant_features(oracle):
    n, e = 30, 120
    src, dst, _ = wl.rmat_graph(n, e, seed=8)
    spec = wl.ModelSpec(wl.SAGE_MEAN, [3, 2])
    params = wl.make_params(spec, 5)
    row = np.array([1.0, -2.0, 0.25])
    x = np.tile(row, (n, 1)).astype(np.float32)
    out = oracle.forward(spec, params, n, src, dst, None, x)[0]
    has = np.bincount(dst, minlength=n) > 0
    W = params.W[0][0].astype(np.float64)
    np.testing.assert_allclose(out[has], np.tile(np.hstack([row, row]) @ W, (has.sum(), 1)), rtol=1e-12)
    np.testing.assert_allclose(out[~has], np.tile(np.hstack([row, 0 * row]) @ W, ((~has).sum(), 1)), rtol=1e-12)


def test_gin_star_hub(oracle):
    """Star: leaves 1..5 -> hub 0.  t_0 = (1+eps) x_0 + sum w_i x_i; identity MLP matrices, positive inputs."""
    k = 5
    src = np.arange(1, k + 1, dtype=np.int32)
    dst = np.zeros(k, dtype=np.int32)
    w = np.array([0.1, 0.2, 0.3, 0.4, 0.5], np.float32)
    spec = wl.ModelSpec(wl.GIN, [2, 2], gin_eps=0.1, weighted=True)
    I = np.eye(2, dtype=np.float32)
    params = wl.Params(W=[[I, I]], b=[[None, None]], att_src=[None], att_dst=[None])
    x = np.arange(1, 2 * (k + 1) + 1, dtype=np.float32).reshape(k + 1, 2)
    out = oracle.forward(spec, params, k + 1, src, dst, w, x)[0]
    expect = 1.1 * x[0].astype(np.float64) + (w.astype(np.float64)[:, None] * x[1:]).sum(axis=0)
    np.testing.assert_allclose(out[0], expect, rtol=1e-14)
    np.testing.assert_allclose(out[3], 1.1 * x[3].astype(np.float64), rtol=1e-14)


def test_gat_zero_attention_is_mean_with_self(oracle):
    n, e = 25, 110
    src, dst, _ = wl.rmat_graph(n, e, seed=9)
    spec = wl.ModelSpec(wl.GAT, [3, 4], heads=2, head_dim=2)
    params = wl.make_params(spec, 6)
    params.att_src[0][:] = 0
    params.att_dst[0][:] = 0
    x = wl.features(n, 3, 6).astype(np.float64)
    z = x @ params.W[0][0].astype(np.float64)
    A = _dense_adj(n, src, dst) + np.eye(n)
    expect = (A / A.sum(axis=1, keepdims=True)) @ z
    out = oracle.forward(spec, params, n, src, dst, None, x)[0]
    np.testing.assert_allclose(out, expect, rtol=1e-12, atol=1e-13)


def test_gat_two_term_softmax_by_hand(oracle):
    """One edge 0 -> 1, one head of width 1, W = [[1]], a_src = 2, a_dst = -1, slope 0.2.
    z = x.  Vertex 1: logits  self: L(-1*x1 + 2*x1),  from 0: L(-1*x1 + 2*x0)."""
    spec = wl.ModelSpec(wl.GAT, [1, 1], heads=1, head_dim=1, leaky_slope=0.2)
    params = wl.Params(W=[[np.array([[1.0]], np.float32)]], b=[[None]],
                       att_src=[np.array([[2.0]], np.float32)], att_dst=[np.array([[-1.0]], np.float32)])
    x = np.array([[-1.5], [0.5]], np.float32)
    out = oracle.forward(spec, params, 2, np.array([0], np.int32), np.array([1], np.int32), None, x)[0]
    e_self = 0.5                      # -0.5 + 1.0 = 0.5 > 0
    e_01 = 0.2 * (-0.5 - 3.0)         # -3.5 < 0 -> slope
    p0 = math.exp(e_01) / (math.exp(e_01) + math.exp(e_self))
    np.testing.assert_allclose(out[1, 0], p0 * -1.5 + (1 - p0) * 0.5, rtol=1e-14)
    np.testing.assert_allclose(out[0, 0], -1.5, rtol=1e-14)          # isolated: attends to itself only


def test_gat_softmax_shift_invariance(oracle):
    """Adding a constant to a_dst . z_v shifts all logits of v on the positive side only; here we
    check the weaker exact property: scaling a_src and a_dst to zero slope region is not needed --
    a uniform shift of every logit of a destination leaves the softmax unchanged, exercised by
    slope = 1 (LeakyReLU becomes the identity, so a_dst only shifts)."""
    n, e = 20, 90
    src, dst, _ = wl.rmat_graph(n, e, seed=10)
    spec = wl.ModelSpec(wl.GAT, [3, 4], heads=2, head_dim=2, leaky_slope=1.0)
    params = wl.make_params(spec, 7)
    x = wl.features(n, 3, 7)
    a = oracle.forward(spec, params, n, src, dst, None, x)[0]
    params.att_dst[0] = params.att_dst[0] * 3.0 + 1.0
    b = oracle.forward(spec, params, n, src, dst, None, x)[0]
    np.testing.assert_allclose(a, b, rtol=1e-10, atol=1e-12)


def test_gin_sum_identity_worked_example(oracle):
    """Fig. 4 / Section III-C: v2 has in-neighbours v1, v3, v4 and v4's embedding changes;
    sum(h1, h3, h4') equals (sum(h1, h3, h4) - h4) + h4'.  Numbers in tests/golden/gin_toy.txt."""
    rows = {}
    with open(os.path.join(GOLDEN, "gin_toy.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            k, *v = line.split()
            rows[k] = np.array([float(t) for t in v])
    src = np.array([1, 3, 4], np.int32)
    dst = np.array([2, 2, 2], np.int32)
    spec = wl.ModelSpec(wl.GIN, [2, 2], gin_eps=0.0)
    I = np.eye(2, dtype=np.float32)
    params = wl.Params(W=[[I, I]], b=[[None, None]], att_src=[None], att_dst=[None])
    x = np.zeros((5, 2), np.float32)
    x[1], x[3], x[4] = rows["h1"], rows["h3"], rows["h4"]
    old = oracle.forward(spec, params, 5, src, dst, None, x)[0][2]
    np.testing.assert_allclose(old, rows["a2_old"], rtol=1e-14)
    x[4] = rows["h4_new"]
    new = oracle.forward(spec, params, 5, src, dst, None, x)[0][2]
    np.testing.assert_allclose(new, rows["a2_new"], rtol=1e-14)
    np.testing.assert_allclose(new, old - rows["h4"] + rows["h4_new"], rtol=1e-14)


# ------------------------------------------------------------------ in_sum primitive alone
def test_in_sum_direction_and_coefficients(oracle):
    src = np.array([0, 0, 2], np.int32)
    dst = np.array([1, 2, 1], np.int32)
    p = np.array([[1.0, 10.0], [2.0, 20.0], [4.0, 40.0]])
    out = oracle.in_sum(3, src, dst, np.array([1.0, 0.5, -2.0]), p)
    np.testing.assert_allclose(out, [[0, 0], [1 - 8, 10 - 80], [0.5, 5.0]])


# ------------------------------------------------------------------ affected sets (Algorithm 4)
def test_affected_sets_hand_enumerated(oracle):
    """Chain 0 -> 1 -> 2 -> 3 -> 4 plus 5 -> 1; insert edge 6 -> 0 (6 has no other edges).
    SAGE (no degree cascade): A_1 = {0} (destination of the updated edge);
    A_2 = {0, 1}; A_3 = {0, 1, 2}.
    GCN: the degree of 0 changes, so 0 is a source already at layer 1: A_1 = {0, 1},
    A_2 = {0, 1, 2}, A_3 = {0, 1, 2, 3}."""
    src = np.array([0, 1, 2, 3, 5, 6], np.int32)         # post-update edges
    dst = np.array([1, 2, 3, 4, 1, 0], np.int32)
    b = wl.empty_batch(2)
    b.ins_src, b.ins_dst = np.array([6], np.int32), np.array([0], np.int32)
    sage = oracle.affected_sets(wl.ModelSpec(wl.SAGE_MEAN, [2, 2, 2, 2]), 7, src, dst, b)
    assert [a.tolist() for a in sage] == [[0], [0, 1], [0, 1, 2]]
    gcn = oracle.affected_sets(wl.ModelSpec(wl.GCN, [2, 2, 2, 2]), 7, src, dst, b)
    assert [a.tolist() for a in gcn] == [[0, 1], [0, 1, 2], [0, 1, 2, 3]]
    # feature replacement at 3 only: A_1 = {3, 4}; GCN adds nothing (no edge update)
    b2 = wl.empty_batch(2)
    b2.feat_ids = np.array([3], np.int32)
    b2.feat_rows = np.zeros((1, 2), np.float32)
    for kind in (wl.GCN, wl.GIN):
        got = oracle.affected_sets(wl.ModelSpec(kind, [2, 2, 2]), 7, src[:5], dst[:5], b2)
        assert [a.tolist() for a in got] == [[3, 4], [3, 4]]


@pytest.mark.parametrize("kind", ALL_KINDS)
def test_affected_sets_match_reachability_powers(oracle, kind):
    n, e = 70, 260
    src, dst, sampler = wl.rmat_graph(n, e, seed=12)
    stream = wl.BatchStream(n, src, dst, None, sampler, 3, seed=1)
    batch = stream.next_batch(4, 4, 2)
    ns, nd, _ = stream.edges()
    spec = wl.ModelSpec(kind, [3, 4, 4, 4], heads=2, head_dim=2, monet_kernels=4)
    got = oracle.affected_sets(spec, n, ns, nd, batch)
    Out = np.zeros((n, n), dtype=np.int64)               # Out[u, v] = 1 for edge u -> v
    Out[ns, nd] = 1
    step = Out + np.eye(n, dtype=np.int64)
    ddst = np.zeros(n, dtype=np.int64)
    ddst[batch.ins_dst] = 1
    ddst[batch.del_dst] = 1
    cur = np.zeros(n, dtype=np.int64)
    cur[batch.feat_ids] = 1
    for l in range(3):
        seeds = np.minimum(cur + ddst, 1) if kind == wl.GCN else cur
        cur = np.minimum(seeds @ step + ddst, 1)
        assert got[l].tolist() == np.flatnonzero(cur).tolist()


# ------------------------------------------------------------------ invariants
@pytest.mark.parametrize("kind", ALL_KINDS)
def test_batch_invariants(oracle, kind):
    n, e = 200, 1500
    src, dst, sampler = wl.rmat_graph(n, e, seed=13)
    weighted = kind in (wl.GIN, wl.PINSAGE) or kind in wl.RELATIONAL
    w = wl.edge_weights(e, 13) if weighted else None
    if kind in wl.RELATIONAL:
        w = wl.relation_ids(e, 3, 13)
    spec = wl.ModelSpec(kind, [6, 8, 4], heads=2, head_dim=4 if kind == wl.GAT else 0, weighted=weighted, monet_kernels=8,
                        n_relations=3)
    if kind == wl.GAT:
        spec = wl.ModelSpec(kind, [6, 8, 8], heads=2, head_dim=4)
    if kind == wl.RGAT:
        spec = wl.ModelSpec(kind, [6, 8, 8], head_dim=8, weighted=True, n_relations=3)
    params = wl.make_params(spec, 9)
    x = wl.features(n, 6, 9)
    base = oracle.forward(spec, params, n, src, dst, w, x)[-1]

    # empty batch: same snapshot, same embeddings, nothing affected
    eb = wl.empty_batch(6, weighted)
    s2, d2, w2, x2 = oracle.apply_batch(n, src, dst, w, x, eb)
    assert np.array_equal(oracle.forward(spec, params, n, s2, d2, w2, x2)[-1], base)
    assert all(a.size == 0 for a in oracle.affected_sets(spec, n, s2, d2, eb))

    # a real batch: rows that changed value are inside the structural affected set
    stream = wl.BatchStream(n, src, dst, w, sampler, 6, seed=2, n_relations=3 if kind in wl.RELATIONAL else 0)
    b = stream.next_batch(10, 10, 3)
    s3, d3, w3, x3 = oracle.apply_batch(n, src, dst, w, x, b)
    after = oracle.forward(spec, params, n, s3, d3, w3, x3)[-1]
    changed = np.flatnonzero(np.any(after != base, axis=1))
    A_L = oracle.affected_sets(spec, n, s3, d3, b)[-1]
    assert np.isin(changed, A_L).all()
    assert changed.size > 0

    # undo: delete what was inserted, insert what was deleted, restore the features
    undo = wl.Batch(b.del_src, b.del_dst, None, b.ins_src, b.ins_dst, b.feat_ids, x[b.feat_ids])
    if weighted:
        keys = src.astype(np.int64) * n + dst
        lookup = {int(k): float(v) for k, v in zip(keys, w)}
        undo.ins_w = np.array([lookup[int(a) * n + int(c)] for a, c in zip(b.del_src, b.del_dst)], np.float32)
    s4, d4, w4, x4 = oracle.apply_batch(n, s3, d3, w3, x3, undo)
    back = oracle.forward(spec, params, n, s4, d4, w4, x4)[-1]
    np.testing.assert_allclose(back, base, rtol=1e-12, atol=1e-13)

    # order of entries inside a batch does not matter (a batch is a set)
    perm = np.random.default_rng(0).permutation(10)
    bp = wl.Batch(b.ins_src[perm], b.ins_dst[perm], None if b.ins_w is None else b.ins_w[perm],
                  b.del_src[::-1], b.del_dst[::-1], b.feat_ids[::-1], b.feat_rows[::-1])
    s5, d5, w5, x5 = oracle.apply_batch(n, src, dst, w, x, bp)
    np.testing.assert_allclose(oracle.forward(spec, params, n, s5, d5, w5, x5)[-1], after, rtol=1e-12, atol=1e-13)


def test_apply_batch_rejects_bad_batches(oracle):
    n = 5
    src = np.array([0, 1], np.int32)
    dst = np.array([1, 2], np.int32)
    x = np.zeros((n, 2), np.float32)

    def mk(ins=(), dele=(), feat=()):
        b = wl.empty_batch(2)
        b.ins_src = np.array([p[0] for p in ins], np.int32)
        b.ins_dst = np.array([p[1] for p in ins], np.int32)
        b.del_src = np.array([p[0] for p in dele], np.int32)
        b.del_dst = np.array([p[1] for p in dele], np.int32)
        b.feat_ids = np.array(feat, np.int32)
        b.feat_rows = np.zeros((len(feat), 2), np.float32)
        return b

    for bad in (mk(ins=[(0, 1)]), mk(dele=[(2, 1)]), mk(ins=[(3, 3)]), mk(ins=[(3, 4), (3, 4)]),
                mk(ins=[(0, 7)]), mk(feat=[1, 1]), mk(dele=[(0, 1), (0, 1)])):
        with pytest.raises(ValueError):
            oracle.apply_batch(n, src, dst, None, x, bad)
    s, d, _, _ = oracle.apply_batch(n, src, dst, None, x, mk(ins=[(1, 0)], dele=[(0, 1)]))
    assert sorted(zip(s.tolist(), d.tolist())) == [(1, 0), (1, 2)]


def test_mean_is_not_associative_but_sum_with_count_is():
    """Section III-C challenge: mean(mean(x, y), z) != mean(x, y, z); keeping the sum and the count
    separately (Table II GraphSAGE row) makes the fold exact."""
    x, y, z = 1.0, 2.0, 6.0
    assert (x + y) / 2 / 2 + z / 2 != (x + y + z) / 3
    s, c = x + y, 2
    assert (s + z) / (c + 1) == (x + y + z) / 3
