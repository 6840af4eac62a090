"""Seeded input generators: determinism, simple-graph contract, batches consistent with the tracked edge set."""
import numpy as np

from paper_2603_20622_amd import workloads as wl


def test_rmat_is_simple_deterministic_and_skewed():
    a = wl.rmat_graph(5000, 60000, seed=3)
    b = wl.rmat_graph(5000, 60000, seed=3)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    src, dst = a[0].astype(np.int64), a[1].astype(np.int64)
    assert src.size == 60000 and np.unique(src * 5000 + dst).size == 60000
    assert not np.any(src == dst) and src.min() >= 0 and dst.max() < 5000
    indeg = np.bincount(dst, minlength=5000)
    assert indeg.max() > 20 * indeg.mean()                 # power-law like: a few hubs
    assert (indeg == 0).mean() > 0.2                       # and many vertices nothing points to
    c = wl.rmat_graph(5000, 60000, seed=4)
    assert not np.array_equal(a[0], c[0])


def test_batch_stream_keeps_a_consistent_edge_set():
    n, e = 2000, 20000
    src, dst, sampler = wl.rmat_graph(n, e, seed=1)
    w = wl.edge_weights(e, 1)
    st = wl.BatchStream(n, src, dst, w, sampler, 8, seed=5)
    keys = set((src.astype(np.int64) * n + dst).tolist())
    for _ in range(5):
        b = st.next_batch(300, 200, 20)
        ins = (b.ins_src.astype(np.int64) * n + b.ins_dst).tolist()
        dele = (b.del_src.astype(np.int64) * n + b.del_dst).tolist()
        assert len(set(ins)) == 300 and len(set(dele)) == 200
        assert not (set(ins) & keys) and set(dele) <= keys and not (set(ins) & set(dele))
        assert np.unique(b.feat_ids).size == 20 and b.feat_rows.shape == (20, 8) and b.ins_w.shape == (300,)
        keys = (keys - set(dele)) | set(ins)
        s2, d2, w2 = st.edges()
        assert set((s2.astype(np.int64) * n + d2).tolist()) == keys and w2.size == len(keys)


def test_batch_stream_refuses_inserts_a_nearly_complete_graph_cannot_hold():
    import pytest
    n = 12
    src, dst, sampler = wl.rmat_graph(n, 100, seed=2)       # 100 of the 132 possible edges
    st = wl.BatchStream(n, src, dst, None, sampler, 4, seed=2)
    with pytest.raises(ValueError):
        st.next_batch(40, 0, 0)
    b = st.next_batch(5, 5, 0)                              # a request that fits is still served
    assert b.ins_src.size == 5 and b.del_src.size == 5


def test_configs_have_the_benchmark_shapes():
    shapes = [(wl.GCN, [64, 64, 16], 10_000, 100_000), (wl.SAGE_MEAN, [128, 128, 64], 1_000_000, 20_000_000),
              (wl.GCN, [128, 256, 256, 64], 4_000_000, 100_000_000), (wl.GIN, [128, 256, 256, 128], 10_000_000, 200_000_000),
              (wl.GAT, [128, 256, 256], 2_000_000, 50_000_000)]
    for i, (kind, dims, n, e) in enumerate(shapes):
        c = wl.config(i)
        assert (c.spec.kind, c.spec.dims, c.n, c.e) == (kind, dims, n, e)
    assert wl.config(4).spec.heads == 4 and wl.config(4).spec.head_dim == 64 and wl.config(3).spec.weighted
    assert wl.config(1).n_ins + wl.config(1).n_del == 1000 and wl.config(1).n_feat == 100
