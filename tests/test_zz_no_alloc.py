"""nrt_graph_export_csc_static, the entry point for callers that cannot allocate: same output as
nrt_graph_export_csc, bit for bit, on two calls in a row (the second on a smaller graph, so whatever the first left
in the library's static device array must not leak into it), after batches have reshaped the lists, and a clear
error beyond the size the static array serves."""
import numpy as np
import pytest

from paper_2603_20622_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _both_exports(nb, torch, graph):
    indptr, indices, weights = nb.nrt_graph_export_csc(graph)
    e = nb.nrt_graph_num_edges(graph)
    ip2 = torch.full((graph.n + 1,), -7, dtype=torch.int64, device="cuda")
    ix2 = torch.full((max(e, 1),), -7, dtype=torch.int32, device="cuda")
    w2 = torch.full((max(e, 1),), -7.0, dtype=torch.float32, device="cuda") if graph.weighted else None
    nb.nrt_graph_export_csc_static(graph, ip2, ix2, w2)
    assert torch.equal(indptr, ip2)
    assert torch.equal(indices, ix2[:e])
    if graph.weighted:
        assert torch.equal(weights, w2[:e])
    return e


def test_static_export_matches_the_workspace_export_twice_in_a_row():
    import torch
    assert torch.cuda.is_available(), "needs the MI355X"
    from paper_2603_20622_amd import binding as nb
    from paper_2603_20622_amd import session as S

    # first call: 300k vertices (293 block sums of the scan), weighted, after a batch that tombstones and appends
    n, e = 300_000, 2_000_000
    src, dst, sampler = wl.rmat_graph(n, e, seed=5)
    w = wl.edge_weights(e, seed=5)
    spec = wl.ModelSpec(wl.GIN, [8, 8, 8], weighted=True)
    ses = S.Session(spec, wl.make_params(spec, 5), n, src, dst, w, wl.features(n, 8, 5))
    stream = wl.BatchStream(n, src, dst, w, sampler, 8, seed=5)
    ses.apply(stream.next_batch(3000, 3000, 10), want_rows=False)
    assert _both_exports(nb, torch, ses.graph) == e
    # second call, right after: a much smaller, unweighted graph (one block sum)
    n2, e2 = 700, 5_000
    src2, dst2, _ = wl.rmat_graph(n2, e2, seed=6)
    spec2 = wl.ModelSpec(wl.GCN, [8, 8])
    ses2 = S.Session(spec2, wl.make_params(spec2, 6), n2, src2, dst2, None, wl.features(n2, 8, 6))
    assert _both_exports(nb, torch, ses2.graph) == e2
    # and the first graph once more
    assert _both_exports(nb, torch, ses.graph) == e


def test_static_export_refuses_graphs_beyond_its_scratch():
    import torch
    from paper_2603_20622_amd import binding as nb

    n = 134_184_960                      # one vertex more than the static array serves
    indptr = torch.zeros(n + 1, dtype=torch.int64, device="cuda")
    g = nb.nrt_graph_create(n, 0, 0, (indptr, None, None), None)
    out = torch.full((n + 1,), -7, dtype=torch.int64, device="cuda")
    idx = torch.zeros(1, dtype=torch.int32, device="cuda")
    with pytest.raises(nb.NrtError) as ei:
        nb.nrt_graph_export_csc_static(g, out, idx, None)
    assert ei.value.status == nb.NRT_ERR_INVALID_ARG and "static scratch" in str(ei.value)
    assert int(out[0]) == -7 and int(out[-1]) == -7          # nothing was written
    ip, ix, _ = nb.nrt_graph_export_csc(g)                   # the workspace variant still serves it
    assert int(ip[-1]) == 0
