"""The five configurations at full size (and the typed-edge models on config 2's graph), in the launch configuration bench.py times: chained batches, then the whole
final-layer cache against one fp64 full-neighbour forward of the oracle on the final snapshot, and the affected
list of the last batch bit-exact for every model.  Config 2 runs its 100 chained batches.  Each case prints its
steps (generation and the oracle forward of the 100M-200M edge graphs take tens of seconds each)."""
import time

import numpy as np
import pytest

from paper_2603_20622_amd import workloads as wl
from tests.test_gpu_parity import TOL, assert_parity, plain_order, rel_err, row_err

pytestmark = pytest.mark.gpu


def run_config(S, oracle, index, batch_sizes):
    run_workload(S, oracle, wl.config(index - 1), batch_sizes)


def run_workload(S, oracle, cfg, batch_sizes):
    t0 = time.time()
    src, dst, w, x, params, stream = wl.build(cfg, seed=0)
    print("[%s] generated in %.0fs" % (cfg.name, time.time() - t0), flush=True)
    frac = cfg.n_ins / max(1, cfg.n_ins + cfg.n_del)
    biggest = max(batch_sizes)
    ses = S.Session(cfg.spec, params, cfg.n, src, dst, w, x, max_batch_edges=2 * biggest + 1024,
                    max_batch_feats=2 * cfg.n_feat + 64)
    print("[%s] caches initialised at %.0fs" % (cfg.name, time.time() - t0), flush=True)
    cur_x = np.array(x, copy=True)
    last = None
    t1 = time.time()
    for k, nb in enumerate(batch_sizes):
        n_ins = int(round(nb * frac))
        b = stream.next_batch(n_ins, nb - n_ins, cfg.n_feat)
        na = ses.apply(b, want_rows=False)
        if len(batch_sizes) <= 5 or k % 25 == 24:
            print("[%s] batch %d of %d edges: %d affected (%.0fs)" % (cfg.name, k + 1, nb, na, time.time() - t1), flush=True)
        if len(b.feat_ids):
            cur_x[b.feat_ids] = b.feat_rows
        last = (b, na)
    b, na = last
    ids = ses.ids[:na].cpu().numpy()                     # the affected list of the last batch, before anything else runs
    fs, fd, fw = stream.edges()
    t2 = time.time()
    ref = oracle.forward(cfg.spec, params, cfg.n, fs, fd, fw, cur_x)[-1]
    print("[%s] oracle forward %.0fs (%d threads)" % (cfg.name, time.time() - t2, oracle.num_threads()), flush=True)
    got = ses.layer(cfg.spec.n_layers).cpu().numpy()
    ses.close()
    del ses
    fresh = None
    if cfg.spec.kind == wl.GIN:
        # the fp32 floor of the un-normalised model at this size: a from-scratch forward of the same library, in the plain
        # operation order, on the final snapshot against the same oracle rows
        ses2 = S.Session(plain_order(cfg.spec), params, cfg.n, fs, fd, fw, cur_x, max_batch_edges=1024, max_batch_feats=64)
        fresh = ses2.layer(cfg.spec.n_layers).cpu().numpy()
        ses2.close()
        del ses2
        print("[%s] from-scratch fp32 forward: element-wise %.3e, row-normalised %.3e"
              % (cfg.name, rel_err(fresh, ref), row_err(fresh, ref)), flush=True)
        assert row_err(fresh, ref) <= TOL
    print("[%s] after %d chained batches: element-wise %.3e, row-normalised %.3e"
          % (cfg.name, len(batch_sizes), rel_err(got, ref), row_err(got, ref)), flush=True)
    assert_parity(cfg.spec.kind, got, ref, cfg.name, fresh)
    sets = oracle.affected_sets(cfg.spec, cfg.n, fs, fd, b)
    assert na == sets[-1].size
    assert np.array_equal(ids, sets[-1])


@pytest.fixture(scope="module")
def S():
    import torch
    assert torch.cuda.is_available()
    from paper_2603_20622_amd import session
    return session


def test_config2_full_size_100_chained_batches(S, oracle):
    run_config(S, oracle, 2, [1000] * 100)


def test_config3_full_size(S, oracle):
    run_config(S, oracle, 3, [1000, 10000, 100000])


def test_config4_full_size(S, oracle):
    run_config(S, oracle, 4, [10000, 10000])


def test_config5_full_size(S, oracle):
    run_config(S, oracle, 5, [50000, 50000])


@pytest.mark.parametrize("index", [2, 5])
def test_full_size_with_aggregate_only_storage(S, oracle, index):
    """Configs 2 (GraphSAGE) and 5 (GAT) at full size on a cache that does not keep its hidden rows (Section IV,
    "recomputation-based embedding storage optimization"): same checks as with the rows kept."""
    import dataclasses
    cfg = wl.config(index - 1, 1.0)
    cfg.spec = dataclasses.replace(cfg.spec, agg_only=True)
    cfg.name += "_agg_only"
    run_workload(S, oracle, cfg, [cfg.n_ins + cfg.n_del] * (20 if index == 2 else 2))


@pytest.mark.parametrize("name", ["rgcn", "rgat"])
def test_typed_edge_models_at_config2_size(S, oracle, name):
    """The typed-edge models of Table II have no configuration of their own: they run on config 2's graph (1 M vertices,
    20 M edges, four relations) and batches, 20 chained batches, with the same checks as the five configurations."""
    if name == "rgcn":
        spec = wl.ModelSpec(wl.RGCN, [128, 128, 64], weighted=True, n_relations=4)
    else:
        spec = wl.ModelSpec(wl.RGAT, [128, 64, 64], head_dim=64, weighted=True, n_relations=4)
    cfg = wl.Workload("cfg2_as_" + name, spec, 1_000_000, 20_000_000, 500, 500, 100, 20)
    run_workload(S, oracle, cfg, [1000] * 20)
