#!/usr/bin/env python3
"""Benchmark of the incremental RTEC hot path on one MI355X.

A step = one nrt_apply_batch (validate + ingest, frontier expansion, delta gather/fold, affected-row update
with write-back, all layers) over one synthetic update batch; batches are chained (each step sees the graph
and caches the previous step left).  Inputs (graph, caches, every batch) are resident in HBM before the timed
region.  Two timed passes of K steps each: the first, with the library's per-phase HIP events off, gives the
headline (value, ms_per_step, latency); the second, over the next K chained batches with the events on (they
cost a few percent), gives the per-kernel durations behind `roofline`, `update_gemm` and the phase breakdown.
Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
FP32_MFMA_PEAK_TFLOPS = 157.3
INFINITY_CACHE_BYTES = 256 * 1024 * 1024


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=1, help="index into BASELINE.json configs (default: configs[1])")
    ap.add_argument("--scale", type=float, default=1.0, help="shrink the workload (debugging only)")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--batch-edges", type=int, default=0, help="override the batch size (edges, config 3 sweep)")
    ap.add_argument("--model", choices=["commnet", "pinsage", "agnn", "monet", "ggcn"], default=None,
                    help="run another Table II model on the chosen config's graph, widths and batches (not the headline)")
    ap.add_argument("--agg-only", action="store_true",
                    help="GCN configs: keep only the aggregates of hidden layers (storage option; not the headline)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (caches resident in one MI355X's HBM, no collectives); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2603_20622_amd import workloads as wl
    from paper_2603_20622_amd import session as S

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)

    cfg = wl.config(args.config, args.scale)
    if args.model:
        kind = {"commnet": wl.COMMNET, "pinsage": wl.PINSAGE, "agnn": wl.AGNN, "monet": wl.MONET, "ggcn": wl.GGCN}[args.model]
        cfg.spec = wl.ModelSpec(kind, list(cfg.spec.dims[:1]) + list(cfg.spec.dims[1:]), weighted=kind == wl.PINSAGE,
                                monet_kernels=64)
        cfg.name = cfg.name + "_as_" + args.model
    if args.agg_only:
        cfg.spec.agg_only = True
        cfg.name = cfg.name + "_agg_only"
    if args.batch_edges:
        frac = cfg.n_ins / max(1, cfg.n_ins + cfg.n_del)
        cfg.n_ins = int(round(args.batch_edges * frac))
        cfg.n_del = args.batch_edges - cfg.n_ins
    t0 = time.time()
    src, dst, w, x, params, stream = wl.build(cfg, args.seed)
    k_modes = min(args.steps, 10)                       # steps per non-incremental mode (comparison legs)
    n_total = 2 * args.steps + args.warmup + 4 * k_modes
    batches = [stream.next_batch(cfg.n_ins, cfg.n_del, cfg.n_feat) for _ in range(n_total)]
    final_edges = stream.edges()
    t_gen = time.time() - t0
    print("[bench] %s: generated graph %d/%d and %d batches in %.1fs" % (cfg.name, cfg.n, cfg.e, n_total, t_gen),
          file=sys.stderr, flush=True)

    ses = S.Session(cfg.spec, params, cfg.n, src, dst, w, x,
                    max_batch_edges=max(1024, 2 * (cfg.n_ins + cfg.n_del)), max_batch_feats=max(64, 2 * cfg.n_feat))
    dev_batches = [S.DeviceBatch(b) for b in batches]
    ses.profiling(False)
    torch.cuda.synchronize()
    print("[bench] caches initialised, running %d warmup + 2 x %d timed steps" % (args.warmup, args.steps),
          file=sys.stderr, flush=True)

    for b in dev_batches[:args.warmup]:
        ses.apply(b)
    torch.cuda.synchronize()

    L = cfg.spec.n_layers
    K = args.steps
    dims = cfg.spec.dims

    # ---- pass 1: the headline
    lat = []
    edge_updates = 0
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for b in dev_batches[args.warmup:args.warmup + K]:
        t1 = time.perf_counter()
        ses.apply(b)
        lat.append((time.perf_counter() - t1) * 1e3)
        edge_updates += b.n_edge_updates
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    ms_per_step = elapsed * 1e3 / K
    value = edge_updates / elapsed

    # ---- pass 2: per-phase HIP events on
    ses.profiling(True)
    agg = {"gather_ms": 0.0, "gather_bytes": 0.0, "gather_launches": 0, "update_ms": 0.0, "update_flop": 0.0,
           "ingest_ms": 0.0, "expand_ms": 0.0, "compact_ms": 0.0, "items_ms": 0.0, "combine_ms": 0.0}
    per_layer = [dict(n_src=0, n_aff=0, n_pairs=0, n_in=0, gather_ms=0.0, update_ms=0.0, bytes=0.0) for _ in range(L)]
    t_start2 = time.perf_counter()
    for b in dev_batches[args.warmup + K:args.warmup + 2 * K]:
        ses.apply(b)
        st = ses.stats()
        agg["ingest_ms"] += st.ms_ingest
        for l in range(L):
            ls = st.layer[l]
            d_in = dims[l]
            # algorithmic bytes of the gather launch: per delta message its in-list id and slot-map entry (8 B);
            # the delta rows: every changed source row once (4*d) while the delta buffer fits the 256 MB Infinity
            # Cache, else one row per delta message; every affected aggregate row read and written (8*d)
            d_agg = dims[l + 1] if cfg.spec.kind == wl.GAT else (cfg.spec.monet_kernels if cfg.spec.kind == wl.MONET else d_in)
            row_fetches = ls.n_src if ls.n_src * 4.0 * d_agg <= INFINITY_CACHE_BYTES else ls.n_pairs
            gbytes = ls.n_pairs * 8.0 + row_fetches * 4.0 * d_agg + ls.n_affected * 8.0 * d_agg if ls.n_src else 0.0
            kin = (2 if cfg.spec.kind in (wl.SAGE_MEAN, wl.COMMNET, wl.PINSAGE) else 1) * d_in
            if cfg.spec.kind == wl.MONET:
                kin = d_agg
            flop = 2.0 * ls.n_affected * kin * dims[l + 1]
            if cfg.spec.kind == wl.GIN:
                flop += 2.0 * ls.n_affected * dims[l + 1] * dims[l + 1]
            if cfg.spec.kind == wl.PINSAGE:                      # message transform of the changed rows (timed under "items")
                flop += 2.0 * ls.n_src * d_in * d_in
            upd_ms = ls.ms_update
            if cfg.spec.kind == wl.GAT:
                flop = 2.0 * ls.n_src * d_in * dims[l + 1]       # z = x W on the rows whose input changed,
                upd_ms = ls.ms_items                             # timed (with the attention scalars) before the gather
                # GAT gather: every fetched z row (full recomputation of constrained destinations, old and new
                # rows of exchanged terms) with its id and attention scalars; aggregate rows read and written
                gbytes = ls.n_pairs * (4.0 * d_agg + 8.0 + 4.0 * cfg.spec.heads) + ls.n_affected * 12.0 * d_agg
            if ls.n_src or (cfg.spec.kind == wl.GAT and ls.n_affected):
                agg["gather_ms"] += ls.ms_gather
                agg["gather_bytes"] += gbytes
                agg["gather_launches"] += 1
            agg["update_ms"] += upd_ms
            agg["update_flop"] += flop
            agg["expand_ms"] += ls.ms_expand
            agg["compact_ms"] += ls.ms_compact
            agg["items_ms"] += ls.ms_items
            agg["combine_ms"] += ls.ms_combine
            pl = per_layer[l]
            pl["n_src"] += ls.n_src; pl["n_aff"] += ls.n_affected; pl["n_pairs"] += ls.n_pairs
            pl["n_in"] += ls.n_in_edges; pl["gather_ms"] += ls.ms_gather; pl["update_ms"] += upd_ms
            pl["bytes"] += gbytes
    torch.cuda.synchronize()
    ms_per_step_events = (time.perf_counter() - t_start2) * 1e3 / K

    # ---- comparison legs (Section II-C): the same chained stream continued with deltas folded at every layer (the
    # default lets the device recompute a layer whose changed sources exceed a quarter of the graph), with every
    # affected vertex recomputed over its whole in-neighbourhood ("unaffected embedding reuse"), and with the whole
    # graph recomputed per batch
    ses.profiling(False)
    mode_ms = {}
    at = args.warmup + 2 * K
    for name, mode in (("incremental_every_layer", 0), ("recompute_affected", 1), ("full_graph", 2)):
        if args.agg_only and mode != 0:                  # recomputation reads hidden rows, which this cache does not keep
            mode_ms[name] = None
            continue
        ses.mode(mode)
        ses.apply(dev_batches[at])                       # one untimed step in the new mode
        torch.cuda.synchronize()
        t3 = time.perf_counter()
        for b in dev_batches[at + 1:at + k_modes]:
            ses.apply(b)
        torch.cuda.synchronize()
        mode_ms[name] = (time.perf_counter() - t3) * 1e3 / max(1, k_modes - 1)
        at += k_modes
    ses.mode(3)

    # ---- on-demand leg (Section IV-D): batches only mark vertices stale, each is followed by a query for the
    # final-layer rows of 1000 random vertices, which recomputes the stale part of their L-hop in-neighbourhood
    on_demand = None
    if cfg.spec.kind not in (wl.GAT, wl.AGNN, wl.GGCN) and not args.agg_only:
        rng = np.random.default_rng(args.seed + 77)
        ses.lazy(True)
        t_apply = t_query = 0.0
        n_rec = 0
        for b in dev_batches[at:at + k_modes]:
            q = rng.choice(cfg.n, min(1000, cfg.n), replace=False).astype(np.int32)
            torch.cuda.synchronize()
            t4 = time.perf_counter()
            ses.apply(b, want_rows=False)
            t5 = time.perf_counter()
            _, nr = ses.query(q)
            t6 = time.perf_counter()
            t_apply += t5 - t4
            t_query += t6 - t5
            n_rec += nr
        t7 = time.perf_counter()
        ses.lazy(False)                                  # recompute everything still stale
        t_flush = time.perf_counter() - t7
        on_demand = {"batches": k_modes, "query_vertices": min(1000, cfg.n),
                     "apply_ms_per_batch": round(t_apply * 1e3 / k_modes, 4),
                     "query_ms": round(t_query * 1e3 / k_modes, 4), "vertices_recomputed_per_query": n_rec / k_modes,
                     "final_flush_ms": round(t_flush * 1e3, 3),
                     "note": "query time includes the upload of the 1000 ids and the allocation of the result"}

    # HBM bytes per launch measured with rocprofv3 counters on this workload (committed summary), if present
    traffic = None
    import glob
    if args.scale == 1.0 and not args.batch_edges:
        for tpath in sorted(glob.glob(os.path.join(ROOT, "profiles", "*_%s_*.txt" % cfg.name))):
            for line in open(tpath):
                if line.startswith("traffic_bytes_per_launch:"):
                    traffic = int(line.split(":")[1].split()[0])
    nl = max(1, agg["gather_launches"])
    g_avg_ms = agg["gather_ms"] / nl
    g_avg_bytes = agg["gather_bytes"] / nl
    achieved = (g_avg_bytes / 1e9) / (g_avg_ms / 1e3) if g_avg_ms > 0 else 0.0
    kname = ("gat_gather_kernel (attention gather: Algorithm 3 exchange / constrained full recomputation)"
             if cfg.spec.kind == wl.GAT else
             "delta-message gather + fold (gather_sparse_kernel on layers with few changed sources, gather_kernel otherwise)")
    roofline = {"kernel": kname, "bound": "hbm",
                "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                "avg_launch_ms": round(g_avg_ms, 4), "avg_launch_bytes": round(g_avg_bytes),
                "launches_per_step": agg["gather_launches"] / K}
    upd_tflops = (agg["update_flop"] / 1e12) / (agg["update_ms"] / 1e3) if agg["update_ms"] > 0 else 0.0

    out = {
        "metric": "edge_updates_per_s", "value": round(value, 1), "unit": "edge updates/s", "n_gpus": 1,
        "steps": K, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": cfg.name, "model": wl.KIND_NAMES[cfg.spec.kind], "dims": dims, "vertices": cfg.n,
                   "edges": cfg.e, "batch_inserts": cfg.n_ins, "batch_deletes": cfg.n_del,
                   "batch_feature_rows": cfg.n_feat, "chained_batches": n_total, "seed": args.seed, "scale": args.scale},
        "latency_ms": {"median": round(float(np.median(lat)), 4), "mean": round(float(np.mean(lat)), 4),
                       "p95": round(float(np.percentile(lat, 95)), 4), "min": round(float(np.min(lat)), 4)},
        "roofline": roofline,
        "events_pass": {"steps": K, "ms_per_step": round(ms_per_step_events, 4),
                        "note": "second timed pass with per-phase HIP events on; roofline, update_gemm, "
                                "phase_ms_per_step and per_layer_avg come from it"},
        "update_gemm": {"bound": "mfma", "achieved": round(upd_tflops, 2), "peak": FP32_MFMA_PEAK_TFLOPS,
                        "unit": "TFLOP/s", "frac": round(upd_tflops / FP32_MFMA_PEAK_TFLOPS, 4)},
        "modes_ms_per_step": {"default_incremental_with_auto_recompute_of_saturated_layers": round(ms_per_step, 4),
                              "incremental_every_layer": None if mode_ms["incremental_every_layer"] is None else round(mode_ms["incremental_every_layer"], 4),
                              "recompute_affected": None if mode_ms["recompute_affected"] is None else round(mode_ms["recompute_affected"], 4),
                              "full_graph": None if mode_ms["full_graph"] is None else round(mode_ms["full_graph"], 4), "steps_each": k_modes - 1},
        "edges_processed_per_step": {"default_mode_source_rows_fetched": round(sum(pl["n_pairs"] for pl in per_layer) / K),
                                     "recompute_affected_in_edges": round(sum(pl["n_in"] for pl in per_layer) / K),
                                     "full_graph": L * cfg.e},
        "on_demand": on_demand,
        "cache_workspace_GB": round(ses.cache.ws.numel() * ses.cache.ws.element_size() / 1e9, 3),
        "gpu_full_forward_ms": round(ses.cache.init_ms, 3),   # nrt_cache_init: full-neighbour L-layer forward on the GPU
        "phase_ms_per_step": {k[:-3]: round(v / K, 4) for k, v in agg.items() if k.endswith("_ms")},
        "per_layer_avg": [{"layer": l + 1, "n_src": pl["n_src"] / K, "n_affected": pl["n_aff"] / K,
                           "delta_messages": pl["n_pairs"] / K, "in_edges_scanned": pl["n_in"] / K,
                           "gather_ms": round(pl["gather_ms"] / K, 4), "update_ms": round(pl["update_ms"] / K, 4),
                           "gather_GBps": round((pl["bytes"] / 1e9) / (pl["gather_ms"] / 1e3), 1) if pl["gather_ms"] > 0 else 0.0}
                          for l, pl in enumerate(per_layer)],
    }

    if not args.no_cpu_baseline:
        from oracle import rtec_oracle as orc
        fs, fd, fw = final_edges
        xf = np.array(x, copy=True)
        for b in batches:
            if len(b.feat_ids):
                xf[b.feat_ids] = b.feat_rows
        # bounded sample: whole recomputations of the final snapshot until about 10 s of CPU work (at most 5)
        t_cpu_total, n_rec = 0.0, 0
        while n_rec < 5 and (n_rec == 0 or t_cpu_total < 10.0):
            t2 = time.perf_counter()
            ref = orc.forward(cfg.spec, params, cfg.n, fs, fd, fw, xf)
            t_cpu_total += time.perf_counter() - t2
            n_rec += 1
        t_cpu = t_cpu_total / n_rec
        per_batch = cfg.n_ins + cfg.n_del
        out["cpu_baseline"] = {"value": round(per_batch / t_cpu, 2), "unit": "edge updates/s",
                               "cores": orc.num_threads(), "kind": "oracle",
                               "sample": "%d fp64 full-neighbour %d-layer recomputations of the final snapshot "
                                         "(%.2f s each), i.e. the cost per batch without any cache" % (n_rec, L, t_cpu),
                               "seconds_per_recompute": round(t_cpu, 3)}
        got = ses.layer(L).cpu().numpy()
        err = float(np.max(np.abs(got.astype(np.float64) - ref[-1]) / np.maximum(np.abs(ref[-1]), 1.0)))
        out["parity_after_chain"] = {"max_rel_err_elementwise": err, "batches_applied": n_total}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
