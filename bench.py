#!/usr/bin/env python3
"""Benchmark of the incremental RTEC hot path on one MI355X.

A step = one nrt_apply_batch (validate + ingest, frontier expansion, delta gather/fold, affected-row update
with write-back, all layers) over one synthetic update batch; batches are chained (each step sees the graph
and caches the previous step left).  Inputs (graph, caches, every batch) are resident in HBM before the timed
region.  Per configuration two timed passes of K steps each: the first, with the library's per-phase HIP events
off, gives value, ms_per_step and latency; the second, over the next K chained batches with the events on (they
cost a few percent), gives the per-kernel durations behind `roofline`, `update_gemm` and the phase breakdown.

The headline (top level of the one JSON line) is the largest configuration, config 4 of the benchmark spec (3-layer
GIN, 10M vertices / 200M weighted edges); `other_configs` carries the same record for the other four
configurations, each timed the same way in the same run with its own CPU-oracle baseline.  `--only` runs the
chosen configuration alone.  `stream_ceilings` are a plain read kernel and a plain copy kernel of the same
library timed in the same process.
"""
import argparse
import gc
import glob
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
HEADLINE = 3                       # index into benchmark configs: config 4, the largest single-GPU configuration
# steps / warmup / steps per comparison mode of the configurations that are not the headline
NESTED_STEPS = {0: (40, 5, 10), 1: (40, 5, 10), 2: (6, 2, 4), 3: (10, 3, 4), 4: (8, 2, 4)}


def log(msg):
    print("[bench] " + msg, file=sys.stderr, flush=True)


def stream_ceilings(torch, nb):
    """What a plain streaming kernel reaches on this GPU: read-only and copy, 2 GiB buffers (far beyond every cache)."""
    n = 512 * 1024 * 1024
    a = torch.empty(n, dtype=torch.float32, device="cuda").fill_(1.0)
    b = torch.empty(n, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    ms_read = nb.nrt_measure_stream(1, b, a, 10)
    ms_copy = nb.nrt_measure_stream(0, b, a, 10)
    del a, b
    torch.cuda.empty_cache()
    return {"read_GBps": round(4.0 * n / 1e9 / (ms_read / 1e3), 1), "copy_GBps_read_plus_write": round(8.0 * n / 1e9 / (ms_copy / 1e3), 1),
            "buffer_GB": round(4.0 * n / 1e9, 2), "passes": 10,
            "note": "stream_read_kernel / stream_copy_kernel of libnrt (16 B per lane and access), HIP events around 10 passes"}


def run_config(args, index, K, W, k_modes, ceilings, with_cpu, with_on_demand):
    import torch
    from paper_2603_20622_amd import workloads as wl
    from paper_2603_20622_amd import session as S

    cfg = wl.config(index, args.scale)
    if args.model:
        kind = {"commnet": wl.COMMNET, "pinsage": wl.PINSAGE, "agnn": wl.AGNN, "monet": wl.MONET, "ggcn": wl.GGCN,
                "rgcn": wl.RGCN, "rgat": wl.RGAT}[args.model]
        mdims = list(cfg.spec.dims)
        if kind == wl.RGAT:                                     # every layer as wide as the last: the group width
            mdims = [mdims[0]] + [mdims[-1]] * (len(mdims) - 1)
        cfg.spec = wl.ModelSpec(kind, mdims, weighted=kind in (wl.PINSAGE, wl.RGCN, wl.RGAT), monet_kernels=64,
                                head_dim=mdims[-1] if kind == wl.RGAT else 0, n_relations=4)
        cfg.name = cfg.name + "_as_" + args.model
    if args.agg_only:
        cfg.spec.agg_only = True
        cfg.name = cfg.name + "_agg_only"
    if args.aggregate_first:
        cfg.spec.aggregate_first = True
        cfg.name = cfg.name + "_aggregate_first"
    if args.batch_edges:
        frac = cfg.n_ins / max(1, cfg.n_ins + cfg.n_del)
        cfg.n_ins = int(round(args.batch_edges * frac))
        cfg.n_del = args.batch_edges - cfg.n_ins
    t0 = time.time()
    src, dst, w, x, params, stream = wl.build(cfg, args.seed)
    # legs a cache with aggregate-only storage refuses are left out, and so are their batches: the final snapshot that
    # the parity check recomputes is the one after exactly the batches applied
    with_on_demand = with_on_demand and not args.agg_only
    n_mode_legs = 1 if (args.agg_only and cfg.spec.kind == wl.GCN) else 3
    n_total = 2 * K + W + n_mode_legs * k_modes + (k_modes if with_on_demand else 0)
    batches = [stream.next_batch(cfg.n_ins, cfg.n_del, cfg.n_feat) for _ in range(n_total)]
    final_edges = stream.edges()
    del stream
    log("%s: generated graph %d/%d and %d batches in %.1fs" % (cfg.name, cfg.n, cfg.e, n_total, time.time() - t0))

    ses = S.Session(cfg.spec, params, cfg.n, src, dst, w, x,
                    max_batch_edges=max(1024, 2 * (cfg.n_ins + cfg.n_del)), max_batch_feats=max(64, 2 * cfg.n_feat))
    del src, dst, w
    dev_batches = [S.DeviceBatch(b) for b in batches]
    ses.profiling(False)
    torch.cuda.synchronize()
    log("%s: caches initialised, running %d warmup + 2 x %d timed steps" % (cfg.name, W, K))

    for b in dev_batches[:W]:
        ses.apply(b)
    torch.cuda.synchronize()

    L = cfg.spec.n_layers
    dims = cfg.spec.dims

    # ---- pass 1: value, ms_per_step, latency
    lat = []
    edge_updates = 0
    launches = 0
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for b in dev_batches[W:W + K]:
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
    per_layer = [dict(n_src=0, n_aff=0, n_pairs=0, n_in=0, gather_ms=0.0, update_ms=0.0, bytes=0.0, flop=0.0) for _ in range(L)]
    t_start2 = time.perf_counter()
    for b in dev_batches[W + K:W + 2 * K]:
        ses.apply(b)
        st = ses.stats()
        launches += st.n_launches
        agg["ingest_ms"] += st.ms_ingest
        for l in range(L):
            ls = st.layer[l]
            d_in = dims[l]
            # algorithmic bytes of the gather launch: per delta message its in-list id and slot-map entry (8 B);
            # the delta rows: every changed source row once (4*d) while the delta buffer fits the 256 MB Infinity
            # Cache, else one row per delta message; every affected aggregate row read and written (8*d)
            # GCN and GIN layers that narrow apply their (first) weight matrix to the messages before the aggregation:
            # the gathered rows and the cached aggregate are then as wide as the layer's output
            weights_first = (cfg.spec.kind in (wl.GCN, wl.GIN, wl.SAGE_MEAN, wl.COMMNET)
                             and (dims[l + 1] < d_in or (dims[l + 1] == d_in and cfg.spec.kind != wl.GCN))
                             and (not cfg.spec.agg_only or cfg.spec.kind != wl.GCN) and not cfg.spec.aggregate_first)
            d_agg = dims[l + 1] if cfg.spec.kind in (wl.GAT, wl.RGCN, wl.RGAT) or weights_first else \
                (cfg.spec.monet_kernels if cfg.spec.kind == wl.MONET else d_in)
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
            if cfg.spec.kind == wl.RGCN:                         # its R message rows per changed source, likewise
                flop += 2.0 * ls.n_src * d_in * cfg.spec.n_relations * dims[l + 1]
            upd_ms = ls.ms_update
            if weights_first:
                # x W on the rows whose input changed (timed before the gather, under "items"); GCN has no product left
                # in its update, GIN its second one
                flop = 2.0 * ls.n_src * d_in * dims[l + 1]
                if cfg.spec.kind == wl.GIN:
                    flop += 2.0 * ls.n_affected * dims[l + 1] * dims[l + 1]
                if cfg.spec.kind in (wl.SAGE_MEAN, wl.COMMNET):      # both halves [W_1 | W_2] on the changed rows; no product
                    flop *= 2.0                                      # is left in the update
                upd_ms = ls.ms_update + ls.ms_items
            if cfg.spec.kind == wl.RGAT:
                # the GAT path with the relations as groups: z is R groups wide, a fetched row is one group's part
                zdim = cfg.spec.n_relations * dims[l + 1]
                flop = 2.0 * ls.n_src * d_in * zdim
                upd_ms = ls.ms_items
                gbytes = ls.n_pairs * (4.0 * d_agg + 16.0) + ls.n_affected * (8.0 * zdim + 4.0 * d_agg)
            if cfg.spec.kind == wl.GAT:
                flop = 2.0 * ls.n_src * d_in * dims[l + 1]       # z = x W on the rows whose input changed,
                upd_ms = ls.ms_items                             # timed (with the attention scalars) before the gather
                # GAT gather: every fetched z row (full recomputation of constrained destinations, old and new
                # rows of exchanged terms) with its id and attention scalars; aggregate rows read and written
                gbytes = ls.n_pairs * (4.0 * d_agg + 8.0 + 4.0 * cfg.spec.heads) + ls.n_affected * 12.0 * d_agg
            if ls.n_src or (cfg.spec.kind in (wl.GAT, wl.RGAT) and ls.n_affected):
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
            pl["bytes"] += gbytes; pl["flop"] += flop
    torch.cuda.synchronize()
    ms_per_step_events = (time.perf_counter() - t_start2) * 1e3 / K

    # ---- comparison legs (Section II-C): the same chained stream continued with deltas folded at every layer (the
    # default lets the device recompute a layer whose changed sources exceed a quarter of the graph), with every
    # affected vertex recomputed over its whole in-neighbourhood ("unaffected embedding reuse"), and with the whole
    # graph recomputed per batch
    ses.profiling(False)
    mode_ms = {}
    at = W + 2 * K
    for name, mode in (("incremental_every_layer", 0), ("recompute_affected", 1), ("full_graph", 2)):
        if args.agg_only and mode != 0 and cfg.spec.kind == wl.GCN:   # recomputation reads hidden rows, which this cache does not keep
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
    # final-layer rows of 1000 random vertices, which brings the stale part of their L-hop in-neighbourhood up to date
    on_demand = None
    if with_on_demand:
        rng = np.random.default_rng(args.seed + 77)
        ses.lazy(True)
        t_apply = t_query = t_both = 0.0
        n_rec = n_upd2 = n_rec2 = 0
        n_sep = max(1, k_modes // 2)
        n_tog = max(1, k_modes - n_sep)
        use = dev_batches[at:at + n_sep + n_tog]
        for i, b in enumerate(use):
            q = rng.choice(cfg.n, min(1000, cfg.n), replace=False).astype(np.int32)
            torch.cuda.synchronize()
            t4 = time.perf_counter()
            if i < n_sep:                                # the batch only marks vertices stale, then a separate query
                ses.apply(b, want_rows=False)
                t5 = time.perf_counter()
                _, nr = ses.query(q)
                t6 = time.perf_counter()
                t_apply += t5 - t4
                t_query += t6 - t5
                n_rec += nr
            else:                                        # batch and query in one call: up-to-date vertices are folded
                _, _, nu, nr = ses.apply_query(b, q)
                t_both += time.perf_counter() - t4
                n_upd2 += nu
                n_rec2 += nr
        t7 = time.perf_counter()
        ses.lazy(False)                                  # bring everything still stale up to date
        t_flush = time.perf_counter() - t7
        on_demand = {"query_vertices": min(1000, cfg.n),
                     "separate_calls": {"batches": n_sep, "apply_ms_per_batch": round(t_apply * 1e3 / n_sep, 4),
                                        "query_ms": round(t_query * 1e3 / n_sep, 4),
                                        "vertices_recomputed_per_query": n_rec / n_sep},
                     "batch_with_query": {"batches": len(use) - n_sep, "ms_per_call": round(t_both * 1e3 / max(1, len(use) - n_sep), 4),
                                          "vertices_updated_per_call": n_upd2 / max(1, len(use) - n_sep),
                                          "of_which_recomputed_in_full": n_rec2 / max(1, len(use) - n_sep)},
                     "final_flush_ms": round(t_flush * 1e3, 3),
                     "note": "times include the upload of the 1000 ids and the allocation of the result"}

    # HBM bytes per launch measured with rocprofv3 counters on this workload: bench.py cannot run the profiler on
    # itself, so the figure is read from the committed summary of the same command (profiles/), which is named
    traffic, traffic_source = None, None
    if args.scale == 1.0 and not args.batch_edges and not args.model and not args.agg_only and not args.aggregate_first:
        for tpath in sorted(glob.glob(os.path.join(ROOT, "profiles", "*_%s_*.txt" % cfg.name))):
            for line in open(tpath):
                if line.startswith("traffic_bytes_per_launch:"):
                    traffic = int(line.split(":")[1].split()[0])
                    traffic_source = os.path.relpath(tpath, ROOT)
    nl = max(1, agg["gather_launches"])
    g_avg_ms = agg["gather_ms"] / nl
    g_avg_bytes = agg["gather_bytes"] / nl
    achieved = (g_avg_bytes / 1e9) / (g_avg_ms / 1e3) if g_avg_ms > 0 else 0.0
    kname = ("gat_gather_kernel (attention gather: Algorithm 3 exchange / constrained full recomputation)"
             if cfg.spec.kind in (wl.GAT, wl.RGAT) else
             "delta-message gather + fold (gather_sparse_kernel on layers with few changed sources, gather_kernel otherwise)")
    roofline = {"kernel": kname, "bound": "hbm",
                "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic, "traffic_source": traffic_source,
                "frac_of_stream_read_ceiling": round(achieved / ceilings["read_GBps"], 4) if ceilings else None,
                "avg_launch_ms": round(g_avg_ms, 4), "avg_launch_bytes": round(g_avg_bytes),
                "launches_per_step": agg["gather_launches"] / K}
    # the launch that takes the longest (one layer): achieved / frac above average over all gather launches of a step,
    # which mixes the bandwidth-bound layers with the small, latency- or cache-bound ones
    heavy = max(range(L), key=lambda l: per_layer[l]["gather_ms"])
    if per_layer[heavy]["gather_ms"] > 0:
        hv = per_layer[heavy]
        hv_gbps = (hv["bytes"] / 1e9) / (hv["gather_ms"] / 1e3)
        roofline["longest_launch"] = {"layer": heavy + 1, "avg_launch_ms": round(hv["gather_ms"] / K, 4),
                                      "avg_launch_bytes": round(hv["bytes"] / K),
                                      "achieved": round(hv_gbps, 1), "frac": round(hv_gbps / HBM_PEAK_GBS, 4)}
    upd_tflops = (agg["update_flop"] / 1e12) / (agg["update_ms"] / 1e3) if agg["update_ms"] > 0 else 0.0

    out = {
        "metric": "edge_updates_per_s", "value": round(value, 1), "unit": "edge updates/s", "n_gpus": 1,
        "steps": K, "warmup": W, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": cfg.name, "vertices": cfg.n, "edges": cfg.e, "batch_inserts": cfg.n_ins,
                   "batch_deletes": cfg.n_del, "batch_feature_rows": cfg.n_feat, "chained_batches": n_total,
                   "seed": args.seed, "scale": args.scale},
        "latency_ms": {"median": round(float(np.median(lat)), 4), "mean": round(float(np.mean(lat)), 4),
                       "p95": round(float(np.percentile(lat, 95)), 4), "min": round(float(np.min(lat)), 4)},
        "roofline": roofline,
        "events_pass": {"steps": K, "ms_per_step": round(ms_per_step_events, 4),
                        "note": "second timed pass with per-phase HIP events on; roofline, update_gemm, "
                                "phase_ms_per_step and per_layer_avg come from it"},
        "update_gemm": {"bound": "mfma", "achieved": round(upd_tflops, 2), "peak": FP32_MFMA_PEAK_TFLOPS,
                        "unit": "TFLOP/s", "frac": round(upd_tflops / FP32_MFMA_PEAK_TFLOPS, 4)},
        "kernel_launches_per_step": round(launches / K, 1),
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
                           "gather_GBps": round((pl["bytes"] / 1e9) / (pl["gather_ms"] / 1e3), 1) if pl["gather_ms"] > 0 else 0.0,
                           "update_TFLOPs": round((pl["flop"] / 1e12) / (pl["update_ms"] / 1e3), 2) if pl["update_ms"] > 0 else 0.0}
                          for l, pl in enumerate(per_layer)],
    }

    got = ses.layer(L).cpu().numpy() if with_cpu else None
    ses.close()
    del ses, dev_batches
    gc.collect()
    torch.cuda.empty_cache()

    if with_cpu:
        from oracle import rtec_oracle as orc
        fs, fd, fw = final_edges
        xf = np.array(x, copy=True)
        for b in batches:
            if len(b.feat_ids):
                xf[b.feat_ids] = b.feat_rows
        # bounded sample: whole recomputations of the final snapshot until about 10 s of CPU work (at most 5; the
        # large configurations take one, 20-45 s)
        t_cpu_total, n_rec = 0.0, 0
        while n_rec < 5 and (n_rec == 0 or t_cpu_total < 10.0):
            t2 = time.perf_counter()
            ref = orc.forward(cfg.spec, params, cfg.n, fs, fd, fw, xf)[-1]
            t_cpu_total += time.perf_counter() - t2
            n_rec += 1
        t_cpu = t_cpu_total / n_rec
        per_batch = cfg.n_ins + cfg.n_del
        out["cpu_baseline"] = {"value": round(per_batch / t_cpu, 2), "unit": "edge updates/s",
                               "cores": orc.num_threads(), "kind": "oracle",
                               "sample": "%d fp64 full-neighbour %d-layer recomputation(s) of the final snapshot "
                                         "(%.2f s each), i.e. the cost per batch without any cache" % (n_rec, L, t_cpu),
                               "seconds_per_recompute": round(t_cpu, 3)}
        d = np.abs(got.astype(np.float64) - ref)
        err = float(np.max(d / np.maximum(np.abs(ref), 1.0)))
        rown = float(np.max(d / np.maximum(np.abs(ref).max(axis=1, keepdims=True), 1.0)))
        out["parity_after_chain"] = {"max_rel_err_elementwise": err, "max_rel_err_row_normalised": rown,
                                     "batches_applied": n_total}
        del ref, d, got, xf
    log("%s: %.3f ms per step, gather %.0f GB/s (%.2f of peak), update %.1f TFLOP/s, done at %.0fs"
        % (cfg.name, ms_per_step, achieved, achieved / HBM_PEAK_GBS, upd_tflops, time.time() - t0))
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="timed steps of the headline configuration (default 10)")
    ap.add_argument("--warmup", type=int, default=-1, help="untimed steps of the headline configuration (default 3)")
    ap.add_argument("--config", type=int, default=HEADLINE, help="index into BASELINE.json configs of the top-level record "
                    "(default 3: config 4, the largest)")
    ap.add_argument("--only", action="store_true", help="run the chosen configuration alone (no other_configs)")
    ap.add_argument("--scale", type=float, default=1.0, help="shrink the workload (debugging only)")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--batch-edges", type=int, default=0, help="override the batch size (edges, config 3 sweep)")
    ap.add_argument("--model", choices=["commnet", "pinsage", "agnn", "monet", "ggcn", "rgcn", "rgat"], default=None,
                    help="run another Table II model on the chosen config's graph, widths and batches (implies --only)")
    ap.add_argument("--aggregate-first", action="store_true",
                    help="GCN / GIN configs: never apply a layer's weights before its aggregation (implies --only)")
    ap.add_argument("--agg-only", action="store_true",
                    help="GCN configs: keep only the aggregates of hidden layers (storage option; implies --only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (caches resident in one MI355X's HBM, no collectives); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2603_20622_amd import binding as nb

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    only = args.only or args.model is not None or args.agg_only or args.aggregate_first or args.batch_edges > 0 or args.scale != 1.0
    t_all = time.time()
    ceilings = stream_ceilings(torch, nb)
    log("stream ceilings: read %.0f GB/s, copy %.0f GB/s" % (ceilings["read_GBps"], ceilings["copy_GBps_read_plus_write"]))
    dK, dW, dM = NESTED_STEPS[args.config]
    K = args.steps if args.steps > 0 else dK
    W = args.warmup if args.warmup >= 0 else dW
    out = run_config(args, args.config, K, W, min(K, dM) if K > 1 else 2, ceilings, not args.no_cpu_baseline, True)
    out["stream_ceilings"] = ceilings
    if not only:
        others = {}
        for index in range(5):
            if index == args.config:
                continue
            k, w, m = NESTED_STEPS[index]
            rec = run_config(args, index, k, w, m, ceilings, not args.no_cpu_baseline, index in (0, 1, 4))
            others[rec["config"]["workload"]] = rec
        out["other_configs"] = others
    out["bench_wall_s"] = round(time.time() - t_all, 1)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
