/*
 * nrt.h -- C ABI of the incremental runtime-embedding-computation (RTEC) library for one MI355X.
 *
 * The library keeps, resident in HBM, a mutable directed graph (out-lists and in-lists) and, for an
 * L-layer GNN, the per-layer caches the paper's incremental layer needs (Algorithm 1 "Require":
 * the previous aggregated neighbour embedding and the previous neighbour context), plus the layer
 * outputs.  nrt_cache_init runs the ordinary full-neighbour forward (Eq. 1) once; nrt_apply_batch
 * then applies a batch of edge insertions, edge deletions and feature replacements by
 *   (1) expanding the affected vertex set hop by hop (Algorithm 4),
 *   (2) gathering delta messages over the affected edges only and folding them into the cached
 *       aggregates (the message and aggregation steps of Algorithm 1, Algorithm 3 for GAT),
 *   (3) re-running the dense update on the affected rows only (the update step of Algorithm 1),
 *   (4) writing the refreshed rows back into the caches,
 * and returns the refreshed final-layer rows with the sorted list of affected vertex ids.
 * By Theorem 1 the result equals a full recomputation on the post-update snapshot.
 *
 * Conventions
 *   - Every call returns an nrt_status.  Nothing throws or aborts.  nrt_last_error() gives a
 *     message for the last failing call on the calling thread (borrowed, valid until the next call).
 *   - "device" pointers are HIP device memory of the current device, "host" pointers ordinary
 *     host memory.  All matrices are dense row-major fp32.  Vertex ids are int32 in [0, N).
 *   - The library allocates no device memory: the caller queries *_workspace_bytes and passes a
 *     device buffer (256-byte aligned) that the handle then owns the use of until it is destroyed.
 *     Inputs are borrowed only for the duration of a call (they are copied into the workspace).
 *   - stream is the caller's hipStream_t passed as void* (NULL = default stream).  Calls that
 *     return counts to the host synchronise that stream before returning.
 *   - Handles are not thread-safe; calls on one handle (and on a cache and its graph) must not overlap.
 *   - Messages flow source -> destination: an edge <u,v> makes u an in-neighbour of v (N(v) in Eq. 1).
 *   - The graph is simple and directed: no duplicate edges, no explicit self-loops (GCN and GAT add
 *     their own implicit self-loop, GraphSAGE and GIN their own self term).
 */
#ifndef NRT_H
#define NRT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define NRT_MAX_LAYERS 4

typedef enum {
    NRT_OK = 0,
    NRT_ERR_INVALID_ARG = 1, /* null pointer, bad size, bad enum, misaligned or undersized workspace */
    NRT_ERR_BAD_BATCH = 2,   /* the batch violates its contract; graph and caches are unchanged      */
    NRT_ERR_STATE = 3,       /* call order misuse                                                     */
    NRT_ERR_OOM = 4,         /* adjacency pool exhausted (batch not applied) or host allocation failed */
    NRT_ERR_DEVICE = 5,      /* a HIP call failed                                                     */
    NRT_ERR_UNSUPPORTED = 6  /* model shape outside what the kernels cover                            */
} nrt_status;

typedef enum { NRT_GCN = 1, NRT_SAGE_MEAN = 2, NRT_GIN = 3, NRT_GAT = 4, NRT_COMMNET = 5, NRT_PINSAGE = 6, NRT_AGNN = 7, NRT_MONET = 8, NRT_GGCN = 9, NRT_RGCN = 10, NRT_RGAT = 11 } nrt_model_kind;

typedef struct nrt_graph nrt_graph;
typedef struct nrt_cache nrt_cache;

/*
 * Model description.  Layer l = 1..L maps width dims[l-1] to dims[l]; hidden layers are activated
 * (ReLU; ELU for GAT), the last layer is linear.  All widths must be multiples of 4 and <= 1024.
 *   NRT_GCN       (Eq. 2; Table II row GCN)   d_v = indeg(v)+1;
 *                 h_v = act( (sum_{u in N(v) U {v}} x_u / sqrt(d_u d_v)) W[l][0] + b[l][0] )
 *   NRT_SAGE_MEAN (Table II row GraphSAGE, update on the concatenation as in the PinSAGE row)
 *                 h_v = act( [x_v || mean_{u in N(v)} x_u] W[l][0] + b[l][0] ),  W is [2 d_{l-1}][d_l]
 *   NRT_GIN       (Fig. 4)  t_v = (1+gin_eps) x_v + sum_u w_uv x_u;
 *                 h_v = act( ReLU(t_v W[l][0] + b[l][0]) W[l][1] + b[l][1] ),  W[l][1] is [d_l][d_l]
 *   NRT_GAT       (Eq. 3-4, Algorithms 2-3)  z = x W[l][0] viewed [heads][head_dim], dims[l] = heads*head_dim;
 *                 e_uv = LeakyReLU_slope(att_dst[l][k] . z_v^k + att_src[l][k] . z_u^k), softmax over
 *                 N(v) U {v}, h_v = act( sum_u alpha_uv z_u + b[l][0] )
 *   NRT_COMMNET   (Table II row CommNet)  a_v = sum_{u in N(v)} x_u (no normalisation);
 *                 h_v = act( [x_v || a_v] W[l][0] + b[l][0] ),  W is [2 d_{l-1}][d_l]: rows W_1 (self), then W_2
 *   NRT_PINSAGE   (Table II row PinSAGE)  m_u = ReLU(x_u W[l][1] + b[l][1]),  W[l][1] is [d_{l-1}][d_{l-1}];
 *                 a_v = (sum_{u in N(v)} w_uv m_u) / |N(v)|  (w_uv = 1 on an unweighted graph, a_v = 0 if N(v) is empty);
 *                 h_v = act( [x_v || a_v] W[l][0] + b[l][0] ),  W[l][0] is [2 d_{l-1}][d_l]
 *   NRT_AGNN      (Table II row A-GNN)  a_v = sum_{u in N(v)} agnn_beta[l] * cos(x_v, x_u) * x_u, the cosine of a
 *                 zero row taken as 0;  h_v = act( a_v W[l][0] + b[l][0] ).  The message reads the destination's own
 *                 row: a "constrained" model (Section III-D), recomputed in full where that row changed
 *   NRT_MONET     (Table II row MoNet)  J = monet_kernels Gaussian kernels per layer with means monet_mu[l] and diagonal
 *                 precisions monet_prec[l] (both [J][d_{l-1}], precisions >= 0):
 *                 g_j(x) = exp( -1/2 sum_k monet_prec[l][j][k] (x_k - monet_mu[l][j][k])^2 );
 *                 a_v = sum_{u in N(v)} g(x_u)  (a J-vector);  h_v = act( a_v W[l][0] + b[l][0] ),  W[l][0] is [J][d_l]
 *   NRT_GGCN      (Table II row G-GCN)  a_v = sum_{u in N(v)} sigmoid(x_u W_1 + x_v W_2) * x_u element by element, with
 *                 W[l][1] = [W_1; W_2] of shape [2 d_{l-1}][d_{l-1}];  h_v = act( a_v W[l][0] + b[l][0] ).  Constrained
 *                 like NRT_AGNN (the gate reads the destination's own row)
 *   NRT_RGCN      (Table II row RGCN)  typed edges: the graph is weighted and the weight of edge <u,v> is its relation id
 *                 r(u,v), an integer in [0, n_relations) stored as a float (an ordered pair of vertices has one edge, hence
 *                 one relation).  W[l][1] = [W_0 | ... | W_{R-1}] of shape [d_{l-1}][R d_l], one column block per relation;
 *                 a_v = (sum_{u in N(v)} x_u W_{r(u,v)}) / |N(v)|  (the count runs over all in-neighbours, a_v = 0 if there
 *                 are none);  h_v = act( x_v W[l][0] + a_v + b[l][0] ),  W[l][0] = W_o is [d_{l-1}][d_l].
 *                 n_relations * d_l <= 4096, vertices * n_relations < 2^31.  nrt_cache_init returns NRT_ERR_INVALID_ARG
 *                 when an edge weight is not such an id, nrt_apply_batch NRT_ERR_BAD_BATCH for an inserted edge
 *   NRT_RGAT      (Table II row RGAT)  typed edges as for NRT_RGCN.  W[l][0] = [W_0 | ... | W_{R-1}] of shape
 *                 [d_{l-1}][R head_dim], att_src[l] and att_dst[l] are [R][head_dim], dims[l] = head_dim for l >= 1.  Per
 *                 relation r: z^r = x W_r, e_uv = LeakyReLU_slope(att_dst[l][r] . z^r_v + att_src[l][r] . z^r_u) and one
 *                 softmax over { u in N(v) : r(u,v) = r } U {v} (as for NRT_GAT the self-loop is a member of every group);
 *                 h_v = act( sum_r sum_u alpha^r_uv z^r_u + b[l][0] ), ELU on hidden layers.  R head_dim <= 1024.
 *                 Constrained like NRT_GAT: where z of the destination changed its groups are recomputed (Algorithm 2),
 *                 elsewhere Algorithm 3 exchanges terms inside the group of each changed edge
 * W, b, att_* are device pointers, row-major [in][out] / [heads][head_dim]; b entries may be NULL (zero).
 * They are copied at nrt_cache_init.
 */
typedef struct {
    int32_t kind;                       /* nrt_model_kind */
    int32_t n_layers;                   /* 1..NRT_MAX_LAYERS */
    int32_t dims[NRT_MAX_LAYERS + 1];   /* d_0..d_L */
    int32_t heads, head_dim;            /* GAT; RGAT reads head_dim (its groups are the relations) */
    float gin_eps;                      /* GIN only */
    float leaky_slope;                  /* GAT, RGAT */
    const float* W[NRT_MAX_LAYERS][2];  /* device */
    const float* b[NRT_MAX_LAYERS][2];  /* device or NULL */
    const float* att_src[NRT_MAX_LAYERS]; /* device, GAT and RGAT */
    const float* att_dst[NRT_MAX_LAYERS]; /* device, GAT and RGAT */
    float agnn_beta[NRT_MAX_LAYERS];    /* A-GNN only: the scalar of layer l+1 (host values) */
    int32_t monet_kernels;              /* MoNet only: J, a multiple of 4 in [4, 1024] */
    const float* monet_mu[NRT_MAX_LAYERS];   /* device, MoNet only */
    const float* monet_prec[NRT_MAX_LAYERS]; /* device, MoNet only */
    int32_t agg_only;                   /* 1: keep only the aggregates of the hidden layers and recompute their rows when
                                           a batch needs them (Section IV, "Recomputation-based embedding storage
                                           optimization").  GCN, GAT, RGAT and MoNet, whose update reads the
                                           aggregate alone, RGCN, and GIN, GraphSAGE, CommNet when aggregate_first is 0 and
                                           d_l <= d_{l-1} for every layer above the first (the row is then read only
                                           through the cached products h W); NRT_ERR_UNSUPPORTED otherwise.  Saves
                                           N * (d_1 + ... + d_{L-1}) floats of the workspace; such a cache refuses
                                           nrt_get_layer for hidden layers and the on-demand mode, a GCN one also
                                           NRT_MODE_RECOMPUTE and NRT_MODE_FULL, whose kernels read those rows (the
                                           others recompute from the cached projections / message tables).       */
    int32_t n_relations;                /* RGCN, RGAT: number of edge types R                                       */
    int32_t aggregate_first;            /* GCN, GIN, GraphSAGE, CommNet.  0 (default): a layer whose output is not wider
                                           than its input (d_l <= d_{l-1}; GCN: d_l < d_{l-1}) applies its weight matrix (GIN: the first one;
                                           GraphSAGE, CommNet: the neighbour half W_2) to the messages before the
                                           aggregation, sum_u c_uv (x_u W) = (sum_u c_uv x_u) W: the rows that the
                                           gather moves and the cached aggregate (nrt_get_aggregate) are then d_l wide,
                                           at the price of one more N x d_l table per such layer (GraphSAGE, CommNet:
                                           two, the self half x W_1 is cached as well).  1: always aggregate
                                           x itself, as Eq. 1-2 and Fig. 4 are written.  The results agree up to
                                           rounding.                                                               */
} nrt_model_desc;

/*
 * One update batch, applied atomically as three sets (Section IV-B: an inserted element contributes
 * a positive message, a deleted one a negative message, a replaced one both).  All arrays are device
 * pointers (may be NULL when the matching count is 0).
 * Contract: ids in range, no self-loops, no entry repeated inside a list, inserted edges absent from
 * the graph, deleted edges present, feature ids distinct.  ins_w is required iff the graph is weighted.
 */
typedef struct {
    int64_t n_ins; const int32_t* ins_src; const int32_t* ins_dst; const float* ins_w;
    int64_t n_del; const int32_t* del_src; const int32_t* del_dst;
    int64_t n_feat; const int32_t* feat_ids; const float* feat_rows; /* [n_feat][d_0] */
} nrt_batch;

/* Per-layer counters and timings of the last nrt_apply_batch (timings only when profiling is on). */
typedef struct {
    int64_t n_src;        /* |sources of change| entering the layer                        */
    int64_t n_affected;   /* |A_l|                                                         */
    int64_t n_items;      /* work items (destination, in-list chunk) of the gather         */
    int64_t n_in_edges;   /* in-edges of A_l scanned by the gather                         */
    int64_t n_pairs;      /* source rows fetched: delta messages folded (GAT: z rows read) (profiling only) */
    float ms_expand, ms_compact, ms_items /* GAT: the z product and attention scalars */,
          ms_gather /* the gather kernels alone */, ms_combine, ms_update;
} nrt_layer_stats;

typedef struct {
    int32_t n_layers;
    nrt_layer_stats layer[NRT_MAX_LAYERS];
    float ms_ingest;      /* validate + structural fold + graph mutation + layer-0 deltas */
    float ms_total;       /* first to last event of the call                              */
    int64_t n_launches;   /* kernel launches the call issued                              */
} nrt_stats;

/* ---- graph -------------------------------------------------------------------------------- */

/* Bytes of device workspace for a graph of n vertices that may grow to e_capacity edges. */
nrt_status nrt_graph_workspace_bytes(int64_t n_vertices, int64_t e_capacity, int32_t weighted, size_t* bytes /*host*/);

/*
 * Build the device graph from CSR (out-edges grouped by source) and/or CSC (in-edges grouped by
 * destination); at least one of the two must be given, the other is derived on the device.
 *   csr_indptr int64[n+1], csr_indices int32[e] (destinations), csr_weights float[e] or NULL   -- device
 *   csc_indptr int64[n+1], csc_indices int32[e] (sources),      csc_weights float[e] or NULL   -- device
 * weighted != 0 requires weights for every given form.  e_capacity >= n_edges bounds later growth.
 * Errors: NRT_ERR_INVALID_ARG (sizes, ids out of range or self-loops found on the device, workspace too
 * small).  *out is written only on success.
 */
nrt_status nrt_graph_create(int64_t n_vertices, int64_t n_edges, int64_t e_capacity, int32_t weighted,
                            const int64_t* csr_indptr, const int32_t* csr_indices, const float* csr_weights,
                            const int64_t* csc_indptr, const int32_t* csc_indices, const float* csc_weights,
                            void* workspace, size_t workspace_bytes, void* stream, nrt_graph** out);
void nrt_graph_destroy(nrt_graph*);
nrt_status nrt_graph_num_edges(const nrt_graph*, int64_t* n_edges /*host*/);

/*
 * Copy the current in-lists out (tests): indptr int64[n+1], indices int32[cap] device buffers with
 * cap >= current edge count; weights may be NULL.  Order inside a list is the storage order.
 */
nrt_status nrt_graph_export_csc(const nrt_graph*, int64_t* indptr, int32_t* indices, float* weights,
                                int64_t cap, void* stream);

/*
 * nrt_graph_export_csc for callers that cannot allocate device memory and hand the library no scratch of their own
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same result, but the
 * block sums of the offset scan live in a device array inside the library (1 MiB per GPU, held until the process
 * ends) instead of the graph's workspace, and the call allocates nothing.  Graphs of more than 134 184 959 vertices
 * do not fit that array: NRT_ERR_INVALID_ARG with a message, nothing written.  All calls on one GPU share the
 * array (it keeps the last call's contents; nothing in it needs to start at zero): calls that overlap on one GPU race.
 * Other arguments, errors and the final stream synchronisation as nrt_graph_export_csc.
 */
nrt_status nrt_graph_export_csc_static(const nrt_graph*, int64_t* indptr, int32_t* indices, float* weights,
                                       int64_t cap, void* stream);

/* ---- caches ------------------------------------------------------------------------------- */

nrt_status nrt_cache_workspace_bytes(const nrt_graph*, const nrt_model_desc*, int64_t max_batch_edges,
                                     int64_t max_batch_feats, size_t* bytes /*host*/);

/*
 * Full L-layer forward over the current graph (Eq. 1 per layer); fills every per-layer cache.
 * features: device float[n][d_0], copied.  The cache borrows the graph for its lifetime.
 */
nrt_status nrt_cache_init(nrt_graph*, const nrt_model_desc*, const float* features, int64_t max_batch_edges,
                          int64_t max_batch_feats, void* workspace, size_t workspace_bytes, void* stream,
                          nrt_cache** out);
void nrt_cache_destroy(nrt_cache*);

/*
 * Apply one batch incrementally (Algorithms 1, 3, 4).
 *   affected_ids  device int32[capacity]: the vertices whose final-layer embedding may have changed,
 *                 ascending, no repeats (the structural affected set of Algorithm 4).
 *   affected_rows device float[capacity][d_L] or NULL: their refreshed final-layer embeddings.
 *   n_affected    host: number of entries written.
 * Errors: NRT_ERR_BAD_BATCH (contract violated, or batch larger than the sizes given at init; state
 * unchanged), NRT_ERR_OOM (adjacency pool exhausted; state unchanged), NRT_ERR_INVALID_ARG (capacity
 * smaller than the affected count: caches ARE updated, only the copy-out is skipped, *n_affected holds the
 * needed capacity).  NRT_ERR_DEVICE (a HIP call failed) and NRT_ERR_STATE (an internal consistency check of the
 * cache layout's bounds, unreachable for a graph within e_capacity) can be raised after the batch has been validated:
 * graph and caches are then unspecified and must be rebuilt (destroy, nrt_graph_create, nrt_cache_init).
 * Synchronises the stream before returning.
 */
nrt_status nrt_apply_batch(nrt_cache*, const nrt_batch*, int32_t* affected_ids, float* affected_rows,
                           int64_t capacity, int64_t* n_affected, void* stream);

/* Borrowed device view of the cached layer output h^l (l = 0: current features), row-major, ld floats per row. */
nrt_status nrt_get_layer(const nrt_cache*, int32_t layer, const float** rows, int64_t* n_rows, int64_t* ld);
/* Borrowed device view of the cached aggregate of layer l = 1..L in context-free form (the sum before
 * msg_cbn is applied: Algorithm 1's a-hat), width floats per row.  What is summed depends on the model and the
 * layer: h^{l-1} rows (width d_{l-1}), or the messages the layer aggregates when those are not h itself (PinSAGE,
 * MoNet, RGCN, GAT, RGAT, and the layers of GCN, GIN, GraphSAGE and CommNet that apply their weights before the
 * aggregation, see nrt_model_desc.aggregate_first): *width tells. */
nrt_status nrt_get_aggregate(const nrt_cache*, int32_t layer, const float** rows, int64_t* n_rows, int64_t* width);
/* Per-layer affected list A_l (l = 1..L) of the last batch: borrowed device int32 array, ascending. */
nrt_status nrt_get_layer_affected(const nrt_cache*, int32_t layer, const int32_t** ids, int64_t* n);

/* How nrt_apply_batch brings the caches up to date (Section II-C, the non-incremental ways of running RTEC
 * that the paper compares against, on the same kernels and the same caches; results are equal up to fp32
 * rounding in every mode, and a cache may switch mode between batches):
 *   NRT_MODE_INCREMENTAL  delta messages over the affected subgraph only (Algorithms 1, 3, 4) at every layer.
 *   NRT_MODE_RECOMPUTE    "unaffected embedding reuse": the same affected sets, but every affected vertex
 *                         re-aggregates its whole in-neighbourhood from the current h^{l-1}.
 *   NRT_MODE_FULL         every vertex of every layer is recomputed on the updated graph; the affected list
 *                         is still produced by the frontier expansion.
 *   NRT_MODE_AUTO         the default: incremental, except that a layer whose changed sources exceed a quarter
 *                         of the vertices (nearly every in-edge of its affected vertices then carries a delta)
 *                         is served as in NRT_MODE_RECOMPUTE; decided per layer on the device.  GAT layers are
 *                         always incremental.
 * Errors: NRT_ERR_INVALID_ARG (null cache, unknown mode), NRT_ERR_UNSUPPORTED (NRT_MODE_RECOMPUTE or NRT_MODE_FULL on
 * a GCN cache with aggregate-only storage). */
typedef enum { NRT_MODE_INCREMENTAL = 0, NRT_MODE_RECOMPUTE = 1, NRT_MODE_FULL = 2, NRT_MODE_AUTO = 3 } nrt_mode;
nrt_status nrt_set_mode(nrt_cache*, int32_t mode);
/* On-demand embedding computation (Section IV-D): serve a small set of query vertices without keeping every
 * cached row up to date.  With the on-demand mode on, nrt_apply_batch validates the batch, mutates the graph,
 * replaces the feature rows and expands the affected sets as usual (affected_ids is filled; affected_rows must be
 * NULL), but instead of refreshing the caches it only records, per layer, that the affected vertices are stale.
 * nrt_query then returns the final-layer rows of the queried vertices on the current snapshot: it intersects the
 * stale sets with the L-hop in-neighbourhood of the query (need_L = Q and stale_L, need_{l-1} = stale_{l-1} and
 * (need_l or their in-neighbours)), recomputes exactly those vertices layer by layer over their whole
 * in-neighbourhoods (the recomputation of NRT_MODE_RECOMPUTE) and clears their stale marks; everything else stays
 * stale until some later query needs it.  Turning the mode off recomputes all remaining stale vertices first.
 * nrt_query also works with the mode off (it then only gathers rows).  Every model kind is served; for the
 * constrained models (GAT, A-GNN, G-GCN; Section III-D) what a layer caches per source vertex (z and the attention
 * scalars, inverse norms, gate projections) is re-derived for exactly the rows a query brings up to date one layer
 * below, and for the rows of h^0 every batch replaces.  Not available with aggregate-only storage.
 *   query_ids  device, n_query ids in [0, N), repeats allowed
 *   rows       device, [n_query][d_L], row i = embedding of query_ids[i]
 *   n_recomputed  host, may be NULL: vertices recomputed, summed over the layers
 * Errors: NRT_ERR_INVALID_ARG (null pointers, an id out of range: rows are then unspecified),
 * NRT_ERR_UNSUPPORTED (aggregate-only storage), NRT_ERR_DEVICE.  Both calls synchronise the stream before returning. */
nrt_status nrt_set_lazy(nrt_cache*, int32_t on, void* stream);
nrt_status nrt_query(nrt_cache*, const int32_t* query_ids, int64_t n_query, float* rows, int64_t* n_recomputed /*host*/,
                     void* stream);
/* A batch and a query in one call, on-demand mode only (Section IV-D: the computation graph of an on-demand batch is
 * the affected subgraph intersected with the K-hop subgraph of the queried vertices).  The batch is applied as by
 * nrt_apply_batch in on-demand mode (graph, features, affected sets, stale marks; affected_ids is filled), then the
 * final-layer rows of query_ids are returned as by nrt_query.  The difference lies in how the needed vertices are
 * brought up to date: one that was up to date before this batch takes the incremental layer (Algorithm 1: delta
 * messages of its changed in-neighbours, the batch's inserted and deleted edges) instead of being summed again over its
 * whole in-neighbourhood; one that an earlier batch had already left stale is recomputed.  Folding is done for the
 * models whose message is h itself and does not read the destination (GCN, GraphSAGE, GIN, CommNet); the others
 * recompute every needed vertex, as nrt_query does.
 *   query_ids device, n_query > 0 ids in [0, N), repeats allowed;  query_rows device [n_query][d_L]
 *   n_updated  host, may be NULL: vertices brought up to date, summed over the layers
 *   n_recomputed host, may be NULL: those of them recomputed over their whole in-neighbourhood
 * Errors: as nrt_apply_batch; NRT_ERR_INVALID_ARG for a query id out of range (nothing is changed, like a bad batch);
 * NRT_ERR_STATE when the on-demand mode is off.  Synchronises the stream. */
nrt_status nrt_apply_batch_query(nrt_cache*, const nrt_batch*, int32_t* affected_ids, int64_t capacity, int64_t* n_affected /*host*/,
                                 const int32_t* query_ids, int64_t n_query, float* query_rows,
                                 int64_t* n_updated /*host*/, int64_t* n_recomputed /*host*/, void* stream);
nrt_status nrt_set_profiling(nrt_cache*, int32_t on);
nrt_status nrt_get_stats(const nrt_cache*, nrt_stats* out /*host*/);

/*
 * Bandwidth ceilings of the device, for the report that sets the gathers' achieved HBM rate beside what a plain
 * streaming kernel reaches on the same GPU (Section V reports response time and throughput; the roofline view is
 * this build's).  kind 0: copy a -> b (n_floats read and n_floats written per pass); kind 1: read a (b receives at most
 * one float).  a, b: device, 16-byte aligned, n_floats each, distinct.  One untimed pass, then `reps` passes timed with
 * HIP events on `stream`; *ms_per_pass (host) is their average.  Synchronises the stream.
 * Errors: NRT_ERR_INVALID_ARG, NRT_ERR_DEVICE.
 */
nrt_status nrt_measure_stream(int32_t kind, float* b, const float* a, int64_t n_floats, int32_t reps, void* stream,
                              float* ms_per_pass /*host*/);

const char* nrt_last_error(void);
const char* nrt_version(void);

#ifdef __cplusplus
}
#endif
#endif /* NRT_H */
