// C ABI of libnrt: handle management and the per-batch orchestration of the kernels.
#include "common.h"

#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>

// ------------------------------------------------------------------ errors
static thread_local char g_err[512] = "";
void nrt_set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}
thread_local int64_t nrt_launch_count = 0;
extern "C" const char* nrt_last_error(void) { return g_err; }
extern "C" const char* nrt_version(void) { return "nrt 0.1 (gfx950)"; }

#define REQUIRE(cond, msg)                     \
    do {                                       \
        if (!(cond)) {                         \
            nrt_set_error("%s", msg);          \
            return NRT_ERR_INVALID_ARG;        \
        }                                      \
    } while (0)

// ------------------------------------------------------------------ cache handle
constexpr int MAX_EVENTS = 16 + 8 * NRT_MAX_LAYERS;
// device counter blocks of a cache: [0 .. NRT_MAX_LAYERS] the per-layer sets of a batch, [NRT_MAX_LAYERS + 1] whole-graph
// passes, then three groups of NRT_MAX_LAYERS + 1 for a batch served together with a query (the vertices the query needs,
// those of them that were up to date before the batch, those that were already stale)
constexpr int LC_BATCH = NRT_MAX_LAYERS + 2;
constexpr int LC_TOTAL = LC_BATCH + 3 * (NRT_MAX_LAYERS + 1);

struct nrt_cache {
    nrt_graph* g;
    int kind, L;
    int dims[NRT_MAX_LAYERS + 1];
    int dagg[NRT_MAX_LAYERS + 1];       // width of the cached aggregate of layer l
    int heads, head_dim;
    float gin_eps, leaky_slope;
    int64_t max_edges, max_feats;
    int maxd;
    float* H[NRT_MAX_LAYERS + 1];
    float* S[NRT_MAX_LAYERS + 1];
    int agg_only;                       // hidden-layer rows h^l are not kept, only the aggregates (GCN, GAT, RGAT)
    float* ES[NRT_MAX_LAYERS + 1];      // agg_only, GCN: h^l of the sources of the batch's updated edges, one row per update
    int32_t* es_rows;                   // agg_only, GCN: those sources, inserts first
    float* R[NRT_MAX_LAYERS + 1];       // A-GNN: inverse norms of the rows of h^l (null otherwise)
    float* P1[NRT_MAX_LAYERS + 1];      // G-GCN: W_1 h^l and W_2 h^l by vertex (null otherwise)
    float* P2[NRT_MAX_LAYERS + 1];
    float* old_p1;                      // G-GCN: [N][max d] compact, W_1 h of the changed rows before the batch
    float* W2t[NRT_MAX_LAYERS];         // G-GCN: transposed W_2 (W_1 sits in Wt[l][1])
    float* r_old;                       // A-GNN: [N] compact, inverse norms of the changed rows before the batch
    float agnn_beta[NRT_MAX_LAYERS];
    float* MP[NRT_MAX_LAYERS + 1];      // PinSAGE, MoNet: message payload of layer l's rows (ReLU(h^l Q + q); the Gaussian
                                        // kernel responses of h^l), null otherwise
    float* MS[NRT_MAX_LAYERS + 1];      // GraphSAGE, CommNet on a weights-first layer l+1: h^l W_1 by vertex, the self half of
                                        // that layer's update (the neighbour half h^l W_2 is MP[l]); RGCN: h^l W_o; else null
    int monet_J;                        // MoNet: kernels per layer = width of its payload and aggregate
    int n_rel;                          // RGCN: relations; MP[l] then holds n_rel message rows W_r h^l per vertex
    // GCN, GIN, GraphSAGE, CommNet: layer l applies its (first / neighbour-side) weight matrix to the messages before the
    // aggregation unless that would widen the aggregated rows (d_l <= d_{l-1}): sum_u c_uv (x_u W) = (sum_u c_uv x_u) W.
    // With equal widths the gather moves the same bytes, but the product runs over the changed source rows, not over the
    // (usually far more numerous) affected rows; GCN is left out of that case, because its update would turn from one
    // fused product into a product plus a separate pass over the affected rows.
    // MP[l-1] = H^{l-1} W then plays the part of PinSAGE's message table, the cached aggregate S^l is d_l wide, and the
    // update has no product left (GCN), one less (GIN) or one of half the depth (GraphSAGE, CommNet: x_v W_1 + S_v).
    // Index: the destination layer l = 1..L.
    bool tf[NRT_MAX_LAYERS + 1];
    int no_reorder;
    float* muT[NRT_MAX_LAYERS];         // MoNet: [d_l][J] transposed means / precisions of layer l+1
    float* precT[NRT_MAX_LAYERS];
    float* Wt[NRT_MAX_LAYERS][2];
    float* bias[NRT_MAX_LAYERS][2];
    int32_t* indeg_old;
    uint32_t *bm_ddst, *bm_feat, *bm[2];
    int64_t nw_pad;
    uint8_t* flags;                     // one byte per vertex: the set an expansion hop is building
    LayerCtrs* lc;                      // device, [LC_TOTAL]
    LayerCtrs* lc_use;                  // counters the layer steps read instead of lc[l] (null: lc[l])
    int mode;                           // nrt_mode
    bool have_history;                  // n_list holds the set sizes of a previous batch (hints for kernel choice)
    bool have_history_prev;             // while a batch runs: lc_host still holds the counters of the batch before it
    int lazy;                           // on-demand mode: batches only record what became stale
    uint32_t* stale[NRT_MAX_LAYERS + 1]; // per layer: vertices whose cached aggregate / embedding is out of date
    // a batch served together with a query (nrt_apply_batch_query): the stale sets as they were before the batch, the sets
    // the query needs per layer ([0]: the sources of change of layer 1), their lists, the two classes of a layer, the
    // bitmap of the queried vertices
    uint32_t* stale_prev[NRT_MAX_LAYERS + 1];
    uint32_t* need_bm[NRT_MAX_LAYERS + 1];
    int32_t* need_list[NRT_MAX_LAYERS + 1];
    int32_t *list_fresh, *list_redo;
    uint32_t* bm_q;
    // sources of a fold given explicitly instead of the previous layer's set of the batch (null: not in use)
    const uint32_t* ov_bm; const int32_t* ov_slot; const float* ov_dp; const uint64_t* ov_count; const uint32_t* ov_coarse;
    LayerCtrs* lc_host;                 // pinned mirror, followed by the mirror of pair_ctr (profiling)
    unsigned long long* pair_host;
    int32_t* xhub_list;
    int64_t xhub_cap;
    int32_t* list[NRT_MAX_LAYERS + 1];
    int64_t n_list[NRT_MAX_LAYERS + 1];
    int32_t* slot[2];
    float* DP[2];
    float* mid;
    // GAT: z = x W, attention scalars, softmax context per (vertex, head)
    float* Z[NRT_MAX_LAYERS + 1];
    float *AS[NRT_MAX_LAYERS + 1], *AD[NRT_MAX_LAYERS + 1], *M[NRT_MAX_LAYERS + 1], *DEN[NRT_MAX_LAYERS + 1];
    float *att_src[NRT_MAX_LAYERS], *att_dst[NRT_MAX_LAYERS];
    float* AS_old;
    float *part_m, *part_den;
    bool is_gat;                        // GAT or RGAT: the kernels of gat.hip serve the layer
    int zdim;                           // their projected width heads * head_dim (RGAT: relations * head_dim, output head_dim)
    float* SD[NRT_MAX_LAYERS + 1];      // structural-delta rows of a batch, [max_edges][dagg[l]]
    float* SDden[NRT_MAX_LAYERS + 1];   // GAT: their attention-sum part, [max_edges][heads]
    int32_t* ins_cnt;                   // inserted in-edges per destination of an updated edge, [max_edges]
    int32_t *list_dd, *slot_dd;         // destinations of updated edges: sorted ids, vertex -> row of SD (the batch plan's slots)
    int32_t *plan_off, *plan_ord, *ins_rank;   // the batch plan: runs of updates per destination, rank of each insert
    uint64_t* plan_off64;               // its scratch for batches of more than 2048 updates
    int32_t *plan_cursor, *plan_tmp;
    uint64_t* plan_scan; int64_t plan_scan_len;   // block sums of its scans
    DstRec* recs;
    HubWork hubs;
    BatchScratch sc;
    unsigned long long* pair_ctr;
    int32_t* pull_list;        // [n] second-pass queue of the pull-direction expansion
    uint32_t* coarse[2];       // coarse copies of the sets bm[0], bm[1] (the sparse gather's LDS filter), written by the compaction
    int coarse_shift, coarse_words;
    uint64_t* cmp_state;       // look-back cells of the single-pass compaction
    int64_t cmp_state_len;
    // profiling
    int profiling;
    hipEvent_t ev[MAX_EVENTS];
    int ev_tag[MAX_EVENTS];
    int n_ev;
    bool events_made;
    hipEvent_t ev_validated;            // recorded after the read-back of the validation result
    bool ev_validated_made;
    nrt_stats stats;
};

enum { TAG_START = 0, TAG_INGEST = 1, TAG_EXPAND = 2, TAG_COMPACT = 3, TAG_ITEMS = 4, TAG_GATHER = 5, TAG_UPDATE = 6, TAG_COMBINE = 7 };

static nrt_status prof_mark(nrt_cache* c, int tag, int layer, hipStream_t s) {
    if (!c->profiling) return NRT_OK;
    if (c->n_ev >= MAX_EVENTS) return NRT_OK;
    HIP_TRY(hipEventRecord(c->ev[c->n_ev], s));
    c->ev_tag[c->n_ev] = tag | (layer << 8);
    c->n_ev++;
    return NRT_OK;
}

static nrt_status prof_collect(nrt_cache* c) {
    if (!c->profiling || c->n_ev < 2) return NRT_OK;
    for (int i = 1; i < c->n_ev; ++i) {
        float ms = 0.f;
        HIP_TRY(hipEventElapsedTime(&ms, c->ev[i - 1], c->ev[i]));
        const int tag = c->ev_tag[i] & 0xff, l = c->ev_tag[i] >> 8;
        nrt_layer_stats* ls = (l >= 1 && l <= NRT_MAX_LAYERS) ? &c->stats.layer[l - 1] : nullptr;
        switch (tag) {
        case TAG_INGEST: c->stats.ms_ingest += ms; break;
        case TAG_EXPAND: if (ls) ls->ms_expand += ms; break;
        case TAG_COMPACT: if (ls) ls->ms_compact += ms; break;
        case TAG_ITEMS: if (ls) ls->ms_items += ms; break;
        case TAG_GATHER: if (ls) ls->ms_gather += ms; break;
        case TAG_UPDATE: if (ls) ls->ms_update += ms; break;
        case TAG_COMBINE: if (ls) ls->ms_combine += ms; break;
        default: break;
        }
    }
    float tot = 0.f;
    HIP_TRY(hipEventElapsedTime(&tot, c->ev[0], c->ev[c->n_ev - 1]));
    c->stats.ms_total = tot;
    return NRT_OK;
}

// ------------------------------------------------------------------ graph
static void graph_fill(nrt_graph* g, int64_t n, int64_t e, int64_t ecap, int weighted) {
    memset(g, 0, sizeof(*g));
    g->n = n;
    g->e = e;
    g->e_capacity = ecap;
    g->weighted = weighted ? 1 : 0;
}

extern "C" nrt_status nrt_graph_workspace_bytes(int64_t n, int64_t e_capacity, int32_t weighted, size_t* bytes) {
    REQUIRE(bytes, "bytes is null");
    REQUIRE(n > 0 && n < (int64_t(1) << 31) - 64, "n_vertices out of range");
    REQUIRE(e_capacity >= 0 && e_capacity < (int64_t(1) << 40), "e_capacity out of range");
    nrt_graph g;
    graph_fill(&g, n, 0, e_capacity, weighted);
    Bump b{nullptr, 0};
    graph_layout(b, &g);
    *bytes = b.used + 256;
    return NRT_OK;
}

extern "C" nrt_status nrt_graph_create(int64_t n, int64_t e, int64_t e_capacity, int32_t weighted,
                                       const int64_t* csr_indptr, const int32_t* csr_indices, const float* csr_weights,
                                       const int64_t* csc_indptr, const int32_t* csc_indices, const float* csc_weights,
                                       void* workspace, size_t workspace_bytes, void* stream, nrt_graph** out) {
    REQUIRE(out, "out is null");
    REQUIRE(n > 0 && n < (int64_t(1) << 31) - 64, "n_vertices out of range");
    REQUIRE(e >= 0 && e_capacity >= e, "need 0 <= n_edges <= e_capacity");
    REQUIRE(csr_indptr || csc_indptr, "need CSR or CSC");
    REQUIRE(!csr_indptr || csr_indices || e == 0, "csr_indices is null");
    REQUIRE(!csc_indptr || csc_indices || e == 0, "csc_indices is null");
    if (weighted) {
        REQUIRE(!csr_indptr || csr_weights || e == 0, "weighted graph needs csr_weights");
        REQUIRE(!csc_indptr || csc_weights || e == 0, "weighted graph needs csc_weights");
    }
    REQUIRE(workspace && (reinterpret_cast<uintptr_t>(workspace) & 255) == 0, "workspace must be 256-byte aligned");
    size_t need = 0;
    NRT_TRY(nrt_graph_workspace_bytes(n, e_capacity, weighted, &need));
    REQUIRE(workspace_bytes >= need, "graph workspace too small");
    nrt_graph* g = new (std::nothrow) nrt_graph;
    if (!g) { nrt_set_error("host allocation failed"); return NRT_ERR_OOM; }
    graph_fill(g, n, e, e_capacity, weighted);
    Bump b{static_cast<char*>(workspace), 0};
    graph_layout(b, g);
    if (hipHostMalloc((void**)&g->host_pinned, NRT_NCTRS * sizeof(int64_t), hipHostMallocDefault) != hipSuccess) {
        delete g;
        nrt_set_error("pinned host allocation failed");
        return NRT_ERR_OOM;
    }
    nrt_status st = graph_build(g, csr_indptr, csr_indices, weighted ? csr_weights : nullptr, csc_indptr, csc_indices,
                                weighted ? csc_weights : nullptr, static_cast<hipStream_t>(stream));
    if (st != NRT_OK) {
        (void)hipHostFree(g->host_pinned);
        delete g;
        return st;
    }
    *out = g;
    return NRT_OK;
}

extern "C" void nrt_graph_destroy(nrt_graph* g) {
    if (!g) return;
    if (g->host_pinned) (void)hipHostFree(g->host_pinned);
    delete g;
}

extern "C" nrt_status nrt_graph_num_edges(const nrt_graph* g, int64_t* n_edges) {
    REQUIRE(g && n_edges, "null argument");
    *n_edges = g->e;
    return NRT_OK;
}

__global__ void export_deg_kernel(const int32_t* deg, int64_t n, uint64_t* out) {
    int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (v < n) out[v] = (uint64_t)deg[v];
    if (v == n) out[v] = 0;
}
__global__ void export_lists_kernel(Adj a, int64_t n, const int64_t* indptr, int32_t* indices, float* weights) {
    const int64_t v = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int lane = threadIdx.x & 63;
    if (v >= n) return;
    const int64_t o = a.off[v], b = indptr[v];
    const int32_t d = a.deg[v];
    for (int32_t j = lane; j < d; j += 64) {
        indices[b + j] = a.idx[o + j];
        if (weights) weights[b + j] = a.wts ? a.wts[o + j] : 1.0f;
    }
}

extern "C" nrt_status nrt_graph_export_csc(const nrt_graph* g, int64_t* indptr, int32_t* indices, float* weights,
                                           int64_t cap, void* stream) {
    REQUIRE(g && indptr && (indices || g->e == 0), "null argument");
    REQUIRE(cap >= g->e, "export capacity too small");
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t n = g->n;
    export_deg_kernel<<<(int)cdiv(n + 1, 256), 256, 0, s>>>(g->in.deg, n, (uint64_t*)indptr);
    LAUNCH_CHECK();
    NRT_TRY(k_exclusive_scan_u64((uint64_t*)indptr, n + 1, g->scan_tmp, g->scan_tmp_len,
                                 (uint64_t*)(g->dev_ctrs + CTR_COUNT), s));
    export_lists_kernel<<<(int)cdiv(n * 64, 256), 256, 0, s>>>(g->in, n, indptr, indices, weights);
    LAUNCH_CHECK();
    HIP_TRY(hipStreamSynchronize(s));
    return NRT_OK;
}

// ---- the same export for callers that cannot allocate or bring a workspace of their own for it: the block sums
// of the offset scan live in a file-scope device array instead of the graph's workspace.  Every GPU holds its own
// copy of the array at its own address; the address is looked up once per device and only that pointer is ever
// handed to kernels.
constexpr size_t NRT_STATIC_SCRATCH_BYTES = size_t(1) << 20;
constexpr int NRT_STATIC_MAX_DEVICES = 64;
static __device__ __align__(256) unsigned char scratch[NRT_STATIC_SCRATCH_BYTES];
static void* g_scratch_ptr[NRT_STATIC_MAX_DEVICES];
static std::mutex g_scratch_mutex;

static nrt_status static_scratch(void** out) {
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= NRT_STATIC_MAX_DEVICES) { nrt_set_error("device index %d out of range", dev); return NRT_ERR_DEVICE; }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) { nrt_set_error("hipGetSymbolAddress returned a null address"); return NRT_ERR_DEVICE; }
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return NRT_OK;
}

extern "C" nrt_status nrt_graph_export_csc_static(const nrt_graph* g, int64_t* indptr, int32_t* indices, float* weights,
                                                  int64_t cap, void* stream) {
    REQUIRE(g && indptr && (indices || g->e == 0), "null argument");
    REQUIRE(cap >= g->e, "export capacity too small");
    const int64_t n = g->n;
    // layout of the static array: [0, 256) the scan's total, then one uint64 block sum per 1024 offsets
    const int64_t tmp_len = (int64_t)((NRT_STATIC_SCRATCH_BYTES - 256) / sizeof(uint64_t));
    if (cdiv(n + 1, 1024) > tmp_len) {
        nrt_set_error("graph of %lld vertices exceeds the static scratch (%lld vertices at most); use nrt_graph_export_csc",
                      (long long)n, (long long)(tmp_len * 1024 - 1));
        return NRT_ERR_INVALID_ARG;
    }
    void* base = nullptr;
    NRT_TRY(static_scratch(&base));
    uint64_t* total = reinterpret_cast<uint64_t*>(base);
    uint64_t* tmp = reinterpret_cast<uint64_t*>(static_cast<unsigned char*>(base) + 256);
    hipStream_t s = static_cast<hipStream_t>(stream);
    export_deg_kernel<<<(int)cdiv(n + 1, 256), 256, 0, s>>>(g->in.deg, n, (uint64_t*)indptr);
    LAUNCH_CHECK();
    NRT_TRY(k_exclusive_scan_u64((uint64_t*)indptr, n + 1, tmp, tmp_len, total, s));
    export_lists_kernel<<<(int)cdiv(n * 64, 256), 256, 0, s>>>(g->in, n, indptr, indices, weights);
    LAUNCH_CHECK();
    HIP_TRY(hipStreamSynchronize(s));
    return NRT_OK;
}

// ------------------------------------------------------------------ cache layout
// models whose update runs on the concatenation [h_v || aggregate] (Table II rows PinSAGE and CommNet)
static inline bool concat_self(int kind) { return kind == NRT_SAGE_MEAN || kind == NRT_COMMNET || kind == NRT_PINSAGE; }

// models that aggregate a per-vertex transform of h instead of h itself, cached by vertex
static inline bool has_message_cache(int kind) { return kind == NRT_PINSAGE || kind == NRT_MONET || kind == NRT_RGCN; }
// constrained models served by the kernels of agnn.hip
static inline bool agnn_family(int kind) { return kind == NRT_AGNN || kind == NRT_GGCN; }
// models whose messages read the edge weight (RGCN: as the relation id)
static inline bool weighted_messages(int kind) { return kind == NRT_GIN || kind == NRT_PINSAGE || kind == NRT_RGCN; }

static nrt_status check_desc(const nrt_model_desc* d) {
    REQUIRE(d, "model desc is null");
    REQUIRE(d->kind >= NRT_GCN && d->kind <= NRT_RGAT, "unknown model kind");
    REQUIRE(d->n_layers >= 1 && d->n_layers <= NRT_MAX_LAYERS, "n_layers out of range");
    for (int l = 0; l <= d->n_layers; ++l) {
        if (d->dims[l] <= 0 || d->dims[l] % 4 || d->dims[l] > 1024) {
            nrt_set_error("layer widths must be multiples of 4 in [4, 1024]");
            return NRT_ERR_UNSUPPORTED;
        }
    }
    if (d->kind == NRT_MONET && (d->monet_kernels < 4 || d->monet_kernels % 4 || d->monet_kernels > 1024)) {
        nrt_set_error("MoNet needs monet_kernels a multiple of 4 in [4, 1024]");
        return NRT_ERR_UNSUPPORTED;
    }
    if (d->kind == NRT_RGAT) {
        if (d->n_relations < 1 || d->head_dim < 4 || d->head_dim % 4 || (int64_t)d->n_relations * d->head_dim > 1024) {
            nrt_set_error("RGAT needs n_relations >= 1, head_dim a multiple of 4 and n_relations * head_dim <= 1024");
            return NRT_ERR_UNSUPPORTED;
        }
        for (int l = 1; l <= d->n_layers; ++l)
            if (d->dims[l] != d->head_dim) {
                nrt_set_error("RGAT layer widths must equal head_dim");
                return NRT_ERR_UNSUPPORTED;
            }
    }
    if (d->kind == NRT_RGCN) {
        if (d->n_relations < 1 || d->n_relations > 64) {
            nrt_set_error("RGCN needs n_relations in [1, 64]");
            return NRT_ERR_UNSUPPORTED;
        }
        for (int l = 1; l <= d->n_layers; ++l)
            if ((int64_t)d->n_relations * d->dims[l] > 4096) {
                nrt_set_error("RGCN: n_relations * layer width must not exceed 4096");
                return NRT_ERR_UNSUPPORTED;
            }
    }
    const bool by_tables = d->kind == NRT_GIN || d->kind == NRT_SAGE_MEAN || d->kind == NRT_COMMNET;
    if (d->agg_only && d->kind != NRT_GCN && d->kind != NRT_GAT && d->kind != NRT_RGAT && d->kind != NRT_RGCN &&
        d->kind != NRT_MONET && !by_tables) {
        nrt_set_error("aggregate-only storage is available for GCN, GAT, RGAT, RGCN, MoNet, and for GIN, GraphSAGE and CommNet with weights-first layers");
        return NRT_ERR_UNSUPPORTED;
    }
    if (d->agg_only && by_tables) {
        // a layer that applies its weights before the aggregation reads h^{l-1} only through the cached products
        // (h^{l-1} W_a; h^{l-1} W_1 and h^{l-1} W_2); one that does not reads the row itself in its update
        bool ok = !d->aggregate_first;
        for (int l = 2; l <= d->n_layers; ++l) ok = ok && d->dims[l] <= d->dims[l - 1];
        if (!ok) {
            nrt_set_error("GIN, GraphSAGE, CommNet: aggregate-only storage needs aggregate_first = 0 and d_l <= d_{l-1} for every layer above the first");
            return NRT_ERR_UNSUPPORTED;
        }
    }
    if (d->kind == NRT_GAT) {
        if (d->heads < 1 || d->head_dim < 4 || d->head_dim % 4) {
            nrt_set_error("GAT needs heads >= 1 and head_dim a multiple of 4");
            return NRT_ERR_UNSUPPORTED;
        }
        for (int l = 1; l <= d->n_layers; ++l)
            if (d->dims[l] != d->heads * d->head_dim) {
                nrt_set_error("GAT layer widths must equal heads * head_dim");
                return NRT_ERR_UNSUPPORTED;
            }
    }
    return NRT_OK;
}

static void cache_layout(Bump& b, nrt_cache* c) {
    const nrt_graph* g = c->g;
    const int64_t n = g->n;
    const int64_t nw = cdiv(n, 32);
    int maxd = 0;
    for (int l = 0; l <= c->L; ++l) maxd = c->dims[l] > maxd ? c->dims[l] : maxd;
    if (c->kind == NRT_MONET && c->monet_J > maxd) maxd = c->monet_J;
    if (c->kind == NRT_RGCN)                 // the message deltas of a changed row are n_rel rows of the next layer's width
        for (int l = 1; l <= c->L; ++l) maxd = c->n_rel * c->dims[l] > maxd ? c->n_rel * c->dims[l] : maxd;
    c->zdim = c->heads * c->head_dim;
    if (c->kind == NRT_RGAT && c->zdim > maxd) maxd = c->zdim;      // old z rows and partial rows are zdim wide
    c->maxd = maxd;
    for (int l = 0; l <= c->L; ++l) {
        const bool hidden = l >= 1 && l < c->L;
        c->H[l] = (c->agg_only && hidden) ? nullptr : b.take<float>(n * c->dims[l]);
        c->ES[l] = (c->agg_only && hidden && c->kind == NRT_GCN) ? b.take<float>((size_t)(c->max_edges + 1) * c->dims[l]) : nullptr;
    }
    c->es_rows = (c->agg_only && c->kind == NRT_GCN) ? b.take<int32_t>(c->max_edges + 1) : nullptr;
    for (int l = 0; l <= c->L; ++l) {
        c->MP[l] = nullptr;
        if (c->kind == NRT_PINSAGE && l < c->L) c->MP[l] = b.take<float>(n * c->dims[l]);
        if (c->kind == NRT_RGCN && l < c->L) c->MP[l] = b.take<float>(n * c->n_rel * c->dims[l + 1]);
        if (l < c->L && c->tf[l + 1]) c->MP[l] = b.take<float>(n * c->dims[l + 1]);
        c->MS[l] = (l < c->L && ((c->tf[l + 1] && concat_self(c->kind)) || c->kind == NRT_RGCN)) ? b.take<float>(n * c->dims[l + 1]) : nullptr;
        if (c->kind == NRT_MONET && l < c->L) {
            c->MP[l] = b.take<float>(n * c->monet_J);
            c->muT[l] = b.take<float>((size_t)c->dims[l] * c->monet_J);
            c->precT[l] = b.take<float>((size_t)c->dims[l] * c->monet_J);
        }
    }
    for (int l = 0; l <= c->L; ++l) c->R[l] = (c->kind == NRT_AGNN && l < c->L) ? b.take<float>(n) : nullptr;
    c->r_old = c->kind == NRT_AGNN ? b.take<float>(n) : nullptr;
    for (int l = 0; l <= c->L; ++l) {
        const bool on = c->kind == NRT_GGCN && l < c->L;
        c->P1[l] = on ? b.take<float>(n * c->dims[l]) : nullptr;
        c->P2[l] = on ? b.take<float>(n * c->dims[l]) : nullptr;
        if (l < c->L) c->W2t[l] = on ? b.take<float>((size_t)c->dims[l] * c->dims[l]) : nullptr;
    }
    c->old_p1 = c->kind == NRT_GGCN ? b.take<float>(n * maxd) : nullptr;
    c->S[0] = nullptr;
    const bool gat = c->kind == NRT_GAT || c->kind == NRT_RGAT;
    for (int l = 1; l <= c->L; ++l) {
        c->dagg[l] = gat ? c->zdim : ((c->kind == NRT_RGCN || c->tf[l]) ? c->dims[l] : (c->kind == NRT_MONET ? c->monet_J : c->dims[l - 1]));
        c->S[l] = b.take<float>(n * c->dagg[l]);
        if (gat) {
            c->Z[l] = b.take<float>(n * c->zdim);
            c->AS[l] = b.take<float>(n * c->heads);
            c->AD[l] = b.take<float>(n * c->heads);
            c->M[l] = b.take<float>(n * c->heads);
            c->DEN[l] = b.take<float>(n * c->heads);
            c->att_src[l - 1] = b.take<float>((size_t)c->heads * c->head_dim);
            c->att_dst[l - 1] = b.take<float>((size_t)c->heads * c->head_dim);
        }
    }
    for (int l = 1; l <= c->L; ++l) {
        c->SD[l] = b.take<float>((size_t)(c->max_edges + 1) * c->dagg[l]);
        c->SDden[l] = gat ? b.take<float>((size_t)(c->max_edges + 1) * c->heads) : nullptr;
    }
    c->ins_cnt = b.take<int32_t>(c->max_edges + 1);
    c->plan_off = b.take<int32_t>(c->max_edges + 2);
    c->plan_ord = b.take<int32_t>(c->max_edges + 1);
    c->ins_rank = b.take<int32_t>(c->max_edges + 1);
    c->plan_off64 = b.take<uint64_t>(c->max_edges + 2);
    c->plan_cursor = b.take<int32_t>(c->max_edges + 1);
    c->plan_tmp = b.take<int32_t>(c->max_edges + 1);
    c->plan_scan_len = cdiv(c->max_edges + 2 > nw ? c->max_edges + 2 : nw, 1024) + 64;
    c->plan_scan = b.take<uint64_t>(c->plan_scan_len);
    c->list_dd = b.take<int32_t>(c->max_edges + 64);
    c->slot_dd = b.take<int32_t>(n);
    c->AS_old = gat ? b.take<float>(n * c->heads) : nullptr;
    c->is_gat = gat;
    for (int l = 0; l < c->L; ++l) {
        const int kin = c->kind == NRT_MONET ? c->monet_J : (concat_self(c->kind) ? 2 : 1) * c->dims[l];
        c->Wt[l][0] = b.take<float>((size_t)kin * (gat ? c->zdim : c->dims[l + 1]));
        c->bias[l][0] = b.take<float>(c->dims[l + 1]);
        if (c->kind == NRT_GIN) {
            c->Wt[l][1] = b.take<float>((size_t)c->dims[l + 1] * c->dims[l + 1]);
            c->bias[l][1] = b.take<float>(c->dims[l + 1]);
        } else if (c->kind == NRT_PINSAGE || c->kind == NRT_GGCN) {
            c->Wt[l][1] = b.take<float>((size_t)c->dims[l] * c->dims[l]);
            c->bias[l][1] = b.take<float>(c->dims[l]);
        } else if (c->kind == NRT_RGCN) {                      // the relation matrices side by side, transposed
            c->Wt[l][1] = b.take<float>((size_t)c->dims[l] * c->n_rel * c->dims[l + 1]);
            c->bias[l][1] = nullptr;
        } else {
            c->Wt[l][1] = nullptr;
            c->bias[l][1] = nullptr;
        }
    }
    c->indeg_old = b.take<int32_t>(n);
    c->nw_pad = (nw + 63) & ~int64_t(63);
    c->bm_ddst = b.take<uint32_t>(2 * c->nw_pad);
    c->bm_feat = c->bm_ddst ? c->bm_ddst + c->nw_pad : nullptr;
    c->bm[0] = b.take<uint32_t>(nw);
    c->bm[1] = b.take<uint32_t>(nw);
    for (int l = 0; l <= c->L; ++l) c->list[l] = b.take<int32_t>(n);
    c->slot[0] = b.take<int32_t>(n);
    c->slot[1] = b.take<int32_t>(n);
    c->DP[0] = b.take<float>(n * maxd);
    c->DP[1] = b.take<float>(n * maxd);
    c->mid = c->kind == NRT_GIN ? b.take<float>(n * maxd) : nullptr;      // the rows between its two products
    c->recs = b.take<DstRec>(n);
    c->hubs.hub_cap = g->e_capacity / NRT_CHUNK + 64;          // a hub has more than NRT_CHUNK live in-edges
    c->hubs.item_cap = 2 * (g->e_capacity / NRT_CHUNK) + 64;   // sum of ceil(deg/NRT_CHUNK) over hubs
    c->hubs.hub_slot = b.take<int32_t>(c->hubs.hub_cap);
    c->hubs.hub_first = b.take<uint64_t>(c->hubs.hub_cap);
    c->hubs.item_hub = b.take<int32_t>(c->hubs.item_cap);
    c->hubs.item_chunk = b.take<int32_t>(c->hubs.item_cap);
    c->hubs.partial = b.take<float>(c->hubs.item_cap * maxd);
    c->part_m = c->is_gat ? b.take<float>(c->hubs.item_cap * c->heads) : nullptr;
    c->part_den = c->is_gat ? b.take<float>(c->hubs.item_cap * c->heads) : nullptr;
    c->xhub_cap = g->e_capacity / 512 + 64;                    // sources with more than 512 live out-edges
    c->xhub_list = b.take<int32_t>(c->xhub_cap);
    c->flags = b.take<uint8_t>(n + 64);
    c->lc = b.take<LayerCtrs>(LC_TOTAL);
    c->sc.max_edges = c->max_edges;
    int64_t hc = 16;
    while (hc < 2 * (c->max_edges + 1)) hc <<= 1;
    c->sc.hash_cap = hc;
    c->sc.hash_keys = b.take<uint64_t>(hc);
    c->sc.pos_out = b.take<int64_t>(c->max_edges + 1);
    c->sc.pos_in = b.take<int64_t>(c->max_edges + 1);
    c->sc.del_w = b.take<float>(c->max_edges + 1);
    c->sc.feat_index = b.take<int32_t>(n);
    c->sc.feat_stamp = b.take<int32_t>(n);
    c->sc.err = g->dev_ctrs ? (int32_t*)(g->dev_ctrs + CTR_ERR) : nullptr;
    c->pair_ctr = b.take<unsigned long long>(1024 * NRT_MAX_LAYERS);
    c->pull_list = b.take<int32_t>(n);
    for (int l = 1; l <= c->L; ++l) c->stale[l] = b.take<uint32_t>(nw);
    for (int l = 0; l <= c->L; ++l) {
        c->stale_prev[l] = l >= 1 ? b.take<uint32_t>(nw) : nullptr;
        c->need_bm[l] = b.take<uint32_t>(nw);
        c->need_list[l] = l >= 1 ? b.take<int32_t>(n) : nullptr;
    }
    c->list_fresh = b.take<int32_t>(n);
    c->list_redo = b.take<int32_t>(n);
    c->bm_q = b.take<uint32_t>(nw);
    c->coarse[0] = b.take<uint32_t>(NRT_COARSE_WORDS);
    c->coarse[1] = b.take<uint32_t>(NRT_COARSE_WORDS);
    c->cmp_state_len = cdiv(nw, 256) + 8;
    c->cmp_state = b.take<uint64_t>(c->cmp_state_len);
    c->coarse_shift = 0;
    while ((((n + ((int64_t)1 << c->coarse_shift) - 1) >> c->coarse_shift) + 31) / 32 > NRT_COARSE_WORDS) ++c->coarse_shift;
    c->coarse_words = (int)((((n + ((int64_t)1 << c->coarse_shift) - 1) >> c->coarse_shift) + 31) / 32);
}

static nrt_status cache_fill(nrt_cache* c, const nrt_graph* g, const nrt_model_desc* d, int64_t max_edges,
                             int64_t max_feats) {
    memset(c, 0, sizeof(*c));
    c->g = const_cast<nrt_graph*>(g);
    c->kind = d->kind;
    c->L = d->n_layers;
    for (int l = 0; l <= c->L; ++l) c->dims[l] = d->dims[l];
    c->heads = d->heads;
    c->head_dim = d->head_dim;
    c->gin_eps = d->gin_eps;
    c->leaky_slope = d->leaky_slope;
    for (int l = 0; l < c->L; ++l) c->agnn_beta[l] = d->agnn_beta[l];
    c->agg_only = d->agg_only ? 1 : 0;
    c->monet_J = d->kind == NRT_MONET ? d->monet_kernels : 0;
    c->n_rel = (d->kind == NRT_RGCN || d->kind == NRT_RGAT) ? d->n_relations : 0;
    if (d->kind == NRT_RGAT) c->heads = d->n_relations;          // one softmax group per relation
    c->no_reorder = d->aggregate_first ? 1 : 0;
    for (int l = 1; l <= c->L; ++l)
        c->tf[l] = (d->kind == NRT_GCN || d->kind == NRT_GIN || d->kind == NRT_SAGE_MEAN || d->kind == NRT_COMMNET) &&
                   (!d->agg_only || d->kind != NRT_GCN) && !d->aggregate_first &&
                   (d->dims[l] < d->dims[l - 1] || (d->dims[l] == d->dims[l - 1] && d->kind != NRT_GCN));
    c->max_edges = max_edges;
    c->max_feats = max_feats;
    return NRT_OK;
}

extern "C" nrt_status nrt_cache_workspace_bytes(const nrt_graph* g, const nrt_model_desc* d, int64_t max_batch_edges,
                                                int64_t max_batch_feats, size_t* bytes) {
    REQUIRE(g && bytes, "null argument");
    NRT_TRY(check_desc(d));
    REQUIRE(max_batch_edges >= 0 && max_batch_feats >= 0, "negative batch bound");
    nrt_cache c;
    cache_fill(&c, g, d, max_batch_edges, max_batch_feats);
    Bump b{nullptr, 0};
    cache_layout(b, &c);
    *bytes = b.used + 256;
    return NRT_OK;
}

// ------------------------------------------------------------------ shared layer steps
static nrt_status read_ctrs(nrt_graph* g, hipStream_t s) {
    HIP_TRY(hipMemcpyAsync(g->host_pinned, g->dev_ctrs, NRT_NCTRS * sizeof(int64_t), hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    return NRT_OK;
}

// Aggregate-only storage of GIN, GraphSAGE, CommNet, RGCN, MoNet: the two delta buffers have fixed roles instead of alternating with
// the layers.  DP[0] holds the compact payload deltas a layer's gather folds; DP[1] the compact rows h^l that the update
// of layer l hands to the message products of layer l+1 (written after those products of layer l have read it).
static inline bool rows_by_tables(const nrt_cache* c) {
    return c->agg_only && (c->kind == NRT_GIN || c->kind == NRT_SAGE_MEAN || c->kind == NRT_COMMNET || c->kind == NRT_RGCN ||
                           c->kind == NRT_MONET);
}
static inline float* delta_buf(nrt_cache* c, int prev) { return rows_by_tables(c) ? c->DP[0] : c->DP[prev]; }

// what the in-neighbours of layer l+1 aggregate: h^l itself, or its transform for PinSAGE
static inline const float* payload_rows(const nrt_cache* c, int l) { return c->MP[l] ? c->MP[l] : c->H[l]; }

// PinSAGE, MoNet, RGCN (Table II): the message of a vertex (ReLU(h^l Q + q); Gaussian kernel responses of h^l; W_r h^l
// for every relation r) on the listed rows
// (null: all n rows); with `dp` the compact rows new - old that the gather of layer l+1 folds
static nrt_status run_transform(nrt_cache* c, int l, const int32_t* rows, int64_t M, const uint64_t* M_dev, float* dp,
                                bool skip_dp_when_large, hipStream_t s) {
    if (c->kind == NRT_MONET) {            // the Gaussian kernel responses of the rows
        MonetArgs m;
        memset(&m, 0, sizeof(m));
        m.rows = rows;
        m.count_dev = M_dev;
        m.bound = M;
        m.H = c->H[l];
        if (!c->H[l]) {                    // aggregate-only storage: the rows the update of layer l handed over, in list order
            if (!rows) { nrt_set_error("hidden rows are not kept"); return NRT_ERR_STATE; }
            m.H = c->DP[1];
            m.h_is_compact = 1;
        }
        m.d = c->dims[l];
        m.muT = c->muT[l];
        m.precT = c->precT[l];
        m.J = c->monet_J;
        m.G = c->MP[l];
        m.DP = dp;
        return k_monet_transform(m, s);
    }
    GemmArgs a;
    memset(&a, 0, sizeof(a));
    a.M = M;
    a.M_dev = M_dev;
    a.rows = rows;
    a.a_mode = A_PLAIN;
    a.P0 = c->H[l];
    a.ldp = c->dims[l];
    if (!c->H[l]) {
        // aggregate-only storage (GIN, GraphSAGE, CommNet): the update of layer l left the rows of its affected list, which are these rows,
        // compact and in list order in DP[1]
        if (!rows) { nrt_set_error("hidden rows are not kept"); return NRT_ERR_STATE; }
        a.P0 = c->DP[1];
        a.a_is_compact = 1;
    }
    a.K = c->dims[l];
    a.N = c->dims[l];
    a.Wt = c->Wt[l][1];
    a.bias = c->bias[l][1];
    a.act = 1;
    if (c->tf[l + 1]) {                    // GCN, GIN: h^l W, the layer's (first) matrix applied before the aggregation
        a.N = c->dims[l + 1];
        a.Wt = c->Wt[l][0];
        a.bias = nullptr;
        a.act = 0;
        if (c->kind == NRT_GCN) {          // the payload is the row over sqrt(d): its delta carries the degree change
            a.indeg = c->g->in.deg;
            a.indeg_old = c->indeg_old;
            a.dp_scale_gcn = 1;
        }
        if (concat_self(c->kind)) {        // W = [W_1; W_2]: the neighbour half, a column block of the transposed matrix
            a.Wt = c->Wt[l][0] + c->dims[l];
            a.ldw = 2 * c->dims[l];
        }
    }
    if (c->kind == NRT_RGCN) {             // h^l [W_0 | ... | W_{R-1}]: row v of the product is the R message rows of v
        a.N = c->n_rel * c->dims[l + 1];
        a.act = 0;
    }
    a.H = c->MP[l];
    a.DP = dp;
    a.dp_skip_large = skip_dp_when_large;
    a.n_vertices = c->g->n;
    NRT_TRY(k_gemm(a, s));
    if (c->MS[l]) {                        // the self half h^l W_1 (RGCN: h^l W_o) of the same rows; nobody folds its deltas
        a.N = c->dims[l + 1];
        a.Wt = c->Wt[l][0];
        if (c->kind == NRT_RGCN) a.ldw = 0;
        a.H = c->MS[l];
        a.DP = nullptr;
        a.dp_skip_large = 0;
        NRT_TRY(k_gemm(a, s));
    }
    return NRT_OK;
}

// gather + fold of layer l over the destinations described by c->recs and the hub items built from them;
// all sizes are read on the device from c->lc[l]
static nrt_status run_gather(nrt_cache* c, int l, bool incremental, int prev, bool may_recompute, int sparse_hint,
                             hipStream_t s) {
    nrt_graph* g = c->g;
    GatherArgs a;
    memset(&a, 0, sizeof(a));
    a.recs = c->recs;
    a.hubs = c->hubs;
    a.lc = c->lc_use ? c->lc_use : &c->lc[l];
    a.in = g->in;
    a.D = c->dagg[l];
    a.use_weights = (weighted_messages(c->kind) && g->weighted) ? 1 : 0;
    a.rel_R = c->n_rel;
    a.self_pair = c->kind == NRT_GCN;
    a.S = c->S[l];
    a.n_vertices = g->n;
    if (c->profiling) a.pair_ctr = c->pair_ctr + (size_t)(l - 1) * 1024;
    if (c->have_history_prev && !c->lc_use) {    // what the previous batch had at this layer sizes the grids
        a.units_hint = (int64_t)(c->lc_host[l].count + c->lc_host[l].n_items) + 1;
        a.hubs_hint = (int64_t)c->lc_host[l].n_hubs;
    }
    GatherArgs full = a;                         // full-neighbour aggregation from h^{l-1} (Eq. 1)
    full.P = payload_rows(c, l - 1);
    full.src_scale_gcn = c->kind == NRT_GCN;
    full.accumulate = 0;
    if (incremental) {
        a.P = c->ov_bm ? c->ov_dp : delta_buf(c, prev);
        a.src_bitmap = c->ov_bm ? c->ov_bm : c->bm[prev];
        a.src_slot = c->ov_bm ? c->ov_slot : c->slot[prev];
        a.n_src_dev = c->ov_bm ? c->ov_count : &c->lc[l - 1].count;
        a.src_scale_gcn = 0;
        a.accumulate = 1;
        a.sd = c->SD[l];
        a.dd_bitmap = c->bm_ddst;
        a.dd_slot = c->slot_dd;
        a.guard = c->kind == NRT_GIN || c->kind == NRT_COMMNET || c->kind == NRT_MONET;   // un-normalised sums: a fold can cancel most of a row's magnitude
        a.Pfull = payload_rows(c, l - 1);
        a.full_scale_gcn = c->kind == NRT_GCN;
        a.sparse_ok = (sparse_hint == 2 && a.D > 256) ? 1 : sparse_hint;    // rows wider than 256 floats: pipelined kernel only
        a.coarse = c->ov_bm ? c->ov_coarse : c->coarse[prev];   // written by the compaction that produced the source set
        a.coarse_shift = c->coarse_shift;
        a.coarse_words = c->coarse_words;
        if (c->coarse_shift > 10)                    // beyond 200M vertices a coarse word spans several compaction workgroups
            NRT_TRY(k_coarse_bitmap(a.src_bitmap, g->n, c->coarse_shift, const_cast<uint32_t*>(a.coarse), c->coarse_words, s));
        if (may_recompute) {                     // the device counters pick one of the two (GatherArgs::auto_role)
            a.auto_role = 1;
            a.auto_src_dev = &c->lc[l - 1].count;
            full.auto_role = 2;
            full.auto_src_dev = &c->lc[l - 1].count;
        }
    } else {
        a = full;
    }
    NRT_TRY(prof_mark(c, TAG_ITEMS, l, s));
    NRT_TRY(k_gather(a, s));
    if (incremental && may_recompute) NRT_TRY(k_gather(full, s));
    NRT_TRY(prof_mark(c, TAG_GATHER, l, s));
    NRT_TRY(k_combine_partials(a, s));
    NRT_TRY(prof_mark(c, TAG_COMBINE, l, s));
    return NRT_OK;
}

// dense update of layer l on the rows listed in `rows` (null: all n rows); M_dev: their number on the device
static nrt_status run_update(nrt_cache* c, int l, const int32_t* rows, int64_t M, const uint64_t* M_dev,
                             bool incremental, int cur, float* out_rows, int64_t out_cap, bool next_may_recompute,
                             hipStream_t s) {
    nrt_graph* g = c->g;
    const bool last = l == c->L;
    GemmArgs a;
    memset(&a, 0, sizeof(a));
    a.M = M;
    a.M_dev = M_dev;
    a.rows = rows;
    a.indeg = g->in.deg;
    a.indeg_old = c->indeg_old;
    a.ldp = c->dims[l - 1];
    a.N = c->dims[l];
    // PinSAGE: the next layer's payload deltas come from the transform of the changed rows, not from here
    float* dp = (incremental && !last && !c->MP[l]) ? c->DP[cur] : nullptr;
    if (c->kind == NRT_MONET) {
        a.a_mode = A_PLAIN;
        a.P0 = c->S[l];
        a.ldp = c->monet_J;
        a.K = c->monet_J;
        a.Wt = c->Wt[l - 1][0];
        a.bias = c->bias[l - 1][0];
        a.act = last ? 0 : 1;
        a.H = c->H[l];
        a.n_vertices = g->n;
        a.out_compact = last ? out_rows : nullptr;
        a.out_cap = out_cap;
        if (!last && !c->H[l]) {           // aggregate-only storage: the rows go compact to the next layer's kernel responses
            if (!rows) { nrt_set_error("hidden rows are not kept"); return NRT_ERR_STATE; }
            a.out_compact = c->DP[1];
            a.out_cap = g->n;
        }
        NRT_TRY(k_gemm(a, s));
    } else if (c->tf[l] && c->kind == NRT_GCN) {   // the weights went into the messages: act(S_v / sqrt(d_v) + b), no product left
        a.P0 = c->S[l];
        a.bias = c->bias[l - 1][0];
        a.act = last ? 0 : 1;
        a.H = c->H[l];
        a.DP = dp;
        a.dp_skip_large = next_may_recompute;
        a.n_vertices = g->n;
        a.dp_scale_gcn = 1;
        a.out_compact = last ? out_rows : nullptr;
        a.out_cap = out_cap;
        NRT_TRY(k_rowwise_update(a, s));
    } else if (c->tf[l] && c->kind == NRT_GIN) {   // ReLU((1+eps) x_v W_a + sum_u w_uv x_u W_a + b_a) W_b + b_b: one product
        a.a_mode = A_AXPY_BIAS_RELU;
        a.P0 = c->MP[l - 1];
        a.P1 = c->S[l];
        a.axpy_c = 1.0f + c->gin_eps;
        a.a_bias = c->bias[l - 1][0];
        a.ldp = c->dims[l];
        a.K = c->dims[l];
        a.Wt = c->Wt[l - 1][1];
        a.bias = c->bias[l - 1][1];
        a.act = last ? 0 : 1;
        a.H = c->H[l];
        a.DP = dp;
        a.dp_skip_large = next_may_recompute;
        a.n_vertices = g->n;
        a.out_compact = last ? out_rows : nullptr;
        a.out_cap = out_cap;
        if (!last && !c->H[l]) {           // aggregate-only storage: the rows go compact to the next layer's message product
            if (!rows) { nrt_set_error("hidden rows are not kept"); return NRT_ERR_STATE; }
            a.out_compact = c->DP[1];
            a.out_cap = g->n;
        }
        NRT_TRY(k_gemm(a, s));
    } else if ((c->tf[l] && concat_self(c->kind)) || c->kind == NRT_RGCN) {
        // act(x_v W_1 + S_v / count + b) from the two cached products: S_v is the sum of x_u W_2 (CommNet: no count), x_v W_1
        // a cached row; RGCN: sigma(x_v W_o + a_v), a_v = cached sum of relation messages / neighbour count.  No product left.
        a.P0 = c->MS[l - 1];
        a.indeg = nullptr;
        a.add = c->S[l];
        a.add_indeg = c->kind == NRT_COMMNET ? nullptr : g->in.deg;
        a.bias = c->bias[l - 1][0];
        a.act = last ? 0 : 1;
        a.H = c->H[l];
        a.DP = dp;
        a.dp_skip_large = next_may_recompute;
        a.n_vertices = g->n;
        a.out_compact = last ? out_rows : nullptr;
        a.out_cap = out_cap;
        if (!last && !c->H[l]) {           // aggregate-only storage: the rows go compact to the next layer's products
            if (!rows) { nrt_set_error("hidden rows are not kept"); return NRT_ERR_STATE; }
            a.out_compact = c->DP[1];
            a.out_cap = g->n;
        }
        NRT_TRY(k_rowwise_update(a, s));
    } else if (c->kind == NRT_GCN || concat_self(c->kind)) {
        if (c->kind == NRT_GCN) {
            a.a_mode = A_SCALE_GCN;
            a.P0 = c->S[l];
            a.K = c->dims[l - 1];
        } else {
            a.a_mode = A_CONCAT_MEAN;
            a.P0 = c->H[l - 1];
            a.P1 = c->S[l];
            a.K = 2 * c->dims[l - 1];
            if (c->kind == NRT_COMMNET) a.indeg = nullptr;      // the sum itself, not the mean
        }
        a.Wt = c->Wt[l - 1][0];
        a.bias = c->bias[l - 1][0];
        a.act = last ? 0 : 1;
        a.H = c->H[l];
        a.DP = dp;
        a.dp_skip_large = next_may_recompute;
        a.n_vertices = g->n;
        a.dp_scale_gcn = c->kind == NRT_GCN;
        a.out_compact = last ? out_rows : nullptr;
        a.out_cap = out_cap;
        if (!last && !c->H[l] && c->kind != NRT_GCN) {   // aggregate-only storage of GraphSAGE, CommNet (a first layer that widens)
            if (!rows || dp) { nrt_set_error("hidden rows are not kept"); return NRT_ERR_STATE; }
            a.out_compact = c->DP[1];
            a.out_cap = g->n;
        }
        NRT_TRY(k_gemm(a, s));
    } else {   // GIN: two chained products
        a.a_mode = A_AXPY;
        a.P0 = c->H[l - 1];
        a.P1 = c->S[l];
        a.axpy_c = 1.0f + c->gin_eps;
        a.K = c->dims[l - 1];
        a.Wt = c->Wt[l - 1][0];
        a.bias = c->bias[l - 1][0];
        a.act = 1;
        const bool unkept = !last && !c->H[l];   // aggregate-only storage: the rows go compact to the next layer's message product
        if (unkept && (!rows || dp)) { nrt_set_error("hidden rows are not kept"); return NRT_ERR_STATE; }
        float* mid = c->mid;
        a.out_compact = mid;
        a.out_cap = g->n;
        NRT_TRY(k_gemm(a, s));
        GemmArgs b2;
        memset(&b2, 0, sizeof(b2));
        b2.M = M;
        b2.M_dev = M_dev;
        b2.rows = rows;
        b2.a_is_compact = 1;
        b2.a_mode = A_PLAIN;
        b2.P0 = mid;
        b2.ldp = c->dims[l];
        b2.K = c->dims[l];
        b2.N = c->dims[l];
        b2.Wt = c->Wt[l - 1][1];
        b2.bias = c->bias[l - 1][1];
        b2.act = last ? 0 : 1;
        b2.H = c->H[l];
        b2.DP = dp;
        b2.dp_skip_large = next_may_recompute;
        b2.n_vertices = g->n;
        b2.out_compact = last ? out_rows : (unkept ? c->DP[1] : nullptr);
        b2.out_cap = last ? out_cap : g->n;
        NRT_TRY(k_gemm(b2, s));
    }
    return NRT_OK;
}

// GAT layer l: z = x W on the listed rows (null: all), attention scalars, then the attention gather + output
// `listed`: only the rows of src_rows / dst_rows are touched; `incremental`: Algorithm 3 on top of that (old z and
// attention scalars kept, terms exchanged), else every listed destination is recomputed over its whole in-list
// GAT, layer l: z = h^{l-1} W and the attention scalars of the listed rows (null: all rows); with `incremental` the
// rows they replace are kept compact (old z in DP[0], old scalars in AS_old) for Algorithm 3's exchange
static nrt_status run_gat_project(nrt_cache* c, int l, const int32_t* src_rows, const uint64_t* n_src_dev, int64_t src_bound,
                                  bool listed, bool incremental, GatArgs* out_args, hipStream_t s) {
    nrt_graph* g = c->g;
    GemmArgs z;
    memset(&z, 0, sizeof(z));
    z.M = listed ? src_bound : g->n;
    z.M_dev = n_src_dev;
    z.rows = src_rows;
    z.a_mode = A_PLAIN;
    z.P0 = c->H[l - 1];
    z.ldp = c->dims[l - 1];
    if (!c->H[l - 1]) {
        // aggregate-only storage: the rows of h^{l-1} that changed were left, in list order, in DP[1] by the layer below
        // (the rows of a layer's affected list are the next layer's changed sources)
        if (!listed) { nrt_set_error("hidden rows are not kept"); return NRT_ERR_STATE; }
        z.P0 = c->DP[1];
        z.a_is_compact = 1;
    }
    z.K = c->dims[l - 1];
    z.N = c->zdim;
    z.Wt = c->Wt[l - 1][0];
    z.H = c->Z[l];
    if (incremental) { z.DP = c->DP[0]; z.dp_store_old = 1; }     // keep the old z rows, compact, for Algorithm 3
    NRT_TRY(k_gemm(z, s));
    GatArgs a;
    memset(&a, 0, sizeof(a));
    a.n = g->n;
    a.heads = c->heads;
    a.head_dim = c->head_dim;
    a.rel = c->kind == NRT_RGAT;
    a.slope = c->leaky_slope;
    a.att_src = c->att_src[l - 1];
    a.att_dst = c->att_dst[l - 1];
    a.Z = c->Z[l];
    a.AS = c->AS[l];
    a.AD = c->AD[l];
    a.rows = src_rows;
    a.n_rows_dev = n_src_dev;
    a.rows_bound = src_bound;
    a.AS_old = incremental ? c->AS_old : nullptr;
    NRT_TRY(k_gat_scalars(a, s));
    if (out_args) *out_args = a;
    return NRT_OK;
}

static nrt_status run_gat_layer(nrt_cache* c, int l, const int32_t* src_rows, const uint64_t* n_src_dev, int64_t src_bound,
                                const int32_t* dst_rows, const uint64_t* n_dst_dev, int64_t dst_bound, bool listed,
                                bool incremental, int prev, float* out_rows, int64_t out_cap, hipStream_t s) {
    nrt_graph* g = c->g;
    const bool last = l == c->L;
    GatArgs a;
    NRT_TRY(run_gat_project(c, l, src_rows, n_src_dev, src_bound, listed, incremental, &a, s));
    NRT_TRY(prof_mark(c, TAG_ITEMS, l, s));
    a.rows = dst_rows;
    a.n_rows_dev = n_dst_dev;
    a.rows_bound = dst_bound;
    a.recs = c->recs;
    a.hubs = c->hubs;
    a.lc = c->lc_use ? c->lc_use : &c->lc[l];
    a.part_m = c->part_m;
    a.part_den = c->part_den;
    a.Z_old = c->DP[0];
    a.in = g->in;
    if (incremental) {
        a.src_bitmap = c->bm[prev];
        a.src_slot = c->slot[prev];
        a.ddst_bitmap = c->bm_ddst;
        a.dd_slot = c->slot_dd;
        a.sd_s = c->SD[l];
        a.sd_den = c->SDden[l];
        a.ins_cnt = c->ins_cnt;
        a.n_src_dev = n_src_dev;
    }
    a.M = c->M[l];
    a.DEN = c->DEN[l];
    a.S = c->S[l];
    a.Hout = c->H[l];
    a.bias = c->bias[l - 1][0];
    a.act = last ? 0 : 2;
    a.out_rows = last ? out_rows : nullptr;
    a.out_cap = out_cap;
    if (!last && !c->H[l]) {                 // aggregate-only storage: this layer's rows go compact to the next layer's product
        if (!listed) { nrt_set_error("hidden rows are not kept"); return NRT_ERR_STATE; }
        a.out_rows = c->DP[1];               // (read by this layer's own product above, which has finished)
        a.out_cap = g->n;
    }
    if (c->profiling) a.pair_ctr = c->pair_ctr + (size_t)(l - 1) * 1024;
    NRT_TRY(k_gat_gather(a, s));
    NRT_TRY(prof_mark(c, TAG_GATHER, l, s));
    return NRT_OK;
}

// Aggregate-only storage (GCN, hidden layer l): h^l of the listed rows from the cached aggregate and the given degree
// vector, not stored by vertex.  out_compact: the rows themselves; dp with dp_no_h 1: minus their payload (old degrees),
// 2: plus their payload added to what dp holds.
static nrt_status run_update_unkept(nrt_cache* c, int l, const int32_t* rows, int64_t M, const uint64_t* M_dev,
                                    const int32_t* indeg, float* out_compact, int64_t out_cap, float* dp, int dp_no_h,
                                    hipStream_t s) {
    GemmArgs a;
    memset(&a, 0, sizeof(a));
    a.M = M;
    a.M_dev = M_dev;
    a.rows = rows;
    a.indeg = indeg;
    a.indeg_old = c->indeg_old;
    a.ldp = c->dims[l - 1];
    a.K = c->dims[l - 1];
    a.N = c->dims[l];
    a.a_mode = A_SCALE_GCN;
    a.P0 = c->S[l];
    a.Wt = c->Wt[l - 1][0];
    a.bias = c->bias[l - 1][0];
    a.act = 1;
    a.DP = dp;
    a.dp_no_h = dp_no_h;
    a.dp_scale_gcn = 1;
    a.n_vertices = c->g->n;
    a.out_compact = out_compact;
    a.out_cap = out_cap;
    return k_gemm(a, s);
}

// A-GNN / G-GCN, layer l: what the messages need of the rows of h^{l-1} that changed (src_rows null: all rows): their
// inverse norms, or for G-GCN the two projections W_1 h and W_2 h; with `incremental` the replaced values are kept compact
static nrt_status run_agnn_project(nrt_cache* c, int l, const int32_t* src_rows, const uint64_t* n_src_dev, int64_t src_bound,
                                   bool incremental, hipStream_t s) {
    nrt_graph* g = c->g;
    const int D = c->dims[l - 1];
    if (c->kind == NRT_GGCN) {
        GemmArgs p;
        memset(&p, 0, sizeof(p));
        p.M = src_rows ? src_bound : g->n;
        p.M_dev = n_src_dev;
        p.rows = src_rows;
        p.a_mode = A_PLAIN;
        p.P0 = c->H[l - 1];
        p.ldp = D;
        p.K = D;
        p.N = D;
        p.n_vertices = g->n;
        p.Wt = c->Wt[l - 1][1];
        p.H = c->P1[l - 1];
        p.DP = (incremental && src_rows) ? c->old_p1 : nullptr;    // the W_1 rows this launch replaces
        p.dp_store_old = 1;
        NRT_TRY(k_gemm(p, s));
        p.Wt = c->W2t[l - 1];
        p.H = c->P2[l - 1];
        p.DP = nullptr;
        return k_gemm(p, s);
    }
    return k_agnn_norms(src_rows, n_src_dev, src_rows ? src_bound : g->n, c->H[l - 1], D, c->R[l - 1],
                        (incremental && src_rows) ? c->r_old : nullptr, s);
}

// One A-GNN or G-GCN layer: norms (G-GCN: the two projections) of the changed rows of h^{l-1} (src_rows null: all rows), the gather over the
// destinations described by c->recs (listed in `rows`, null: all n), the sums of long in-lists, the dense update.
static nrt_status run_agnn_layer(nrt_cache* c, int l, const int32_t* src_rows, const uint64_t* n_src_dev, int64_t src_bound,
                                 const int32_t* rows, const uint64_t* M_dev, int64_t M, bool incremental, int prev, int cur,
                                 float* out_rows, int64_t out_cap, hipStream_t s) {
    nrt_graph* g = c->g;
    const bool last = l == c->L;
    const int D = c->dims[l - 1];
    const bool gate = c->kind == NRT_GGCN;
    NRT_TRY(run_agnn_project(c, l, src_rows, n_src_dev, src_bound, incremental, s));
    NRT_TRY(prof_mark(c, TAG_ITEMS, l, s));
    AgnnArgs a;
    memset(&a, 0, sizeof(a));
    a.recs = c->recs;
    a.hubs = c->hubs;
    a.lc = c->lc_use ? c->lc_use : &c->lc[l];
    a.in = g->in;
    a.H = c->H[l - 1];
    a.R = c->R[l - 1];
    a.D = D;
    a.beta = c->agnn_beta[l - 1];
    a.gate = gate ? 1 : 0;
    a.P1 = c->P1[l - 1];
    a.P2 = c->P2[l - 1];
    a.old_p1 = c->old_p1;
    a.S = c->S[l];
    if (c->profiling) a.pair_ctr = c->pair_ctr + (size_t)(l - 1) * 1024;
    if (incremental) {
        a.incremental = 1;
        a.src_bitmap = c->bm[prev];
        a.src_slot = c->slot[prev];
        a.old_rows = c->DP[prev];
        a.old_r = c->r_old;
        a.sd = c->SD[l];
        a.dd_bitmap = c->bm_ddst;
        a.dd_slot = c->slot_dd;
    }
    NRT_TRY(k_agnn_gather(a, s));
    NRT_TRY(prof_mark(c, TAG_GATHER, l, s));
    NRT_TRY(k_agnn_combine(a, s));
    NRT_TRY(prof_mark(c, TAG_COMBINE, l, s));
    GemmArgs u;
    memset(&u, 0, sizeof(u));
    u.M = M;
    u.M_dev = M_dev;
    u.rows = rows;
    u.a_mode = A_PLAIN;
    u.P0 = c->S[l];
    u.ldp = D;
    u.K = D;
    u.N = c->dims[l];
    u.Wt = c->Wt[l - 1][0];
    u.bias = c->bias[l - 1][0];
    u.act = last ? 0 : 1;
    u.H = c->H[l];
    u.DP = (incremental && !last) ? c->DP[cur] : nullptr;      // the rows this update replaces: the next layer's old terms
    u.dp_store_old = 1;
    u.n_vertices = g->n;
    u.out_compact = last ? out_rows : nullptr;
    u.out_cap = out_cap;
    return k_gemm(u, s);
}

// Full-neighbour forward over every vertex of every layer (Eq. 1) from the current h^0 and graph; fills all caches.
// Every vertex is a destination: records and hub items are built once, with their counters in the spare
// LayerCtrs slot (zero on entry), and serve all layers.
static nrt_status full_forward(nrt_cache* c, hipStream_t s) {
    nrt_graph* g = c->g;
    const int64_t n = g->n;
    LayerCtrs* all = &c->lc[NRT_MAX_LAYERS + 1];
    NRT_TRY(k_dst_records(nullptr, n, g->in, c->recs, c->hubs, all, true, nullptr, s));
    NRT_TRY(k_fill_u64(&all->count, 1, (uint64_t)n, s));
    c->lc_use = all;
    nrt_status st = NRT_OK;
    if (c->agg_only)                       // hidden rows live in the two delta buffers while the aggregates are built
        for (int l = 1; l < c->L; ++l) c->H[l] = c->DP[l & 1];
    for (int l = 1; l <= c->L && st == NRT_OK; ++l) {
        if (c->is_gat) {
            st = run_gat_layer(c, l, nullptr, nullptr, n, nullptr, nullptr, n, false, false, 0, nullptr, 0, s);
            continue;
        }
        if (agnn_family(c->kind)) {
            st = run_agnn_layer(c, l, nullptr, nullptr, n, nullptr, nullptr, n, false, 0, 0, nullptr, 0, s);
            continue;
        }
        if (c->MP[l - 1]) st = run_transform(c, l - 1, nullptr, n, nullptr, nullptr, false, s);
        if (st == NRT_OK) st = run_gather(c, l, false, 0, false, 0, s);
        if (st == NRT_OK) st = run_update(c, l, nullptr, n, nullptr, false, 0, nullptr, 0, false, s);
    }
    c->lc_use = nullptr;
    if (c->agg_only)
        for (int l = 1; l < c->L; ++l) c->H[l] = nullptr;
    return st;
}

// ------------------------------------------------------------------ cache init
extern "C" nrt_status nrt_cache_init(nrt_graph* g, const nrt_model_desc* d, const float* features,
                                     int64_t max_batch_edges, int64_t max_batch_feats, void* workspace,
                                     size_t workspace_bytes, void* stream, nrt_cache** out) {
    REQUIRE(g && out && features, "null argument");
    NRT_TRY(check_desc(d));
    REQUIRE(workspace && (reinterpret_cast<uintptr_t>(workspace) & 255) == 0, "workspace must be 256-byte aligned");
    size_t need = 0;
    NRT_TRY(nrt_cache_workspace_bytes(g, d, max_batch_edges, max_batch_feats, &need));
    REQUIRE(workspace_bytes >= need, "cache workspace too small");
    if (g->has_cache) { nrt_set_error("graph already has a cache"); return NRT_ERR_STATE; }
    if (d->kind == NRT_RGCN || d->kind == NRT_RGAT)
        REQUIRE(g->weighted, "RGCN and RGAT need a weighted graph: the edge weights are the relation ids");
    if (d->kind == NRT_RGCN)
        REQUIRE(g->n * d->n_relations <= (int64_t)INT32_MAX, "RGCN: vertices * relations must fit 31 bits");
    for (int l = 0; l < d->n_layers; ++l) {
        REQUIRE(d->W[l][0], "W[l][0] is null");
        if (d->kind == NRT_GIN) REQUIRE(d->W[l][1], "GIN needs W[l][1]");
        if (d->kind == NRT_PINSAGE) REQUIRE(d->W[l][1], "PinSAGE needs W[l][1]");
        if (d->kind == NRT_GGCN) REQUIRE(d->W[l][1], "G-GCN needs W[l][1] = [W_1; W_2]");
        if (d->kind == NRT_RGCN) REQUIRE(d->W[l][1], "RGCN needs W[l][1] = [W_0 | ... | W_{R-1}]");
        if (d->kind == NRT_MONET) REQUIRE(d->monet_mu[l] && d->monet_prec[l], "MoNet needs monet_mu[l] and monet_prec[l]");
        if (d->kind == NRT_GAT || d->kind == NRT_RGAT) REQUIRE(d->att_src[l] && d->att_dst[l], "GAT and RGAT need att_src[l] and att_dst[l]");
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    nrt_cache* c = new (std::nothrow) nrt_cache;
    if (!c) { nrt_set_error("host allocation failed"); return NRT_ERR_OOM; }
    cache_fill(c, g, d, max_batch_edges, max_batch_feats);
    Bump b{static_cast<char*>(workspace), 0};
    cache_layout(b, c);
    const size_t lc_bytes = (LC_TOTAL * sizeof(LayerCtrs) + 255) & ~size_t(255);
    if (hipHostMalloc((void**)&c->lc_host, lc_bytes + 1024 * NRT_MAX_LAYERS * sizeof(unsigned long long),
                      hipHostMallocDefault) != hipSuccess) {
        delete c;
        nrt_set_error("pinned host allocation failed");
        return NRT_ERR_OOM;
    }
    c->pair_host = reinterpret_cast<unsigned long long*>(reinterpret_cast<char*>(c->lc_host) + lc_bytes);
    const int64_t n = g->n;
    auto run = [&]() -> nrt_status {
        NRT_TRY(k_copy_f32(c->H[0], features, n * c->dims[0], s));
        NRT_TRY(k_fill_u32((uint32_t*)c->sc.feat_stamp, n, 0, s));
        NRT_TRY(k_fill_u32((uint32_t*)c->flags, (n + 64) / 4, 0, s));
        NRT_TRY(k_fill_u64((uint64_t*)c->lc, LC_TOTAL * sizeof(LayerCtrs) / 8, 0, s));
        NRT_TRY(k_fill_u64(c->cmp_state, c->cmp_state_len, 0, s));
        for (int l = 0; l < c->L; ++l) {
            const int kin = c->kind == NRT_MONET ? c->monet_J : (concat_self(c->kind) ? 2 : 1) * c->dims[l];
            NRT_TRY(k_transpose(d->W[l][0], c->Wt[l][0], kin, c->is_gat ? c->zdim : c->dims[l + 1], s));
            if (d->b[l][0]) NRT_TRY(k_copy_f32(c->bias[l][0], d->b[l][0], c->dims[l + 1], s));
            else NRT_TRY(k_fill_u32((uint32_t*)c->bias[l][0], c->dims[l + 1], 0, s));
            if (c->kind == NRT_GGCN) {                     // W[l][1] is [2 d][d]: W_1 on top of W_2
                const int dq = c->dims[l];
                NRT_TRY(k_transpose(d->W[l][1], c->Wt[l][1], dq, dq, s));
                NRT_TRY(k_transpose(d->W[l][1] + (size_t)dq * dq, c->W2t[l], dq, dq, s));
            }
            if (c->kind == NRT_MONET) {
                NRT_TRY(k_transpose(d->monet_mu[l], c->muT[l], c->monet_J, c->dims[l], s));
                NRT_TRY(k_transpose(d->monet_prec[l], c->precT[l], c->monet_J, c->dims[l], s));
            }
            if (c->is_gat) {
                NRT_TRY(k_copy_f32(c->att_src[l], d->att_src[l], (int64_t)c->heads * c->head_dim, s));
                NRT_TRY(k_copy_f32(c->att_dst[l], d->att_dst[l], (int64_t)c->heads * c->head_dim, s));
            }
            if (c->kind == NRT_RGCN)
                NRT_TRY(k_transpose(d->W[l][1], c->Wt[l][1], c->dims[l], c->n_rel * c->dims[l + 1], s));
            if (c->kind == NRT_GIN || c->kind == NRT_PINSAGE) {
                const int dq = c->kind == NRT_GIN ? c->dims[l + 1] : c->dims[l];
                NRT_TRY(k_transpose(d->W[l][1], c->Wt[l][1], dq, dq, s));
                if (d->b[l][1]) NRT_TRY(k_copy_f32(c->bias[l][1], d->b[l][1], dq, s));
                else NRT_TRY(k_fill_u32((uint32_t*)c->bias[l][1], dq, 0, s));
            }
        }
        for (int l = 1; l <= c->L; ++l)
            if (c->stale[l]) NRT_TRY(k_fill_u32(c->stale[l], (n + 31) / 32, 0, s));
        if (c->n_rel) {                                        // typed edges: every edge weight must be a relation id
            int32_t* bad = (int32_t*)(g->dev_ctrs + CTR_ERR) + 7;
            NRT_TRY(k_fill_u32((uint32_t*)bad, 1, 0, s));
            NRT_TRY(k_check_list_relations(g->in, n, c->n_rel, bad, s));
            NRT_TRY(read_ctrs(g, s));
            if (((const int32_t*)(g->host_pinned + CTR_ERR))[7]) {
                nrt_set_error("an edge weight is not a relation id in [0, n_relations)");
                return NRT_ERR_INVALID_ARG;
            }
        }
        NRT_TRY(full_forward(c, s));
        HIP_TRY(hipStreamSynchronize(s));
        return NRT_OK;
    };
    nrt_status st = run();
    if (st != NRT_OK) { (void)hipHostFree(c->lc_host); delete c; return st; }
    c->mode = NRT_MODE_AUTO;
    if (hipEventCreateWithFlags(&c->ev_validated, hipEventDisableTiming) != hipSuccess) {
        (void)hipHostFree(c->lc_host);
        delete c;
        nrt_set_error("hipEventCreate failed");
        return NRT_ERR_DEVICE;
    }
    c->ev_validated_made = true;
    g->has_cache = true;
    *out = c;
    return NRT_OK;
}

extern "C" void nrt_cache_destroy(nrt_cache* c) {
    if (!c) return;
    if (c->events_made)
        for (int i = 0; i < MAX_EVENTS; ++i) (void)hipEventDestroy(c->ev[i]);
    if (c->ev_validated_made) (void)hipEventDestroy(c->ev_validated);
    if (c->lc_host) (void)hipHostFree(c->lc_host);
    if (c->g) c->g->has_cache = false;
    delete c;
}

// ------------------------------------------------------------------ apply batch
struct QueryArgs {                  // the query served together with a batch in on-demand mode (ids null: none)
    const int32_t* ids; int64_t n; float* rows;
    int64_t *n_updated, *n_recomputed;      // host, may be null
};
static nrt_status serve_query_after_batch(nrt_cache* c, const QueryArgs& q, bool fold, hipStream_t s);

static nrt_status apply_batch_impl(nrt_cache* c, const nrt_batch* b, int32_t* affected_ids, float* affected_rows,
                                   int64_t capacity, int64_t* n_affected, const QueryArgs& q, void* stream) {
    REQUIRE(c && b && n_affected, "null argument");
    REQUIRE(b->n_ins >= 0 && b->n_del >= 0 && b->n_feat >= 0, "negative batch count");
    REQUIRE(capacity >= 0 && (capacity == 0 || affected_ids), "affected_ids is null");
    REQUIRE(!(c->lazy && affected_rows), "on-demand mode returns no rows from nrt_apply_batch (use nrt_query)");
    nrt_graph* g = c->g;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t n = g->n;
    if (b->n_ins + b->n_del > c->max_edges || b->n_feat > c->max_feats) {
        nrt_set_error("batch larger than the bounds given to nrt_cache_init");
        return NRT_ERR_BAD_BATCH;
    }
    if ((b->n_ins && (!b->ins_src || !b->ins_dst)) || (b->n_del && (!b->del_src || !b->del_dst)) ||
        (b->n_feat && (!b->feat_ids || !b->feat_rows)) || (b->n_ins && g->weighted && !b->ins_w)) {
        nrt_set_error("batch array is null");
        return NRT_ERR_BAD_BATCH;
    }
    if (g->e + b->n_ins - b->n_del > g->e_capacity) {
        nrt_set_error("batch would exceed e_capacity");
        return NRT_ERR_OOM;
    }
    memset(&c->stats, 0, sizeof(c->stats));
    c->stats.n_layers = c->L;
    c->n_ev = 0;
    nrt_launch_count = 0;
    int64_t prev_n_list[NRT_MAX_LAYERS + 1];            // sizes of the previous batch's sets: hints for this one
    for (int l = 0; l <= c->L; ++l) { prev_n_list[l] = c->n_list[l]; c->n_list[l] = 0; }
    const bool had_history = c->have_history;
    c->have_history = false;
    c->have_history_prev = had_history;
    NRT_TRY(prof_mark(c, TAG_START, 0, s));

    // ---- validate (no state change yet)
    {
        // per-batch scratch of the cache is cleared in the validation's fill launch: set bitmaps, layer counters,
        // the rows that collect structural terms (none of it is state, so a rejected batch loses nothing)
        FillJobs f;
        memset(&f, 0, sizeof(f));
        f.add(c->bm_ddst, 2 * c->nw_pad);                     // bm_ddst and bm_feat are adjacent
        f.add(c->lc, (int64_t)(LC_TOTAL * sizeof(LayerCtrs) / 4));
        if (c->profiling) f.add(c->pair_ctr, 2 * 1024 * NRT_MAX_LAYERS);
        if (b->n_ins + b->n_del > 2048) {                     // scratch of the batch plan's counting form
            f.add(c->plan_off64, 2 * (b->n_ins + b->n_del + 1));
            f.add(c->plan_cursor, b->n_ins + b->n_del);
        }
        if (q.ids) f.add(c->bm_q, (n + 31) / 32);
        c->sc.bm_dst = c->bm_ddst;                            // the batch's sets are marked by the validation kernels
        c->sc.bm_feat = c->bm_feat;
        NRT_TRY(graph_validate_batch(g, b, c->sc, &f, s));
    }
    // The verdict travels to the host while the device goes on with work that touches only per-batch scratch and
    // tolerates a bad batch (ids are range-checked there, caches are only read): the host waits for the event, not
    // for the stream, so the queue never runs dry between validation and mutation.
    if (q.ids)                                                // the queried set; an id out of range rejects the call like a bad batch
        NRT_TRY(k_mark_ids(c->bm_q, q.ids, q.n, n, (int32_t*)(g->dev_ctrs + CTR_ERR) + 6, s));
    if (c->n_rel)                                             // typed edges: the inserted edges' relation ids
        NRT_TRY(k_check_relations(b->ins_w, b->n_ins, c->n_rel, (int32_t*)(g->dev_ctrs + CTR_ERR) + 7, s));
    HIP_TRY(hipMemcpyAsync(g->host_pinned, g->dev_ctrs, NRT_NCTRS * sizeof(int64_t), hipMemcpyDeviceToHost, s));
    HIP_TRY(hipEventRecord(c->ev_validated, s));
    const bool empty_batch = b->n_ins + b->n_del + b->n_feat == 0;
    // ---- sets of the batch, structural terms on the old caches (scratch only)
    const bool gcn = c->kind == NRT_GCN;
    // a query served with the batch folds deltas into the vertices that were up to date before the batch (the models
    // whose messages are h itself and do not read the destination); that needs the same structural terms and layer-0
    // deltas as eager incremental maintenance
    const bool foldq = c->lazy && q.ids && !empty_batch &&
                       (c->kind == NRT_GCN || c->kind == NRT_SAGE_MEAN || c->kind == NRT_GIN || c->kind == NRT_COMMNET);
    const bool inc = foldq || (!c->lazy && (c->mode == NRT_MODE_INCREMENTAL || c->mode == NRT_MODE_AUTO));
    // layers that may switch to recomputation on the device: only where the previous batch had a large source set
    // (no extra launches for small frontiers); the device counters of this batch take the decision
    bool may_rec[NRT_MAX_LAYERS + 2];
    for (int l = 0; l <= c->L + 1; ++l)
        may_rec[l] = !c->lazy && c->mode == NRT_MODE_AUTO && !c->is_gat && !agnn_family(c->kind) && (!c->agg_only || c->kind != NRT_GCN) && l >= 1 && l <= c->L && prev_n_list[l - 1] * 8 > n;
    if (gcn && inc && !empty_batch) NRT_TRY(k_copy_i32(c->indeg_old, g->in.deg, n, s));
    uint64_t* n_slots_dev = (uint64_t*)(g->dev_ctrs + CTR_COUNT);
    if (b->n_ins + b->n_del > 0) {
        // the batch plan: updates grouped by destination in a fixed order.  Its slots are the compact rows that collect
        // the structural terms; its ranks place the inserted in-edges (bm[1] is scratch here)
        PlanArgs p;
        memset(&p, 0, sizeof(p));
        p.n_ins = b->n_ins; p.n_del = b->n_del; p.n = n;
        p.ins_src = b->ins_src; p.ins_dst = b->ins_dst; p.del_src = b->del_src; p.del_dst = b->del_dst;
        p.dst_bitmap = c->bm_ddst;
        p.scratch_bm = c->bm[1];
        p.list = c->list_dd; p.slot_of = c->slot_dd;
        p.off = c->plan_off; p.ord = c->plan_ord; p.ins_cnt = c->ins_cnt; p.ins_rank = c->ins_rank;
        p.count = n_slots_dev;
        p.off64 = c->plan_off64; p.cursor = c->plan_cursor; p.tmp = c->plan_tmp;
        p.total = (uint64_t*)(g->dev_ctrs + CTR_PLAN_TOTAL);
        p.cmp_state = c->cmp_state; p.cmp_state_len = c->cmp_state_len;
        NRT_TRY(k_batch_plan(p, c->plan_scan, c->plan_scan_len, s));
    }
    c->sc.plan_slot_of = c->slot_dd;
    c->sc.plan_ins_cnt = c->ins_cnt;
    c->sc.plan_ins_rank = c->ins_rank;

    // ---- structural terms on the old caches, all layers in one launch
    if (inc && c->is_gat) {
        GatFoldArgs f;
        memset(&f, 0, sizeof(f));
        f.n_ins = b->n_ins; f.n_del = b->n_del;
        f.del_src = b->del_src; f.del_dst = b->del_dst;
        f.del_w = c->kind == NRT_RGAT ? c->sc.del_w : nullptr;
        f.n_slots = n_slots_dev; f.off = c->plan_off; f.ord = c->plan_ord; f.list = c->list_dd;
        f.n = n;
        f.n_layers = c->L; f.heads = c->heads; f.head_dim = c->head_dim; f.slope = c->leaky_slope;
        for (int l = 1; l <= c->L; ++l) {
            f.Z[l - 1] = c->Z[l]; f.AS[l - 1] = c->AS[l]; f.AD[l - 1] = c->AD[l]; f.M[l - 1] = c->M[l];
            f.SDS[l - 1] = c->SD[l]; f.SDDEN[l - 1] = c->SDden[l];
        }
        NRT_TRY(k_gat_structural_fold(f, s));
    }
    if (inc && agnn_family(c->kind)) {
        AgnnFoldArgs f;
        memset(&f, 0, sizeof(f));
        f.n_ins = b->n_ins; f.n_del = b->n_del; f.n = n;
        f.ins_src = b->ins_src; f.del_src = b->del_src;
        f.n_slots = n_slots_dev; f.off = c->plan_off; f.ord = c->plan_ord; f.list = c->list_dd;
        f.n_layers = c->L;
        for (int l = 1; l <= c->L; ++l) {
            f.H[l - 1] = c->H[l - 1]; f.R[l - 1] = c->R[l - 1]; f.SD[l - 1] = c->SD[l];
            f.D[l - 1] = c->dagg[l]; f.beta[l - 1] = c->agnn_beta[l - 1];
            f.P1[l - 1] = c->P1[l - 1]; f.P2[l - 1] = c->P2[l - 1];
        }
        f.gate = c->kind == NRT_GGCN;
        NRT_TRY(k_agnn_structural_fold(f, s));
    }
    if (inc && !c->is_gat && !agnn_family(c->kind)) {
        FoldArgs f;
        memset(&f, 0, sizeof(f));
        f.n_ins = b->n_ins; f.n_del = b->n_del;
        f.ins_src = b->ins_src; f.ins_dst = b->ins_dst; f.del_src = b->del_src; f.del_dst = b->del_dst;
        if (weighted_messages(c->kind) && g->weighted) { f.ins_w = b->ins_w; f.del_w = c->sc.del_w; }
        f.rel_R = c->n_rel;
        if (c->agg_only && gcn && c->L > 1 && b->n_ins + b->n_del > 0) {
            // the hidden rows of the updated edges' sources are not kept: recompute them from the (old) aggregates
            const int64_t nops = b->n_ins + b->n_del;
            NRT_TRY(k_concat_ids(c->es_rows, b->ins_src, b->n_ins, b->del_src, b->n_del, n, s));
            for (int l = 1; l < c->L; ++l)
                NRT_TRY(run_update_unkept(c, l, c->es_rows, nops, nullptr, g->in.deg, c->ES[l], nops, nullptr, 0, s));
        }
        f.indeg_old = gcn ? g->in.deg : nullptr;
        f.n_layers = c->L;
        f.n = n;
        f.n_slots = n_slots_dev; f.off = c->plan_off; f.ord = c->plan_ord;
        for (int l = 1; l <= c->L; ++l) {
            f.Hprev[l - 1] = payload_rows(c, l - 1);
            if (c->agg_only && gcn && l - 1 >= 1) { f.Hprev[l - 1] = c->ES[l - 1]; f.compact_src[l - 1] = 1; }
            f.SD[l - 1] = c->SD[l];
            f.D[l - 1] = c->dagg[l];
        }
        NRT_TRY(k_structural_fold(f, s));
    }

    HIP_TRY(hipEventSynchronize(c->ev_validated));
    {
        const int32_t* err = (const int32_t*)(g->host_pinned + CTR_ERR);
        const char* msg = nullptr;
        if (err[0]) msg = "vertex id out of range";
        else if (err[1]) msg = "self-loop in batch";
        else if (err[4]) msg = "edge repeated inside the batch";
        else if (err[5]) msg = "feature id repeated inside the batch";
        else if (err[2]) msg = "inserted edge already present";
        else if (err[3]) msg = "deleted edge not present";
        else if (err[7]) msg = "relation id of an inserted edge out of range";
        nrt_status bad = NRT_OK;
        if (msg) { nrt_set_error("%s", msg); bad = NRT_ERR_BAD_BATCH; }
        else if (err[6]) { nrt_set_error("query id out of range"); bad = NRT_ERR_INVALID_ARG; }
        else if (g->host_pinned[CTR_HEAD_OUT] + g->host_pinned[CTR_GROW] > g->out.pool_cap ||
                 g->host_pinned[CTR_HEAD_IN] + g->host_pinned[CTR_GROW + 1] > g->in.pool_cap) {
            nrt_set_error("adjacency pool exhausted");
            bad = NRT_ERR_OOM;
        }
        if (bad != NRT_OK) {
            NRT_TRY(graph_cancel_batch(g, b, s));
            HIP_TRY(hipStreamSynchronize(s));
            return bad;
        }
    }
    if (b->n_ins + b->n_del + b->n_feat == 0) {
        NRT_TRY(graph_mutate(g, b, c->sc, s));
        *n_affected = 0;
        if (q.ids) {                                          // nothing changed: the query alone
            int64_t nr = 0;
            NRT_TRY(nrt_query(c, q.ids, q.n, q.rows, &nr, stream));
            if (q.n_updated) *q.n_updated = nr;
            if (q.n_recomputed) *q.n_recomputed = nr;
        }
        return NRT_OK;
    }

    // ---- graph mutation
    NRT_TRY(graph_mutate(g, b, c->sc, s));

    // ---- sources of change for layer 1 (replaced features; for GCN also the re-normalised destinations)
    const int64_t n0_bound = b->n_feat + (gcn ? b->n_ins + b->n_del : 0);
    CompactExtra cx;
    memset(&cx, 0, sizeof(cx));
    cx.err = &c->lc[0].pad[0];
    cx.coarse_shift = c->coarse_shift;
    cx.coarse_words = c->coarse_words;
    cx.coarse = c->coarse_shift <= 10 ? c->coarse[0] : nullptr;
    NRT_TRY(k_compact(nullptr, c->bm_feat, gcn ? c->bm_ddst : nullptr, c->bm[0], n, c->list[0], c->slot[0], c->cmp_state,
                      c->cmp_state_len, &c->lc[0].count, s, nullptr, &cx));
    {
        DeltaArgs da;
        memset(&da, 0, sizeof(da));
        da.list = c->list[0];
        da.n_dev = &c->lc[0].count;
        da.bound = n0_bound;
        da.feat_bitmap = c->bm_feat;
        da.feat_index = c->sc.feat_index;
        da.feat_rows = b->feat_rows;
        da.H0 = c->H[0];
        da.DP = c->DP[0];
        da.D = c->dims[0];
        if (gcn && inc) { da.indeg_new = g->in.deg; da.indeg_old = c->indeg_old; }
        da.store_old = agnn_family(c->kind);
        NRT_TRY(k_layer0_delta(da, s));
    }
    if (q.ids) NRT_TRY(k_copy_i32((int32_t*)c->need_bm[0], (const int32_t*)c->bm[0], (n + 31) / 32, s));   // bm[0] is reused by the hops
    NRT_TRY(prof_mark(c, TAG_INGEST, 0, s));

    // ---- layers: no host round trip, every size stays on the device
    int prev = 0;
    for (int l = 1; l <= c->L; ++l) {
        const int cur = 1 - prev;
        const int64_t src_bound = l == 1 ? n0_bound : n;
        PullArgs pull;
        memset(&pull, 0, sizeof(pull));
        pull.allowed = prev_n_list[l - 1] * 16 > n;      // hint from the previous batch; the device decides (8x)
        pull.n = n;
        pull.src_bitmap = c->bm[prev];
        pull.long_list = c->pull_list;
        pull.long_cap = n;
        pull.long_count = (unsigned long long*)&c->lc[l - 1].n_pull_long;
        NRT_TRY(k_expand_frontier(g->out, c->list[l - 1], &c->lc[l - 1].count, src_bound, c->flags, &c->lc[l - 1],
                                  c->xhub_list, c->xhub_cap, g->in, pull, s));
        NRT_TRY(prof_mark(c, TAG_EXPAND, l, s));
        cx.coarse = (c->coarse_shift <= 10 && !c->lazy) ? c->coarse[cur] : nullptr;   // on-demand mode: the set only becomes
        cx.list2 = l == c->L ? affected_ids : nullptr;              // stale; slot map and coarse copy of layer 1's sources stay
        cx.cap2 = capacity;                                         // (the last set is also the caller's list)
        NRT_TRY(k_compact(c->flags, c->bm_ddst, c->bm[prev], c->bm[cur], n, c->list[l], c->lazy ? nullptr : c->slot[cur],
                          c->cmp_state, c->cmp_state_len, &c->lc[l].count, s, nullptr, &cx));
        if (c->lazy) {                                     // on-demand mode: A_l only becomes stale
            if (q.ids) NRT_TRY(k_copy_i32((int32_t*)c->stale_prev[l], (const int32_t*)c->stale[l], (n + 31) / 32, s));
            // h^0 is never stale, so neither may be what layer 1 caches of it by vertex: message rows, z and the
            // attention scalars, inverse norms, gate projections
            if (c->MP[0] && l == 1)                        // (a query folded with this batch takes the rows' deltas from DP[0])
                NRT_TRY(run_transform(c, 0, c->list[0], src_bound, &c->lc[0].count, foldq ? c->DP[0] : nullptr, false, s));
            if (c->is_gat && l == 1)
                NRT_TRY(run_gat_project(c, 1, c->list[0], &c->lc[0].count, src_bound, true, false, nullptr, s));
            if (agnn_family(c->kind) && l == 1)
                NRT_TRY(run_agnn_project(c, 1, c->list[0], &c->lc[0].count, src_bound, false, s));
            NRT_TRY(k_or_words(c->stale[l], c->stale[l], c->bm[cur], (n + 31) / 32, s));
            prev = cur;
            continue;
        }
        if (c->mode == NRT_MODE_FULL) {                    // only the affected lists are needed layer by layer
            NRT_TRY(prof_mark(c, TAG_COMPACT, l, s));
            prev = cur;
            continue;
        }
        // GAT with only edge updates in the layer (no z changed): every destination takes the O(#updates) path of
        // Algorithm 3, also those with long in-lists, so no items are cut
        NRT_TRY(k_dst_records(c->list[l], n, g->in, c->recs, c->hubs, &c->lc[l], false,
                              (c->is_gat && inc) ? &c->lc[l - 1].count : nullptr, s));
        NRT_TRY(prof_mark(c, TAG_COMPACT, l, s));
        if (c->is_gat) {
            NRT_TRY(run_gat_layer(c, l, c->list[l - 1], &c->lc[l - 1].count, src_bound, c->list[l], &c->lc[l].count, n, true,
                                  inc, prev, l == c->L ? affected_rows : nullptr, capacity, s));
        } else if (agnn_family(c->kind)) {
            NRT_TRY(run_agnn_layer(c, l, c->list[l - 1], &c->lc[l - 1].count, src_bound, c->list[l], &c->lc[l].count, n, inc,
                                   prev, cur, l == c->L ? affected_rows : nullptr, capacity, s));
        } else {
            // which gather kernel: the previous batch's source count at this layer is the hint; a clearly sparse or
            // clearly dense layer launches one kernel, in between both are launched and the device counter decides
            const int64_t pn = prev_n_list[l - 1];
            const int sparse_hint = !had_history ? 1 : (pn * 64 <= n ? 2 : (pn * 4 > n ? 0 : 1));
            if (c->MP[l - 1])
                NRT_TRY(run_transform(c, l - 1, c->list[l - 1], src_bound, &c->lc[l - 1].count, inc ? delta_buf(c, prev) : nullptr,
                                      may_rec[l], s));
            if (c->agg_only && gcn && l < c->L) {
                // the layer's rows are not kept: the payload deltas of its affected rows are minus the old payload,
                // computed from the aggregate before the fold, plus the new one, computed after it
                NRT_TRY(run_update_unkept(c, l, c->list[l], n, &c->lc[l].count, c->indeg_old, nullptr, 0, c->DP[cur], 1, s));
                NRT_TRY(run_gather(c, l, inc, prev, false, sparse_hint, s));
                NRT_TRY(run_update_unkept(c, l, c->list[l], n, &c->lc[l].count, g->in.deg, nullptr, 0, c->DP[cur], 2, s));
            } else {
                NRT_TRY(run_gather(c, l, inc, prev, may_rec[l], sparse_hint, s));
                NRT_TRY(run_update(c, l, c->list[l], n, &c->lc[l].count, inc, cur, l == c->L ? affected_rows : nullptr,
                                   capacity, may_rec[l + 1], s));
            }
        }
        NRT_TRY(prof_mark(c, TAG_UPDATE, l, s));
        prev = cur;
    }
    if (c->lazy && q.ids) NRT_TRY(serve_query_after_batch(c, q, foldq, s));
    if (c->mode == NRT_MODE_FULL && !c->lazy) {
        NRT_TRY(full_forward(c, s));
        if (affected_rows)
            NRT_TRY(k_gather_rows(affected_rows, c->H[c->L], c->list[c->L], &c->lc[c->L].count, capacity, n, c->dims[c->L], s));
        NRT_TRY(prof_mark(c, TAG_UPDATE, c->L, s));
    }
    HIP_TRY(hipMemcpyAsync(c->lc_host, c->lc, LC_TOTAL * sizeof(LayerCtrs), hipMemcpyDeviceToHost, s));
    if (c->profiling)
        HIP_TRY(hipMemcpyAsync(c->pair_host, c->pair_ctr, 1024 * NRT_MAX_LAYERS * sizeof(unsigned long long),
                               hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    if (c->lc_host[0].pad[0]) { nrt_set_error("internal: a compaction wait gave up"); return NRT_ERR_DEVICE; }
    for (int l = 0; l <= c->L; ++l) c->n_list[l] = (int64_t)c->lc_host[l].count;
    c->have_history = true;
    for (int l = 1; l <= c->L; ++l) {
        nrt_layer_stats* ls = &c->stats.layer[l - 1];
        ls->n_src = c->n_list[l - 1];
        ls->n_affected = c->n_list[l];
        ls->n_items = (int64_t)c->lc_host[l].n_items;
        for (int q = 0; q < 16; ++q) ls->n_in_edges += (int64_t)c->lc_host[l].in_edges[q];
        // Cannot happen: the capacities are bounds that follow from the graph's own limits (a destination with more than
        // NRT_CHUNK in-edges owns more than NRT_CHUNK of at most e_capacity edges, so there are fewer than
        // e_capacity / NRT_CHUNK of them and they have at most twice that many items; likewise for sources with long
        // out-lists), and the kernels clamp to the capacities, so nothing was written out of bounds.  Kept as a
        // consistency check of those bounds; the batch has been applied by now, so if it ever fires the caches must be
        // rebuilt (nrt.h documents NRT_ERR_STATE from this call that way).
        if ((int64_t)c->lc_host[l].n_hubs > c->hubs.hub_cap || (int64_t)c->lc_host[l].n_items > c->hubs.item_cap ||
            (int64_t)c->lc_host[l - 1].n_xhubs > c->xhub_cap) {
            nrt_set_error("internal: hub buffers too small (a bound of the cache layout is violated); rebuild the caches");
            return NRT_ERR_STATE;
        }
    }
    if (c->mode == NRT_MODE_FULL && !c->lazy) {
        const LayerCtrs& all = c->lc_host[NRT_MAX_LAYERS + 1];
        if ((int64_t)all.n_hubs > c->hubs.hub_cap || (int64_t)all.n_items > c->hubs.item_cap) {
            nrt_set_error("internal: hub buffers too small");
            return NRT_ERR_STATE;
        }
    }
    if (c->lazy && q.ids) {
        const LayerCtrs* need = c->lc_host + LC_BATCH;
        const LayerCtrs* redo = need + 2 * (NRT_MAX_LAYERS + 1);
        int64_t nu = 0, nr = 0;
        for (int l = 1; l <= c->L; ++l) {
            nu += (int64_t)need[l].count;
            nr += foldq ? (int64_t)redo[l].count : (int64_t)need[l].count;
            for (int k = 0; k < 3; ++k) {
                const LayerCtrs& t = need[k * (NRT_MAX_LAYERS + 1) + l];
                if ((int64_t)t.n_hubs > c->hubs.hub_cap || (int64_t)t.n_items > c->hubs.item_cap || (int64_t)t.n_xhubs > c->xhub_cap) {
                    nrt_set_error("internal: hub buffers too small (a bound of the cache layout is violated); rebuild the caches");
                    return NRT_ERR_STATE;
                }
            }
        }
        if (q.n_updated) *q.n_updated = nu;
        if (q.n_recomputed) *q.n_recomputed = nr;
        c->have_history = false;                          // the sets of this call are not those of an eager batch
    }
    c->stats.n_launches = nrt_launch_count;
    NRT_TRY(prof_collect(c));
    if (c->profiling) {
        for (int l = 1; l <= c->L; ++l) {
            unsigned long long tot = 0;
            for (int i = 0; i < 1024; ++i) tot += c->pair_host[(size_t)(l - 1) * 1024 + i];
            c->stats.layer[l - 1].n_pairs = (int64_t)tot;
        }
    }
    const int64_t na = c->n_list[c->L];
    *n_affected = na;
    if (na > capacity) {
        nrt_set_error("capacity %lld is smaller than the affected count %lld", (long long)capacity, (long long)na);
        return NRT_ERR_INVALID_ARG;
    }
    return NRT_OK;
}

extern "C" nrt_status nrt_apply_batch(nrt_cache* c, const nrt_batch* b, int32_t* affected_ids, float* affected_rows,
                                      int64_t capacity, int64_t* n_affected, void* stream) {
    QueryArgs none;
    memset(&none, 0, sizeof(none));
    return apply_batch_impl(c, b, affected_ids, affected_rows, capacity, n_affected, none, stream);
}

extern "C" nrt_status nrt_apply_batch_query(nrt_cache* c, const nrt_batch* b, int32_t* affected_ids, int64_t capacity,
                                            int64_t* n_affected, const int32_t* query_ids, int64_t n_query, float* query_rows,
                                            int64_t* n_updated, int64_t* n_recomputed, void* stream) {
    REQUIRE(c && query_ids && query_rows && n_query > 0, "null argument or empty query");
    if (!c->lazy) { nrt_set_error("nrt_apply_batch_query needs the on-demand mode (nrt_set_lazy)"); return NRT_ERR_STATE; }
    if (n_updated) *n_updated = 0;
    if (n_recomputed) *n_recomputed = 0;
    QueryArgs q;
    q.ids = query_ids; q.n = n_query; q.rows = query_rows; q.n_updated = n_updated; q.n_recomputed = n_recomputed;
    return apply_batch_impl(c, b, affected_ids, nullptr, capacity, n_affected, q, stream);
}

// ------------------------------------------------------------------ views, stats
extern "C" nrt_status nrt_get_layer(const nrt_cache* c, int32_t layer, const float** rows, int64_t* n_rows, int64_t* ld) {
    REQUIRE(c && rows && n_rows && ld, "null argument");
    REQUIRE(layer >= 0 && layer <= c->L, "layer out of range");
    if (!c->H[layer]) { nrt_set_error("the rows of hidden layers are not kept with aggregate-only storage"); return NRT_ERR_UNSUPPORTED; }
    *rows = c->H[layer];
    *n_rows = c->g->n;
    *ld = c->dims[layer];
    return NRT_OK;
}
extern "C" nrt_status nrt_get_aggregate(const nrt_cache* c, int32_t layer, const float** rows, int64_t* n_rows,
                                        int64_t* width) {
    REQUIRE(c && rows && n_rows && width, "null argument");
    REQUIRE(layer >= 1 && layer <= c->L, "layer out of range");
    *rows = c->S[layer];
    *n_rows = c->g->n;
    *width = c->dagg[layer];
    return NRT_OK;
}
extern "C" nrt_status nrt_get_layer_affected(const nrt_cache* c, int32_t layer, const int32_t** ids, int64_t* n) {
    REQUIRE(c && ids && n, "null argument");
    REQUIRE(layer >= 1 && layer <= c->L, "layer out of range");
    *ids = c->list[layer];
    *n = c->n_list[layer];
    return NRT_OK;
}
// ------------------------------------------------------------------ on-demand mode
// Recompute, layer by layer, the vertices listed in c->list[l] (counts in c->lc[l].count) over their whole
// in-neighbourhoods from the current h^{l-1}, and clear their stale bits.
static nrt_status recompute_listed(nrt_cache* c, hipStream_t s) {
    nrt_graph* g = c->g;
    const int64_t n = g->n;
    c->have_history_prev = false;            // the sizes of a query say nothing about the last batch's (no grid hints)
    for (int l = 1; l <= c->L; ++l) {
        NRT_TRY(k_dst_records(c->list[l], n, g->in, c->recs, c->hubs, &c->lc[l], false, nullptr, s));
        if (c->is_gat || agnn_family(c->kind)) {
            // constrained models (Section III-D): the rows of h^{l-1} brought up to date one layer below are re-projected
            // (layer 1 reads h^0, whose projections every batch keeps current), then the listed destinations are summed
            // over their whole in-neighbourhoods
            const int64_t sb = l == 1 ? 0 : n;
            if (c->is_gat)
                NRT_TRY(run_gat_layer(c, l, c->list[l - 1], &c->lc[l - 1].count, sb, c->list[l], &c->lc[l].count, n, true, false,
                                      0, nullptr, 0, s));
            else
                NRT_TRY(run_agnn_layer(c, l, c->list[l - 1], &c->lc[l - 1].count, sb, c->list[l], &c->lc[l].count, n, false, 0, 0,
                                       nullptr, 0, s));
            NRT_TRY(k_clear_listed_bits(c->stale[l], c->list[l], &c->lc[l].count, n, s));
            continue;
        }
        NRT_TRY(run_gather(c, l, false, 0, false, 0, s));
        NRT_TRY(run_update(c, l, c->list[l], n, &c->lc[l].count, false, 0, nullptr, 0, false, s));
        if (c->MP[l] && l < c->L)                           // message rows follow every h row that is brought up to date
            NRT_TRY(run_transform(c, l, c->list[l], n, &c->lc[l].count, nullptr, false, s));
        NRT_TRY(k_clear_listed_bits(c->stale[l], c->list[l], &c->lc[l].count, n, s));
    }
    return NRT_OK;
}

static nrt_status finish_recompute(nrt_cache* c, int64_t* n_recomputed, hipStream_t s) {
    HIP_TRY(hipMemcpyAsync(c->lc_host, c->lc, LC_TOTAL * sizeof(LayerCtrs), hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    int64_t tot = 0;
    for (int l = 1; l <= c->L; ++l) {
        tot += (int64_t)c->lc_host[l].count;
        if ((int64_t)c->lc_host[l].n_hubs > c->hubs.hub_cap || (int64_t)c->lc_host[l].n_items > c->hubs.item_cap ||
            (int64_t)c->lc_host[l].n_xhubs > c->xhub_cap) {
            nrt_set_error("internal: hub buffers too small");
            return NRT_ERR_STATE;
        }
    }
    if (n_recomputed) *n_recomputed = tot;
    c->have_history = false;        // the set sizes of this pass are not those of a batch
    return NRT_OK;
}

// The query of nrt_apply_batch_query, after the batch's hops have marked A_l stale (Section IV-D: the computation graph
// of an on-demand batch is the affected subgraph intersected with the K-hop subgraph of the queried vertices).
//   backwards  need_L = Q and stale_L;  need_{l-1} = stale_{l-1} and (need_l or in-neighbours(need_l))
//   forwards   a needed vertex that was up to date before the batch (`fold`, models whose message is h itself) takes the
//              incremental layer of Algorithm 1: its changed in-neighbours are all needed one layer below, where their
//              payload deltas were just produced, and the batch's structural terms are ready; a needed vertex that was
//              already stale is summed again over its whole in-neighbourhood.  Both kinds then run the dense update,
//              which also leaves the payload deltas for the next layer, and lose their stale mark.
// An up-to-date vertex has only up-to-date in-neighbours (the stale sets are closed under "out-neighbour at the next
// layer"), so what its cached aggregate holds of a source is exactly the cached row the delta is taken against.
static nrt_status serve_query_after_batch(nrt_cache* c, const QueryArgs& q, bool fold, hipStream_t s) {
    nrt_graph* g = c->g;
    const int64_t n = g->n;
    LayerCtrs* need = c->lc + LC_BATCH;
    LayerCtrs* fresh = need + (NRT_MAX_LAYERS + 1);
    LayerCtrs* redo = fresh + (NRT_MAX_LAYERS + 1);
    c->have_history_prev = false;
    CompactExtra cx;
    memset(&cx, 0, sizeof(cx));
    cx.err = &c->lc[0].pad[0];
    cx.coarse_shift = c->coarse_shift;
    cx.coarse_words = c->coarse_words;
    // ---- backwards: what the queried rows depend on
    NRT_TRY(k_compact(nullptr, c->bm_q, nullptr, c->need_bm[c->L], n, c->need_list[c->L], nullptr, c->cmp_state, c->cmp_state_len,
                      &need[c->L].count, s, c->stale[c->L], &cx));
    PullArgs no_pull;
    memset(&no_pull, 0, sizeof(no_pull));
    for (int l = c->L; l >= 2; --l) {
        NRT_TRY(k_expand_frontier(g->in, c->need_list[l], &need[l].count, n, c->flags, &need[l], c->xhub_list, c->xhub_cap, g->out,
                                  no_pull, s));
        NRT_TRY(k_compact(c->flags, c->need_bm[l], nullptr, c->need_bm[l - 1], n, c->need_list[l - 1], nullptr, c->cmp_state,
                          c->cmp_state_len, &need[l - 1].count, s, c->stale[l - 1], &cx));
    }
    // ---- forwards
    int prev = 0;
    for (int l = 1; l <= c->L; ++l) {
        const int cur = 1 - prev;
        // the needed set once more, now with its slot map and coarse copy (the next layer's sources)
        cx.coarse = c->coarse_shift <= 10 ? c->coarse[cur] : nullptr;
        NRT_TRY(k_compact(nullptr, c->need_bm[l], nullptr, c->bm[cur], n, c->need_list[l], c->slot[cur], c->cmp_state,
                          c->cmp_state_len, &need[l].count, s, nullptr, &cx));
        cx.coarse = nullptr;
        if (fold) {
            cx.and_invert = 1;
            NRT_TRY(k_compact(nullptr, c->need_bm[l], nullptr, c->bm[1 - cur], n, c->list_fresh, nullptr, c->cmp_state,
                              c->cmp_state_len, &fresh[l].count, s, c->stale_prev[l], &cx));
            cx.and_invert = 0;
            NRT_TRY(k_compact(nullptr, c->need_bm[l], nullptr, c->bm[1 - cur], n, c->list_redo, nullptr, c->cmp_state,
                              c->cmp_state_len, &redo[l].count, s, c->stale_prev[l], &cx));
            // layers that aggregate transformed rows: the rows brought up to date one layer below are transformed again
            // and leave the deltas the fold reads (layer 1: done with the batch, on the rows the batch replaced)
            if (c->MP[l - 1] && l >= 2)
                NRT_TRY(run_transform(c, l - 1, c->need_list[l - 1], n, &need[l - 1].count, c->DP[prev], false, s));
            // up to date before the batch: fold the deltas of the changed in-neighbours and the structural terms
            NRT_TRY(k_dst_records(c->list_fresh, n, g->in, c->recs, c->hubs, &fresh[l], false, nullptr, s));
            c->lc_use = &fresh[l];
            c->ov_bm = c->need_bm[l - 1];
            c->ov_slot = c->slot[prev];
            c->ov_dp = c->DP[prev];
            c->ov_count = l == 1 ? &c->lc[0].count : &need[l - 1].count;
            c->ov_coarse = c->coarse[prev];
            nrt_status st = run_gather(c, l, true, prev, false, 1, s);
            c->ov_bm = nullptr;
            if (st == NRT_OK) {                      // already stale: the whole in-neighbourhood again
                st = k_dst_records(c->list_redo, n, g->in, c->recs, c->hubs, &redo[l], false, nullptr, s);
                c->lc_use = &redo[l];
                if (st == NRT_OK) st = run_gather(c, l, false, 0, false, 0, s);
            }
            c->lc_use = nullptr;
            NRT_TRY(st);
            NRT_TRY(run_update(c, l, c->need_list[l], n, &need[l].count, true, cur, nullptr, 0, false, s));
        } else {
            NRT_TRY(k_dst_records(c->need_list[l], n, g->in, c->recs, c->hubs, &need[l], false, nullptr, s));
            c->lc_use = &need[l];
            nrt_status st = NRT_OK;
            if (c->is_gat || agnn_family(c->kind)) {
                const int64_t sb = l == 1 ? 0 : n;   // layer 1 reads h^0, whose projections every batch keeps current
                if (c->is_gat)
                    st = run_gat_layer(c, l, c->need_list[l - 1], &need[l - 1].count, sb, c->need_list[l], &need[l].count, n, true,
                                       false, 0, nullptr, 0, s);
                else
                    st = run_agnn_layer(c, l, c->need_list[l - 1], &need[l - 1].count, sb, c->need_list[l], &need[l].count, n, false,
                                        0, 0, nullptr, 0, s);
            } else {
                st = run_gather(c, l, false, 0, false, 0, s);
                if (st == NRT_OK) st = run_update(c, l, c->need_list[l], n, &need[l].count, false, 0, nullptr, 0, false, s);
                if (st == NRT_OK && c->MP[l] && l < c->L)
                    st = run_transform(c, l, c->need_list[l], n, &need[l].count, nullptr, false, s);
            }
            c->lc_use = nullptr;
            NRT_TRY(st);
        }
        NRT_TRY(k_clear_listed_bits(c->stale[l], c->need_list[l], &need[l].count, n, s));
        prev = cur;
    }
    return k_gather_rows_checked(q.rows, c->H[c->L], q.ids, q.n, n, c->dims[c->L], s);
}

extern "C" nrt_status nrt_set_lazy(nrt_cache* c, int32_t on, void* stream) {
    REQUIRE(c, "null argument");
    if (c->agg_only) {
        nrt_set_error("on-demand mode is not available with aggregate-only storage");
        return NRT_ERR_UNSUPPORTED;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (c->lazy && !on) {            // bring every stale vertex up to date before batches are applied eagerly again
        nrt_graph* g = c->g;
        const int64_t n = g->n;
        NRT_TRY(k_fill_u64((uint64_t*)c->lc, LC_TOTAL * sizeof(LayerCtrs) / 8, 0, s));
        for (int l = 1; l <= c->L; ++l)
            NRT_TRY(k_compact(nullptr, c->stale[l], nullptr, c->bm[0], n, c->list[l], nullptr, c->cmp_state, c->cmp_state_len,
                              &c->lc[l].count, s));
        NRT_TRY(recompute_listed(c, s));
        NRT_TRY(finish_recompute(c, nullptr, s));
    }
    c->lazy = on ? 1 : 0;
    return NRT_OK;
}

extern "C" nrt_status nrt_query(nrt_cache* c, const int32_t* query_ids, int64_t n_query, float* rows,
                                int64_t* n_recomputed, void* stream) {
    REQUIRE(c && n_query >= 0 && (n_query == 0 || (query_ids && rows)), "null argument or negative count");
    if (n_recomputed) *n_recomputed = 0;
    if (n_query == 0) return NRT_OK;
    nrt_graph* g = c->g;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t n = g->n;
    const int64_t nw = (n + 31) / 32;
    LayerCtrs* spare = &c->lc[NRT_MAX_LAYERS + 1];          // count = n_query for the final row gather; in_edges[0] = bad-id flag
    NRT_TRY(k_fill_u64((uint64_t*)c->lc, LC_TOTAL * sizeof(LayerCtrs) / 8, 0, s));
    NRT_TRY(k_fill_u64(&spare->count, 1, (uint64_t)n_query, s));
    if (c->lazy) {
        // ---- which stale vertices do the queried embeddings depend on?  Backwards from the last layer:
        // need_L = Q and stale_L;  need_{l-1} = stale_{l-1} and (need_l or in-neighbours(need_l))
        NRT_TRY(k_fill_u32(c->bm_feat, nw, 0, s));
        NRT_TRY(k_mark_ids(c->bm_feat, query_ids, n_query, n, (int32_t*)&spare->in_edges[0], s));
        int cur = 0;
        NRT_TRY(k_compact(nullptr, c->bm_feat, nullptr, c->bm[cur], n, c->list[c->L], nullptr, c->cmp_state, c->cmp_state_len,
                          &c->lc[c->L].count, s, c->stale[c->L]));
        PullArgs no_pull;
        memset(&no_pull, 0, sizeof(no_pull));
        for (int l = c->L; l >= 2; --l) {
            // the in-lists play the part of out-lists: flags[u] = 1 for every in-neighbour u of need_l
            NRT_TRY(k_expand_frontier(g->in, c->list[l], &c->lc[l].count, n, c->flags, &c->lc[l], c->xhub_list, c->xhub_cap,
                                      g->out, no_pull, s));
            NRT_TRY(k_compact(c->flags, c->bm[cur], nullptr, c->bm[1 - cur], n, c->list[l - 1], nullptr, c->cmp_state,
                              c->cmp_state_len, &c->lc[l - 1].count, s, c->stale[l - 1]));
            cur = 1 - cur;
        }
        NRT_TRY(recompute_listed(c, s));
    } else {
        NRT_TRY(k_fill_u32(c->bm_feat, nw, 0, s));
        NRT_TRY(k_mark_ids(c->bm_feat, query_ids, n_query, n, (int32_t*)&spare->in_edges[0], s));   // only validates the ids
    }
    // rows of the queried vertices (ids already range-checked: a bad id makes the whole call fail below, and the
    // gather skips nothing it should not read because such ids are replaced by vertex 0)
    NRT_TRY(k_gather_rows_checked(rows, c->H[c->L], query_ids, n_query, n, c->dims[c->L], s));
    NRT_TRY(finish_recompute(c, n_recomputed, s));
    if (c->lc_host[NRT_MAX_LAYERS + 1].in_edges[0] != 0) {
        nrt_set_error("query id out of range");
        return NRT_ERR_INVALID_ARG;
    }
    return NRT_OK;
}

extern "C" nrt_status nrt_set_mode(nrt_cache* c, int32_t mode) {
    REQUIRE(c, "null argument");
    REQUIRE(mode == NRT_MODE_INCREMENTAL || mode == NRT_MODE_RECOMPUTE || mode == NRT_MODE_FULL || mode == NRT_MODE_AUTO,
            "unknown mode");
    // (GAT and RGAT recompute from the cached projections z, GIN, GraphSAGE and CommNet from the message tables, which are kept for every vertex)
    if (c->agg_only && c->kind == NRT_GCN && (mode == NRT_MODE_RECOMPUTE || mode == NRT_MODE_FULL)) {
        nrt_set_error("with aggregate-only storage the hidden rows that recomputation reads are not kept");
        return NRT_ERR_UNSUPPORTED;
    }
    c->mode = mode;
    return NRT_OK;
}
extern "C" nrt_status nrt_measure_stream(int32_t kind, float* b, const float* a, int64_t n_floats, int32_t reps, void* stream,
                                         float* ms_per_pass) {
    REQUIRE(a && b && ms_per_pass, "null argument");
    REQUIRE(kind == 0 || kind == 1, "kind must be 0 (copy) or 1 (read)");
    REQUIRE(n_floats >= 4 && reps >= 1, "need n_floats >= 4 and reps >= 1");
    REQUIRE(((reinterpret_cast<uintptr_t>(a) | reinterpret_cast<uintptr_t>(b)) & 15) == 0, "buffers must be 16-byte aligned");
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipEvent_t e0, e1;
    HIP_TRY(hipEventCreate(&e0));
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); nrt_set_error("hipEventCreate failed"); return NRT_ERR_DEVICE; }
    auto run = [&]() -> nrt_status {
        NRT_TRY(kind == 0 ? k_stream_copy(b, a, n_floats, s) : k_stream_read(b, a, n_floats, s));     // untimed first pass
        HIP_TRY(hipEventRecord(e0, s));
        for (int r = 0; r < reps; ++r) NRT_TRY(kind == 0 ? k_stream_copy(b, a, n_floats, s) : k_stream_read(b, a, n_floats, s));
        HIP_TRY(hipEventRecord(e1, s));
        HIP_TRY(hipEventSynchronize(e1));
        float ms = 0.f;
        HIP_TRY(hipEventElapsedTime(&ms, e0, e1));
        *ms_per_pass = ms / (float)reps;
        return NRT_OK;
    };
    const nrt_status st = run();
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return st;
}

extern "C" nrt_status nrt_set_profiling(nrt_cache* c, int32_t on) {
    REQUIRE(c, "null argument");
    if (on && !c->events_made) {
        for (int i = 0; i < MAX_EVENTS; ++i) HIP_TRY(hipEventCreate(&c->ev[i]));
        c->events_made = true;
    }
    c->profiling = on ? 1 : 0;
    return NRT_OK;
}
extern "C" nrt_status nrt_get_stats(const nrt_cache* c, nrt_stats* out) {
    REQUIRE(c && out, "null argument");
    *out = c->stats;
    return NRT_OK;
}
