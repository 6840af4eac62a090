// Internal declarations shared by the HIP sources of libnrt (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <string.h>
#include "nrt.h"

#define NRT_WAVE 64
// layout of the device counter block (int64 cells) mirrored to pinned host memory in one copy
enum { CTR_GROW = 0 /*2*/, CTR_HEAD_OUT = 8, CTR_HEAD_IN = 9, CTR_ERR = 16 /*8 x int32*/, CTR_COUNT = 24,
       CTR_PLAN_TOTAL = 25 /* updates that entered the batch plan */, NRT_NCTRS = 64 };
#define NRT_COARSE_WORDS 6144  // 24 KiB of LDS for the coarse changed-source filter of the sparse gather
#define NRT_CHUNK 256          // in-list entries per gather work item (one wave each)

// ---------------------------------------------------------------- error plumbing (api.hip)
void nrt_set_error(const char* fmt, ...);
#define HIP_TRY(expr)                                                                      \
    do {                                                                                   \
        hipError_t _e = (expr);                                                            \
        if (_e != hipSuccess) {                                                            \
            nrt_set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(_e), __FILE__, __LINE__); \
            return NRT_ERR_DEVICE;                                                         \
        }                                                                                  \
    } while (0)
#define NRT_TRY(expr)                     \
    do {                                  \
        nrt_status _s = (expr);           \
        if (_s != NRT_OK) return _s;      \
    } while (0)
// kernel launches issued by the calling thread since the counter was last cleared (a statistic of nrt_get_stats)
extern thread_local int64_t nrt_launch_count;
#define LAUNCH_CHECK() do { ++nrt_launch_count; HIP_TRY(hipGetLastError()); } while (0)

static inline int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }

// ---------------------------------------------------------------- workspace bump allocator
struct Bump {
    char* base;      // may be null when only sizing
    size_t used;
    template <typename T>
    T* take(size_t count) {
        used = (used + 255) & ~size_t(255);
        T* p = base ? reinterpret_cast<T*>(base + used) : nullptr;
        used += count * sizeof(T);
        return p;
    }
};

// ---------------------------------------------------------------- adjacency in one direction
// Vertex v owns pool[off[v] .. off[v]+cap[v]) of which the first deg[v] entries are live.
struct Adj {
    int64_t* off;
    int32_t* deg;
    int32_t* cap;
    int32_t* idx;      // pool of neighbour ids
    float* wts;        // pool of weights or null
    int64_t pool_cap;
    int64_t* head;     // device counter: first free pool entry
};

struct nrt_graph {
    int64_t n, e, e_capacity;
    int weighted;
    Adj out, in;       // out: keyed by source, holds destinations; in: keyed by destination, holds sources
    // scan scratch shared by graph and cache kernels
    uint64_t* scan_tmp;   // block sums
    int64_t scan_tmp_len;
    int32_t* stamp[2];    // per-direction ownership stamps for batch mutation
    int32_t* inscnt[2];   // per-direction per-vertex pending insert counts (zero between batches)
    int32_t* delcnt[2];
    int32_t epoch;
    int64_t* host_pinned; // small pinned read-back area (64 int64)
    int64_t* dev_ctrs;    // device counters mirrored into host_pinned (64 int64)
    bool has_cache;
};

// ---------------------------------------------------------------- per-layer device counters
// Sizes that only the device knows while a batch is in flight.  Kernels read them from here and size their
// own loops, so the host launches fixed or bounded grids and synchronises once, at the end of the batch.
struct LayerCtrs {
    uint64_t count;        // |list| : affected vertices of the layer (layer 0: sources of change of layer 1)
    uint64_t n_hubs;       // destinations with more than NRT_CHUNK in-edges
    uint64_t n_items;      // their items of NRT_CHUNK in-list entries
    uint64_t n_xhubs;      // sources with a long out-list queued by the expansion
    uint64_t in_edges[16]; // in-edges of the affected vertices (a statistic, spread over cells)
    uint64_t n_pull_long;  // vertices queued by the pull-direction expansion for its second pass
    uint64_t pad[3];
};

// ---------------------------------------------------------------- prims.hip
nrt_status k_fill_u32(uint32_t* p, int64_t n, uint32_t v, hipStream_t s);
// several fills in one launch (a batch clears a dozen small scratch areas; separate launches would cost more than the stores)
struct FillJob { uint32_t* p; int64_t n; uint32_t v; };      // n 32-bit words
struct FillJobs {
    FillJob j[16];
    int count;
    void add(void* p, int64_t n_words, uint32_t v = 0) { if (n_words > 0 && count < 16) { j[count].p = (uint32_t*)p; j[count].n = n_words; j[count].v = v; ++count; } }
};
nrt_status k_multi_fill(const FillJobs& f, hipStream_t s);
// dst[i][:] = src[list[i]][:] for i < min(*count, cap); rows of D floats, D a multiple of 4
nrt_status k_gather_rows(float* dst, const float* src, const int32_t* list, const uint64_t* count, int64_t cap, int64_t bound,
                         int D, hipStream_t s);
nrt_status k_fill_u64(uint64_t* p, int64_t n, uint64_t v, hipStream_t s);
nrt_status k_or_words(uint32_t* dst, const uint32_t* a, const uint32_t* b, int64_t nwords, hipStream_t s);
nrt_status k_copy_i32(int32_t* dst, const int32_t* src, int64_t n, hipStream_t s);
// dst = [a | b] with every id outside [0, n) replaced by 0
nrt_status k_concat_ids(int32_t* dst, const int32_t* a, int64_t na, const int32_t* b, int64_t nb, int64_t n, hipStream_t s);
nrt_status k_copy_f32(float* dst, const float* src, int64_t n, hipStream_t s);
// dst[0 .. min(*count, cap)) = src[...]
nrt_status k_copy_counted_i32(int32_t* dst, const int32_t* src, const uint64_t* count, int64_t cap, int64_t bound, hipStream_t s);
// exclusive scan of n uint64 values in place; writes the total to *total (device)
nrt_status k_exclusive_scan_u64(uint64_t* data, int64_t n, uint64_t* tmp, int64_t tmp_len, uint64_t* total, hipStream_t s);
// Compaction of a vertex set into a sorted id list, in one launch.  The set is the union of the byte flags (one byte
// per vertex, may be null; they are cleared on the way), and up to two bitmaps or_a, or_b (may be null), intersected
// with and_mask when given.  Writes the set as bitmap `out_bm`, its sorted ids to `list`, slot[id] = position (slot
// may be null), *count = size.  `state` (state_len >= n / 8192 + 3 cells, zero before its first use, used by nothing
// else) carries the look-back of the workgroups from call to call.
struct CompactExtra {
    int32_t* list2; int64_t cap2;     // second copy of the first cap2 ids (the caller's output buffer), or null
    uint32_t* coarse;                 // coarse copy of the set for the sparse gather's LDS filter, or null
    int coarse_shift; int64_t coarse_words;
    uint64_t* err;                    // raised if a look-back wait gave up (device), or null
    int and_invert;                   // intersect with the complement of and_mask instead
};
nrt_status k_compact(uint8_t* flags, const uint32_t* or_a, const uint32_t* or_b, uint32_t* out_bm, int64_t n,
                     int32_t* list, int32_t* slot, uint64_t* state, int64_t state_len, uint64_t* count, hipStream_t s,
                     const uint32_t* and_mask = nullptr, const CompactExtra* extra = nullptr);
// dst[i][:] = src[ids[i]][:] for i < n_ids (host count); an id outside [0, n) reads row 0
nrt_status k_gather_rows_checked(float* dst, const float* src, const int32_t* ids, int64_t n_ids, int64_t n, int D,
                                 hipStream_t s);
// bm |= ids; an id outside [0, n) sets *bad (device) instead
nrt_status k_mark_ids(uint32_t* bm, const int32_t* ids, int64_t n_ids, int64_t n, int32_t* bad, hipStream_t s);
// typed edges: *bad = 1 when a weight is not an integer relation id in [0, R) (w: a plain array; a: the live list entries)
nrt_status k_check_relations(const float* w, int64_t count, int R, int32_t* bad, hipStream_t s);
nrt_status k_check_list_relations(const Adj& a, int64_t n, int R, int32_t* bad, hipStream_t s);
// bm &= ~(list[0 .. *count))
nrt_status k_clear_listed_bits(uint32_t* bm, const int32_t* list, const uint64_t* count, int64_t bound, hipStream_t s);

// streaming kernels for the bandwidth ceilings reported beside the gathers: copy a -> b, or read a (b receives nothing)
nrt_status k_stream_copy(float* b, const float* a, int64_t n_floats, hipStream_t s);
nrt_status k_stream_read(float* b, const float* a, int64_t n_floats, hipStream_t s);

// ---------------------------------------------------------------- frontier.hip
// flags[v] = 1 for every out-neighbour v of the sources src_list[0 .. *ns_dev) that is not itself a source
// (sources may or may not get their flag: the caller ORs the source set in afterwards).
struct PullArgs {              // pull direction of the hop, used when the source set is a large part of the graph
    int allowed;               // host hint: the previous batch had a large source set at this hop
    int64_t n;                 // vertices
    const uint32_t* src_bitmap;   // the source set as a bitmap
    int32_t* long_list;        // [long_cap] vertices handed from the first to the second pull pass
    int64_t long_cap;
    unsigned long long* long_count;   // device counter, zero on entry
};
nrt_status k_expand_frontier(const Adj& out, const int32_t* src_list, const uint64_t* ns_dev, int64_t ns_bound,
                             uint8_t* flags, LayerCtrs* lc, int32_t* xhub_list, int64_t xhub_cap, const Adj& in,
                             const PullArgs& pull, hipStream_t s);

// ---------------------------------------------------------------- gather.hip
// What a gather wave needs to know about destination slot s, in one 16-byte load.
struct __attribute__((aligned(16))) DstRec {
    int64_t off;   // first pool entry of the in-list
    int32_t deg;   // live entries
    int32_t v;     // vertex id
};
// Destinations with more than NRT_CHUNK in-edges ("hubs") are cut into items of NRT_CHUNK entries.
struct HubWork {
    int32_t* hub_slot;     // [hub_cap] destination slots of the hubs (unordered)
    uint64_t* hub_first;   // [hub_cap] first item of each hub
    int32_t* item_hub;     // [item_cap] hub index of an item
    int32_t* item_chunk;   // [item_cap] chunk index inside the hub's in-list
    int64_t hub_cap, item_cap;
    float* partial;        // [item_cap][D] one partial row per item
};
// relation id held in an edge weight, clamped into [0, R) so that a bad id can never address outside the table
__host__ __device__ inline int nrt_rel_of(float w, int R) {
    int r = (int)w;
    return r < 0 ? 0 : (r >= R ? R - 1 : r);
}

struct GatherArgs {
    const DstRec* recs;        // [*count]
    HubWork hubs;
    const LayerCtrs* lc;       // count, n_hubs, n_items of the destination layer
    Adj in;
    const float* P;            // source rows of width D
    int D;
    const uint32_t* src_bitmap; // null: every source contributes and row index = vertex id
    const int32_t* src_slot;
    const uint64_t* n_src_dev; // number of changed sources; the launch does nothing when it is 0 (null: not checked)
    int src_scale_gcn;         // multiply each source row by 1/sqrt(indeg[u]+1) (full forward, GCN)
    int use_weights;           // multiply by the edge weight
    int rel_R;                 // > 0 (RGCN): the edge weight holds a relation id r and source row i is row i * rel_R + r of P,
                               // taken with coefficient 1 (P holds rel_R message rows per source)
    int self_pair;             // GCN: the destination's own row is one more neighbour
    int accumulate;            // 1: S[v] += sum, 0: S[v] = sum
    float* S;                  // [N][D]
    unsigned long long* pair_ctr; // null or 1024 counters
    // structural terms of the batch (inserted / deleted in-edges), one compact row per destination of an updated
    // edge, added by the wave that owns the destination (null: none)
    const float* sd;
    const uint32_t* dd_bitmap; // destinations of updated edges
    const int32_t* dd_slot;    // their rows in sd
    // cancellation guard: when a fold removes most of a row's magnitude the row is rebuilt from the full
    // in-neighbourhood, rows read from Pfull (the current h^{l-1})
    int guard;
    const float* Pfull;
    int full_scale_gcn;
    // layers whose changed sources are few are served by the short-instruction variant of the gather:
    // 0 never, 1 the device counters decide (both kernels are launched), 2 always (only that kernel is launched)
    int sparse_ok;
    int64_t n_vertices;
    // Automatic choice per layer between folding deltas and recomputing the affected aggregates from h^{l-1}: when
    // the changed sources are a large part of the graph nearly every in-edge carries a delta, so recomputation reads
    // the same rows without slot lookups, without reading the old aggregate, and spares the previous layer's
    // write-back its payload deltas.  auto_role 1: this launch folds deltas and yields when 4 * changed > n_vertices;
    // auto_role 2: this launch recomputes and runs only then; 0: no test.  auto_src_dev: the changed-source count.
    int auto_role;
    const uint64_t* auto_src_dev;
    // What the previous batch had at this layer (0: unknown).  The kernels stride over their work with whatever grid they
    // get; on small layers a grid sized to the expected work saves the time a large one takes merely to start and exit.
    int64_t units_hint;        // destinations + hub items
    int64_t hubs_hint;         // destinations with long in-lists
    const uint32_t* coarse;    // coarse copy of src_bitmap: bit i covers vertices [i << coarse_shift, (i+1) << coarse_shift)
    int coarse_shift;
    int coarse_words;          // at most NRT_COARSE_WORDS
};
// destination records of list[0 .. *count) (list null: all n vertices), hub list and hub items; fills lc
// `plain_if_zero` (may be null): when the device counter it points to is 0, long in-lists are not cut into items
nrt_status k_dst_records(const int32_t* list, int64_t bound, const Adj& in, DstRec* recs, const HubWork& hubs,
                         LayerCtrs* lc, bool all_vertices, const uint64_t* plain_if_zero, hipStream_t s);
nrt_status k_gather(const GatherArgs& a, hipStream_t s);
nrt_status k_coarse_bitmap(const uint32_t* fine, int64_t n, int shift, uint32_t* coarse, int64_t n_words, hipStream_t s);
nrt_status k_combine_partials(const GatherArgs& a, hipStream_t s);

// ---------------------------------------------------------------- plan.hip
struct PlanArgs {   // the batch's edge updates grouped by destination in a fixed order (see plan.hip)
    int64_t n_ins, n_del, n;
    const int32_t *ins_src, *ins_dst, *del_src, *del_dst;
    const uint32_t* dst_bitmap;    // destinations of the updates (more than 2048 updates: the slots come from it)
    uint32_t* scratch_bm;          // [n / 32] scratch of the compaction
    int32_t* list;                 // [updates] destination of a slot, ascending
    int32_t* slot_of;              // [n] vertex -> slot (only entries of this batch's destinations are current)
    int32_t* off;                  // [updates + 1] first position of a slot's run in ord
    int32_t* ord;                  // [updates] update numbers, run by run
    int32_t* ins_cnt;              // [updates] inserts in a slot's run
    int32_t* ins_rank;             // [n_ins] rank of an insert among the inserts of its destination
    uint64_t* count;               // device: number of slots
    // scratch of the form for more than 2048 updates (zero on entry: off64, cursor)
    uint64_t* off64;               // [updates + 1]
    int32_t* cursor;               // [updates]
    int32_t* tmp;                  // [updates]
    uint64_t* total;               // device: updates that entered the plan
    uint64_t* cmp_state; int64_t cmp_state_len;   // look-back cells of the compaction (k_compact)
};
nrt_status k_batch_plan(const PlanArgs& a, uint64_t* scan_tmp, int64_t scan_tmp_len, hipStream_t s);

struct FoldArgs {   // structural terms of a batch, evaluated on the pre-update caches, one owner wave per destination
    int64_t n_ins, n_del, n;
    const uint64_t* n_slots;      // the batch plan: number of destinations, their runs of updates
    const int32_t* off;
    const int32_t* ord;
    const int32_t *ins_src, *ins_dst, *del_src, *del_dst;
    const float *ins_w, *del_w;  // null when unweighted
    int rel_R;                   // > 0 (RGCN): the weights are relation ids and pick one of rel_R rows per source, coefficient 1
    int n_layers;                // blockIdx.y walks the layers
    const float* Hprev[NRT_MAX_LAYERS];   // h^{l-1} (old)
    float* SD[NRT_MAX_LAYERS];            // compact structural-delta rows, one per destination of an updated edge (plan slot)
    int D[NRT_MAX_LAYERS];
    const int32_t* indeg_old;    // for the GCN payload scale, else null
    int compact_src[NRT_MAX_LAYERS];      // Hprev[l] holds one row per updated edge (inserts first) instead of one per vertex
};
nrt_status k_structural_fold(const FoldArgs& a, hipStream_t s);

struct DeltaArgs {  // layer-0 delta payloads and feature scatter
    const int32_t* list; const uint64_t* n_dev; int64_t bound;
    const uint32_t* feat_bitmap; const int32_t* feat_index; const float* feat_rows;
    float* H0; float* DP; int D;
    const int32_t* indeg_new; const int32_t* indeg_old;   // GCN payload scale, else null
    int store_old;                  // DP receives the replaced row itself instead of new - old (A-GNN: old h^0)
};
nrt_status k_layer0_delta(const DeltaArgs& a, hipStream_t s);

// ---------------------------------------------------------------- gemm.hip
enum { A_PLAIN = 0, A_SCALE_GCN = 1, A_CONCAT_MEAN = 2, A_AXPY = 3, A_PLAIN_ADD = 4, A_AXPY_BIAS_RELU = 5 };
struct GemmArgs {
    int64_t M; int K; int N;        // K = total inner width (CONCAT: 2*K0); M is a bound when M_dev is given
    const uint64_t* M_dev;          // number of rows on the device, or null
    int64_t out_cap;                // rows that fit in out_compact
    const int32_t* rows;            // null: row m is vertex m
    int a_is_compact;               // A rows are already compact (row m), rows[] only addresses the write-back
    int a_mode;
    const float* P0; const float* P1; int ldp;   // source rows (width ldp each)
    float axpy_c;                   // A_AXPY: c*P0 + P1
    const float* a_bias;            // A_AXPY_BIAS_RELU: [K], the operand is ReLU(c*P0 + P1 + a_bias)
    const float* add;               // A_PLAIN_ADD: before the activation y += add[v][:] / add_indeg[v] (RGCN: W_o h_v + mean message);
    const int32_t* add_indeg;       // rows of width N by vertex; a zero count adds nothing; null add_indeg: the rows themselves
    const int32_t* indeg;           // for A_SCALE_GCN / A_CONCAT_MEAN
    const float* Wt;                // transposed weights [N][K]
    int ldw;                        // floats between consecutive rows of Wt (0: K); a column block of a wider matrix otherwise
    const float* bias;              // [N] or null
    int act;                        // 0 none, 1 relu, 2 elu
    // epilogue
    float* out_compact;             // [M][N] or null
    float* H;                       // [.][N] scattered by vertex or null
    float* DP;                      // [M][N] delta payload for the next layer or null
    const int32_t* indeg_old;       // GCN payload scale for DP (with indeg as new), else null
    int dp_scale_gcn;
    int dp_store_old;               // DP receives the overwritten row of H instead of a payload delta (GAT: old z)
    int dp_no_h;                    // H null (rows of the layer are not kept): 1: DP = -(old payload), computed from the
                                    // aggregate before the fold; 2: DP += new payload, computed after it
    int dp_skip_large;              // leave DP (and the read of the old rows) out when 4 * rows > n_vertices
    int64_t n_vertices;
};
nrt_status k_gemm(const GemmArgs& a, hipStream_t s);
// The write-back of k_gemm without a product, on the listed rows, P0 of width N: y = act(P0[v] / sqrt(indeg(v)+1) + bias)
// with a degree vector (a GCN layer whose weights were applied to the messages before the aggregation), or
// y = act(P0[v] + bias + add[v] / add_indeg(v)) without one (GraphSAGE, CommNet: both halves of the weights applied
// before the aggregation); H, DP, out_compact as for k_gemm
nrt_status k_rowwise_update(const GemmArgs& a, hipStream_t s);
nrt_status k_transpose(const float* W, float* Wt, int K, int N, hipStream_t s);   // Wt[n][k] = W[k][n]

// ---------------------------------------------------------------- gat.hip
struct GatArgs {
    const int32_t* rows;            // listed vertices (null: all n)
    const uint64_t* n_rows_dev;     // their number on the device (with rows)
    int64_t rows_bound;             // launch bound for the listed rows
    int64_t n;
    int heads, head_dim;
    int rel;                        // 1 (RGAT): the heads are relations, an edge joins only the group of its relation (its
                                    // weight), and the layer output is the sum of the groups (width head_dim)
    float slope;
    const float* att_src; const float* att_dst;   // [heads][head_dim]
    float* Z;                       // [N][D] current z = x W
    float* AS; float* AD;           // [N][heads] attention scalars
    float* AS_old;                  // [rows][heads] compact: scalars before this batch (k_gat_scalars writes, gather reads)
    const float* Z_old;             // [rows][D] compact: z before this batch
    // gather only: destination records, hub items and counters of the destination layer
    const DstRec* recs;
    HubWork hubs;
    const LayerCtrs* lc;
    float* part_m; float* part_den; // [item_cap][heads] partial max / sum of hub items
    Adj in;
    const uint32_t* src_bitmap;     // vertices whose z changed (null: full forward for every row)
    const int32_t* src_slot;        // their slots in Z_old / AS_old
    const uint32_t* ddst_bitmap;    // destinations of updated edges
    // structural terms of the batch for those destinations (Algorithm 3 applied to edge updates): compact rows,
    // one per destination of an updated edge, holding minus the old attention terms of its deleted in-edges
    // relative to the destination's cached bound m; its inserted in-edges are the last ins_cnt entries of its in-list
    const int32_t* dd_slot;         // vertex -> row of sd_s / sd_den / ins_cnt
    const float* sd_s;              // [rows][D]
    const float* sd_den;            // [rows][heads]
    const int32_t* ins_cnt;         // [rows]
    const uint64_t* n_src_dev;      // number of vertices whose z changed in this layer (gather, incremental)
    unsigned long long* pair_ctr;   // null or 1024 counters: z rows fetched by the gather (a statistic)
    float* M; float* DEN;           // [N][heads]
    float* S;                       // [N][D]
    float* Hout;                    // [N][D] layer output ([N][head_dim] with rel); null: the rows are not kept by vertex
                                    // (aggregate-only storage), out_rows then carries them to the next layer
    const float* bias; int act;
    float* out_rows; int64_t out_cap;
};
nrt_status k_gat_scalars(const GatArgs& a, hipStream_t s);
struct GatFoldArgs {   // structural terms of a batch for GAT, evaluated on the pre-update caches, all layers in one launch
    int64_t n_ins, n_del, n;
    const int32_t *del_src, *del_dst;
    const float* del_w;         // RGAT: relation ids of the deleted edges (a deleted edge leaves only its relation's group), else null
    const uint64_t* n_slots;    // the batch plan: destinations, their runs of updates (inserts first)
    const int32_t* off;
    const int32_t* ord;
    const int32_t* list;        // destination vertex of a slot
    int n_layers, heads, head_dim;
    float slope;
    const float* Z[NRT_MAX_LAYERS]; const float* AS[NRT_MAX_LAYERS]; const float* AD[NRT_MAX_LAYERS];
    const float* M[NRT_MAX_LAYERS];
    float* SDS[NRT_MAX_LAYERS]; float* SDDEN[NRT_MAX_LAYERS];
};
nrt_status k_gat_structural_fold(const GatFoldArgs& a, hipStream_t s);
nrt_status k_gat_gather(const GatArgs& a, hipStream_t s);

// ---------------------------------------------------------------- agnn.hip
struct AgnnArgs {
    const DstRec* recs;             // destination records, hub items and counters of the destination layer
    HubWork hubs;
    const LayerCtrs* lc;
    Adj in;
    const float* H;                 // [N][D] h^{l-1}, current
    const float* R;                 // [N] inverse norms of its rows (0 for a zero row)
    int D;
    float beta;                     // the layer's scalar w
    int incremental;                // 0: every destination is summed over its whole in-list
    const uint32_t* src_bitmap;     // vertices whose h^{l-1} changed (incremental)
    const int32_t* src_slot;        // their rows in old_rows / old_r
    const float* old_rows;          // [changed][D] compact: h^{l-1} before this batch
    const float* old_r;             // [changed] compact: inverse norms before this batch
    const float* sd;                // structural terms, one compact row per destination of an updated edge (or null)
    const uint32_t* dd_bitmap;
    const int32_t* dd_slot;
    float* S;                       // [N][D] cached aggregate
    unsigned long long* pair_ctr;   // null or 1024 counters: rows of h fetched (a statistic)
    int gate;                       // G-GCN: element-wise gate sigmoid(P1[u] + P2[v]) instead of the cosine
    const float* P1; const float* P2;   // [N][D] W_1 h and W_2 h, current
    const float* old_p1;            // [changed][D] compact: W_1 h before this batch
};
struct AgnnFoldArgs {   // structural terms of a batch, evaluated on the pre-update caches, all layers in one launch
    int64_t n_ins, n_del, n;
    const int32_t *ins_src, *del_src;
    const uint64_t* n_slots;        // the batch plan: destinations, their runs of updates
    const int32_t* off;
    const int32_t* ord;
    const int32_t* list;            // destination vertex of a slot
    int n_layers;
    const float* H[NRT_MAX_LAYERS];   // h^{l-1} (old)
    const float* R[NRT_MAX_LAYERS];   // its inverse norms (old)
    float* SD[NRT_MAX_LAYERS];
    int D[NRT_MAX_LAYERS];
    float beta[NRT_MAX_LAYERS];
    int gate;                         // G-GCN
    const float* P1[NRT_MAX_LAYERS]; const float* P2[NRT_MAX_LAYERS];
};
// R[v] = 1/|H[v]| for v in list[0 .. *count_dev) (list null: rows 0 .. bound); r_old[m] (may be null) keeps the old value
nrt_status k_agnn_norms(const int32_t* list, const uint64_t* count_dev, int64_t bound, const float* H, int D, float* R,
                        float* r_old, hipStream_t s);
nrt_status k_agnn_gather(const AgnnArgs& a, hipStream_t s);
nrt_status k_agnn_combine(const AgnnArgs& a, hipStream_t s);   // after the gather, same arguments: destinations with long in-lists
nrt_status k_agnn_structural_fold(const AgnnFoldArgs& a, hipStream_t s);

// ---------------------------------------------------------------- monet.hip
struct MonetArgs {
    const int32_t* rows;            // listed vertices (null: rows 0 .. bound)
    const uint64_t* count_dev;      // their number on the device (with rows)
    int64_t bound;
    const float* H; int d;          // [N][d] layer input
    int h_is_compact;               // H holds the listed rows only, in list order (rows[] addresses G alone)
    const float* muT; const float* precT;   // [d][J] transposed means and diagonal precisions
    int J;
    float* G;                       // [N][J] kernel responses, by vertex
    float* DP;                      // [listed][J] compact: new - old (or null)
};
nrt_status k_monet_transform(const MonetArgs& a, hipStream_t s);

// ---------------------------------------------------------------- graph.hip
nrt_status graph_layout(Bump& b, nrt_graph* g);
nrt_status graph_build(nrt_graph* g, const int64_t* csr_indptr, const int32_t* csr_indices, const float* csr_w,
                       const int64_t* csc_indptr, const int32_t* csc_indices, const float* csc_w, hipStream_t s);
struct BatchScratch {
    int64_t max_edges;
    uint64_t* hash_keys; int64_t hash_cap;     // open-addressing set of (src<<32|dst), tag in bit 63 for deletes
    int64_t* pos_out; int64_t* pos_in;          // per deleted edge: pool positions in both directions
    float* del_w;                               // per deleted edge: its weight before deletion
    int32_t* err;                               // device error flags [8] (inside the counter block)
    int32_t* feat_index;                        // [N] position of a vertex in the batch's feature list
    int32_t* feat_stamp;                        // [N] epoch stamps that detect repeated feature ids
    // the sets of the batch, marked while it is validated (both cleared by the validation's fill launch; null: not wanted)
    uint32_t* bm_dst;                           // destinations of the edge updates
    uint32_t* bm_feat;                          // vertices whose feature row is replaced
    // from the batch plan: where an inserted in-edge goes in its destination's list (reproducible list order)
    const int32_t* plan_slot_of;                // [N] vertex -> plan slot
    const int32_t* plan_ins_cnt;                // [slots] inserts per destination
    const int32_t* plan_ins_rank;               // [n_ins] rank of an insert among those of its destination
};
// validate (no state change); err flags and growth need are read back by the caller
// `clears`: scratch areas of the caller to zero in the same launch as the validation's own (may be null)
nrt_status graph_validate_batch(nrt_graph* g, const nrt_batch* b, BatchScratch& sc, const FillJobs* clears, hipStream_t s);
nrt_status graph_cancel_batch(nrt_graph* g, const nrt_batch* b, hipStream_t s);   // undo counters after a failed validation
nrt_status graph_mutate(nrt_graph* g, const nrt_batch* b, BatchScratch& sc, hipStream_t s);
