// Device-resident mutable directed graph: out-lists and in-lists with per-vertex slack.
//
// The paper keeps a packed-memory-array CSR in host memory (Section IV "Packed-memory-array-based CSR
// structure"); here both directions live in HBM.  Each vertex owns a segment [off, off+cap) of a pool, the
// first deg entries are live.  A batch (a) turns deleted entries into tombstones, (b) lets one workgroup per
// touched vertex (one wave for the short lists of a large batch) squeeze its list and, if the pending inserts do
// not fit, move the list to a fresh, larger segment at the pool head, (c) appends the inserted entries.
#include "common.h"

namespace {

constexpr int RB_THREADS = 1024;   // threads of a list-rebuild workgroup
constexpr int RB_EPT = 4;
constexpr int RB_FEW = 256;        // up to this many deletions a list is patched instead of squeezed
constexpr int VAL_THREADS = 1024; // threads of an edge-validation workgroup
constexpr int VAL_UNROLL = 4;     // independent list loads per thread and trip
constexpr int WAVE_LIST_MAX = 1024;        // longest list one wave searches or squeezes by itself
constexpr int64_t PACKED_MIN_OPS = 4096;   // batches with more edge updates than this pack 16 updates into a workgroup

__device__ inline int32_t new_cap_for(int32_t need) { return need + need / 2 + 4; }
__device__ inline int32_t initial_cap_for(int32_t deg) { return deg + deg / 8 + 2; }

// ------------------------------------------------------------------ build
__global__ void deg_from_indptr_kernel(const int64_t* indptr, int64_t n, int32_t* deg) {
    int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (v < n) deg[v] = (int32_t)(indptr[v + 1] - indptr[v]);
}
__global__ void count_other_kernel(const int32_t* indices, int64_t e, int64_t n, int32_t* deg, int32_t* err) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < e; i += stride) {
        int32_t v = indices[i];
        if (v < 0 || v >= n) { err[0] = 1; continue; }
        atomicAdd(&deg[v], 1);
    }
}
__global__ void caps_kernel(const int32_t* deg, int64_t n, int32_t* cap, uint64_t* off_as_counts) {
    int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (v < n) {
        int32_t c = initial_cap_for(deg[v]);
        cap[v] = c;
        off_as_counts[v] = (uint64_t)c;
    }
}
// one wave per vertex: copy its list from the caller's compressed form into its segment
__global__ void copy_lists_kernel(const int64_t* indptr, const int32_t* indices, const float* w, int64_t n,
                                  Adj a, int32_t* err) {
    const int64_t v = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int lane = threadIdx.x & 63;
    if (v >= n) return;
    const int64_t b = indptr[v], e = indptr[v + 1], o = a.off[v];
    for (int64_t j = b + lane; j < e; j += 64) {
        int32_t u = indices[j];
        if (u < 0 || u >= n) err[0] = 1;
        if (u == v) err[1] = 1;
        a.idx[o + (j - b)] = u;
        if (a.wts) a.wts[o + (j - b)] = w[j];
    }
}
// one wave per key vertex of the given direction: scatter into the other direction with cursors (sort_lists_kernel
// then fixes the order inside each list)
__global__ void transpose_fill_kernel(const int64_t* indptr, const int32_t* indices, const float* w, int64_t n,
                                      Adj other, int32_t* cursor) {
    const int64_t k = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int lane = threadIdx.x & 63;
    if (k >= n) return;
    const int64_t b = indptr[k], e = indptr[k + 1];
    for (int64_t j = b + lane; j < e; j += 64) {
        int32_t t = indices[j];
        if (t < 0 || t >= n) continue;
        int32_t p = atomicAdd(&cursor[t], 1);
        other.idx[other.off[t] + p] = (int32_t)k;
        if (other.wts) other.wts[other.off[t] + p] = w[j];
    }
}

// The cursors above hand out positions in whatever order the waves arrive.  The gathers sum a destination's messages
// in the order of its in-list, so a derived direction is brought into a fixed order afterwards: every list sorted by
// neighbour id (ids are distinct inside a list), weights moved along.  A wave sorts a list of up to 64 entries in
// its registers (rank by counting); longer lists are left to the whole workgroup, which sorts them with a bitonic
// network (ascending compare-exchanges only, so positions past the end act as +infinity and any length works), in
// LDS up to SORT_LDS entries and in place in global memory beyond.
constexpr int SORT_THREADS = 1024;
constexpr int SORT_LDS = 4096;

__device__ inline void sort_cex(int32_t* ki, float* kw, int lo, int hi) {
    const int32_t x = ki[lo], y = ki[hi];
    if (x > y) {
        ki[lo] = y; ki[hi] = x;
        if (kw) { const float t = kw[lo]; kw[lo] = kw[hi]; kw[hi] = t; }
    }
}
// all threads of the workgroup; ki/kw point to LDS or global memory holding len entries
__device__ inline void sort_network(int32_t* ki, float* kw, int len) {
    int P = 2;
    while (P < len) P <<= 1;
    for (int k = 2; k <= P; k <<= 1) {
        const int half = k >> 1;
        for (int t = threadIdx.x; t < (P >> 1); t += SORT_THREADS) {         // first step of a merge: mirror pairs
            const int blk = t / half, o = t - blk * half;
            const int lo = blk * k + o, hi = blk * k + k - 1 - o;
            if (hi < len) sort_cex(ki, kw, lo, hi);
        }
        __syncthreads();
        for (int j = half >> 1; j > 0; j >>= 1) {
            for (int t = threadIdx.x; t < (P >> 1); t += SORT_THREADS) {
                const int lo = ((t & ~(j - 1)) << 1) | (t & (j - 1)), hi = lo | j;
                if (hi < len) sort_cex(ki, kw, lo, hi);
            }
            __syncthreads();
        }
    }
}

__global__ void __launch_bounds__(SORT_THREADS) sort_lists_kernel(Adj a, int64_t n) {
    __shared__ int32_t s_idx[SORT_LDS];
    __shared__ float s_wts[SORT_LDS];
    __shared__ int32_t s_long[SORT_THREADS / 64];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int64_t per_round = SORT_THREADS / 64;
    const int64_t rounds = (n + (int64_t)gridDim.x * per_round - 1) / ((int64_t)gridDim.x * per_round);   // uniform trip count
    for (int64_t r = 0; r < rounds; ++r) {
        const int64_t v = (r * gridDim.x + blockIdx.x) * per_round + w;
        int32_t is_long = -1;
        if (v < n) {
            const int32_t d = a.deg[v];
            const int64_t o = a.off[v];
            if (d > 64) {
                is_long = (int32_t)v;
            } else if (d > 1) {
                const int32_t mine = lane < d ? a.idx[o + lane] : 0x7fffffff;
                const float mw = (a.wts && lane < d) ? a.wts[o + lane] : 0.f;
                int rank = 0;
                for (int j = 0; j < d; ++j) rank += __builtin_amdgcn_readlane(mine, j) < mine;   // d is wave-uniform
                if (lane < d) {
                    a.idx[o + rank] = mine;
                    if (a.wts) a.wts[o + rank] = mw;
                }
            }
        }
        if (lane == 0) s_long[w] = is_long;
        __syncthreads();
        for (int t = 0; t < SORT_THREADS / 64; ++t) {
            const int32_t lv = s_long[t];                           // uniform over the workgroup
            if (lv < 0) continue;
            const int32_t d = a.deg[lv];
            const int64_t o = a.off[lv];
            if (d <= SORT_LDS) {
                for (int i = threadIdx.x; i < d; i += SORT_THREADS) {
                    s_idx[i] = a.idx[o + i];
                    if (a.wts) s_wts[i] = a.wts[o + i];
                }
                __syncthreads();
                sort_network(s_idx, a.wts ? s_wts : nullptr, d);
                for (int i = threadIdx.x; i < d; i += SORT_THREADS) {
                    a.idx[o + i] = s_idx[i];
                    if (a.wts) a.wts[o + i] = s_wts[i];
                }
                __syncthreads();
            } else {
                sort_network(a.idx + o, a.wts ? a.wts + o : nullptr, d);
            }
        }
        __syncthreads();
    }
}

// ------------------------------------------------------------------ validation
__device__ inline uint64_t mix64(uint64_t x) {
    x ^= x >> 33; x *= 0xff51afd7ed558ccdULL; x ^= x >> 33; x *= 0xc4ceb9fe1a85ec53ULL; x ^= x >> 33;
    return x;
}

// workgroup-cooperative search of `target` in the live part of vertex k's list; every thread gets the pool
// position or -1.  The whole list is scanned with independent loads (edges are unique, so at most one hit).
__device__ inline int64_t find_in_list(const Adj& a, int32_t k, int32_t target, int64_t* s_pos) {
    const int64_t o = a.off[k];
    const int32_t d = a.deg[k];
    if (threadIdx.x == 0) *s_pos = -1;
    __syncthreads();
    for (int32_t j = threadIdx.x; j < d; j += VAL_UNROLL * VAL_THREADS) {
        int32_t e[VAL_UNROLL];
#pragma unroll
        for (int t = 0; t < VAL_UNROLL; ++t) {
            const int32_t jj = j + t * VAL_THREADS;
            e[t] = jj < d ? a.idx[o + jj] : -2;
        }
#pragma unroll
        for (int t = 0; t < VAL_UNROLL; ++t)
            if (e[t] == target) *s_pos = o + j + t * VAL_THREADS;
    }
    __syncthreads();
    const int64_t r = *s_pos;
    __syncthreads();
    return r;
}

// err: [0] id out of range  [1] self-loop  [2] inserted edge present  [3] deleted edge absent
//      [4] repeated entry   [5] repeated feature id
struct ValArgs {
    Adj out, in;
    int64_t n, n_ins, n_del;
    const int32_t *ins_src, *ins_dst, *del_src, *del_dst;
    uint64_t* hash; int64_t hash_cap;
    int64_t *pos_out, *pos_in;
    float* del_w;
    int32_t* err;
    int32_t *inscnt0, *inscnt1, *delcnt0, *delcnt1;
    uint32_t* bm_dst;          // set of the destinations of the batch's edge updates (cleared by the launch before), or null
};

// records the update in the batch's set of (src, dst) keys; a key met twice is a repeated entry
__device__ inline void note_key(const ValArgs& A, int32_t u, int32_t v) {
    const uint64_t key = (((uint64_t)(uint32_t)u) << 32 | (uint32_t)v) + 1;   // 0 marks an empty cell
    uint64_t h = mix64(key) & (uint64_t)(A.hash_cap - 1);
    for (int64_t probe = 0; probe < A.hash_cap; ++probe) {
        unsigned long long prev = atomicCAS((unsigned long long*)&A.hash[h], 0ULL, (unsigned long long)key);
        if (prev == 0ULL) break;
        if (prev == key) { A.err[4] = 1; break; }
        h = (h + 1) & (uint64_t)(A.hash_cap - 1);
    }
}

// what a validated update leaves behind: positions and weight of a deleted edge, the per-vertex counts
__device__ inline void note_delete(const ValArgs& A, int64_t i, int32_t u, int32_t v, int64_t po, int64_t pi) {
    A.pos_out[i] = po;
    A.pos_in[i] = pi;
    if (A.del_w) A.del_w[i] = A.out.wts ? A.out.wts[po] : 1.0f;
    atomicAdd(&A.delcnt0[u], 1);
    atomicAdd(&A.delcnt1[v], 1);
}
__device__ inline void note_insert(const ValArgs& A, int32_t u, int32_t v) {
    atomicAdd(&A.inscnt0[u], 1);
    atomicAdd(&A.inscnt1[v], 1);
}

// One update checked by the whole workgroup (every condition below is uniform over the workgroup).
__device__ inline void validate_by_workgroup(const ValArgs& A, int64_t op, bool with_key, int64_t* s_pos) {
    const bool lead = threadIdx.x == 0;
    const bool is_del = op >= A.n_ins;
    const int64_t i = is_del ? op - A.n_ins : op;
    const int32_t u = is_del ? A.del_src[i] : A.ins_src[i];
    const int32_t v = is_del ? A.del_dst[i] : A.ins_dst[i];
    if (u < 0 || u >= A.n || v < 0 || v >= A.n) { if (lead) A.err[0] = 1; return; }
    if (u == v) { if (lead) A.err[1] = 1; return; }
    if (lead && with_key) {
        note_key(A, u, v);
        if (A.bm_dst) atomicOr(&A.bm_dst[v >> 5], 1u << (v & 31));
    }
    if (is_del) {
        const int64_t po = find_in_list(A.out, u, v, s_pos);
        const int64_t pi = find_in_list(A.in, v, u, s_pos);
        if (po < 0 || pi < 0) { if (lead) A.err[3] = 1; return; }
        if (lead) note_delete(A, i, u, v, po, pi);
    } else {
        const bool use_out = A.out.deg[u] <= A.in.deg[v];
        const int64_t p = use_out ? find_in_list(A.out, u, v, s_pos) : find_in_list(A.in, v, u, s_pos);
        if (p >= 0) { if (lead) A.err[2] = 1; return; }
        if (lead) note_insert(A, u, v);
    }
}

// One workgroup per updated edge: the latency of a batch of a few thousand updates is that of its longest lists.
__global__ void __launch_bounds__(VAL_THREADS) validate_edges_kernel(ValArgs A) {
    __shared__ int64_t s_pos;
    validate_by_workgroup(A, blockIdx.x, true, &s_pos);
}

// search by one wave; every lane gets the pool position or -1 (edges are unique, so at most one hit)
__device__ inline int64_t wave_find_in_list(const Adj& a, int32_t k, int32_t target, int lane) {
    const int64_t o = a.off[k];
    const int32_t d = a.deg[k];
    int32_t found = -1;
    for (int32_t j0 = 0; j0 < d; j0 += VAL_UNROLL * 64) {
        int32_t e[VAL_UNROLL];
#pragma unroll
        for (int t = 0; t < VAL_UNROLL; ++t) {
            const int32_t jj = j0 + t * 64 + lane;
            e[t] = jj < d ? a.idx[o + jj] : -2;
        }
#pragma unroll
        for (int t = 0; t < VAL_UNROLL; ++t)
            if (e[t] == target) found = j0 + t * 64 + lane;
    }
#pragma unroll
    for (int sft = 1; sft < 64; sft <<= 1) found = max(found, __shfl_xor(found, sft, 64));
    return found < 0 ? -1 : o + found;
}

// Large batches: a workgroup takes 16 updates, one per wave.  Most lists are short and a wave checks its update
// alone; updates that need a list longer than WAVE_LIST_MAX are then checked one after the other by the whole
// workgroup.  No queue and no second launch: the many short updates no longer pay for a workgroup each.
__global__ void __launch_bounds__(VAL_THREADS) validate_edges_packed_kernel(ValArgs A) {
    __shared__ int64_t s_pos;
    __shared__ int32_t s_long[VAL_THREADS / 64];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int64_t nops = A.n_ins + A.n_del;
    const int64_t op0 = (int64_t)blockIdx.x * (VAL_THREADS / 64);
    const int64_t op = op0 + w;
    int32_t is_long = 0;
    if (op < nops) {
        const bool is_del = op >= A.n_ins;
        const int64_t i = is_del ? op - A.n_ins : op;
        const int32_t u = is_del ? A.del_src[i] : A.ins_src[i];
        const int32_t v = is_del ? A.del_dst[i] : A.ins_dst[i];
        if (u < 0 || u >= A.n || v < 0 || v >= A.n) {
            if (lane == 0) A.err[0] = 1;
        } else if (u == v) {
            if (lane == 0) A.err[1] = 1;
        } else {
            if (lane == 0) {
                note_key(A, u, v);
                if (A.bm_dst) atomicOr(&A.bm_dst[v >> 5], 1u << (v & 31));
            }
            const int32_t du = A.out.deg[u], dv = A.in.deg[v];
            if (is_del) {
                if (du > WAVE_LIST_MAX || dv > WAVE_LIST_MAX) {
                    is_long = 1;
                } else {
                    const int64_t po = wave_find_in_list(A.out, u, v, lane);
                    const int64_t pi = wave_find_in_list(A.in, v, u, lane);
                    if (po < 0 || pi < 0) { if (lane == 0) A.err[3] = 1; }
                    else if (lane == 0) note_delete(A, i, u, v, po, pi);
                }
            } else {
                if (min(du, dv) > WAVE_LIST_MAX) {
                    is_long = 1;
                } else {
                    const int64_t p = du <= dv ? wave_find_in_list(A.out, u, v, lane) : wave_find_in_list(A.in, v, u, lane);
                    if (p >= 0) { if (lane == 0) A.err[2] = 1; }
                    else if (lane == 0) note_insert(A, u, v);
                }
            }
        }
    }
    if (lane == 0) s_long[w] = is_long;
    __syncthreads();
    for (int t = 0; t < VAL_THREADS / 64; ++t)
        if (s_long[t]) validate_by_workgroup(A, op0 + t, false, &s_pos);     // uniform over the workgroup
}

__global__ void validate_feats_kernel(int64_t n, int64_t n_feat, const int32_t* ids, int32_t* feat_index,
                                      int32_t* feat_stamp, int32_t epoch, int32_t* err, uint32_t* bm_feat) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_feat) return;
    int32_t v = ids[i];
    if (v < 0 || v >= n) { err[0] = 1; return; }
    if (bm_feat) atomicOr(&bm_feat[v >> 5], 1u << (v & 31));
    int32_t old = atomicMax(&feat_stamp[v], epoch);
    if (old >= epoch) { err[5] = 1; return; }
    feat_index[v] = (int32_t)i;
}

// thread per (op, direction): the first to stamp a key vertex sums what its list would need
__global__ void plan_growth_kernel(Adj out, Adj in, int64_t n, int64_t n_ins, int64_t n_del, const int32_t* ins_src,
                                   const int32_t* ins_dst, const int32_t* del_src, const int32_t* del_dst,
                                   int32_t* stamp0, int32_t* stamp1, int32_t epoch, const int32_t* inscnt0,
                                   const int32_t* inscnt1, const int32_t* delcnt0, const int32_t* delcnt1,
                                   unsigned long long* grow /* [2] */) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t nops = n_ins + n_del;
    if (t >= 2 * nops) return;
    const int dir = t >= nops;
    const int64_t op = dir ? t - nops : t;
    const bool is_del = op >= n_ins;
    const int64_t i = is_del ? op - n_ins : op;
    int32_t k = dir == 0 ? (is_del ? del_src[i] : ins_src[i]) : (is_del ? del_dst[i] : ins_dst[i]);
    if (k < 0 || k >= n) return;
    int32_t* stamp = dir ? stamp1 : stamp0;
    if (atomicMax(&stamp[k], epoch) >= epoch) return;
    const Adj& a = dir ? in : out;
    int32_t need = a.deg[k] - (dir ? delcnt1 : delcnt0)[k] + (dir ? inscnt1 : inscnt0)[k];
    if (need > a.cap[k]) atomicAdd(&grow[dir], (unsigned long long)new_cap_for(need));
}

__global__ void cancel_counts_kernel(int64_t n, int64_t n_ins, int64_t n_del, const int32_t* ins_src,
                                     const int32_t* ins_dst, const int32_t* del_src, const int32_t* del_dst,
                                     int32_t* inscnt0, int32_t* inscnt1, int32_t* delcnt0, int32_t* delcnt1) {
    const int64_t op = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (op >= n_ins + n_del) return;
    const bool is_del = op >= n_ins;
    const int64_t i = is_del ? op - n_ins : op;
    const int32_t u = is_del ? del_src[i] : ins_src[i];
    const int32_t v = is_del ? del_dst[i] : ins_dst[i];
    if (u >= 0 && u < n) { inscnt0[u] = 0; delcnt0[u] = 0; }
    if (v >= 0 && v < n) { inscnt1[v] = 0; delcnt1[v] = 0; }
}

// ------------------------------------------------------------------ mutation
__global__ void tombstone_kernel(Adj out, Adj in, int64_t n_del, const int64_t* pos_out, const int64_t* pos_in) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_del) return;
    out.idx[pos_out[i]] = -1;
    in.idx[pos_in[i]] = -1;
}

__device__ inline uint32_t block_excl_scan_u32(uint32_t v, uint32_t* total, uint32_t* wsum /* [RB_THREADS/64] shared */) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    uint32_t inc = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        uint32_t o = __shfl_up(inc, d, 64);
        if (lane >= d) inc += o;
    }
    if (lane == 63) wsum[w] = inc;
    __syncthreads();
    uint32_t base = 0, tot = 0;
    for (int i = 0; i < RB_THREADS / 64; ++i) {
        uint32_t t = wsum[i];
        if (i < w) base += t;
        tot += t;
    }
    __syncthreads();
    *total = tot;
    return base + inc - v;
}

struct RebuildArgs {
    Adj out, in;
    int64_t n_ins, n_del;
    const int32_t *ins_src, *ins_dst, *del_src, *del_dst;
    int32_t *stamp0, *stamp1;
    int32_t epoch;
    int32_t *inscnt0, *inscnt1, *delcnt0, *delcnt1;
};
struct RebuildShared {
    uint32_t wsum[RB_THREADS / 64];
    int64_t newoff;
    int nh;
    int32_t hole[RB_FEW];
};

__device__ inline int32_t rebuild_key(const RebuildArgs& A, int64_t op, int dir) {
    const bool is_del = op >= A.n_ins;
    const int64_t i = is_del ? op - A.n_ins : op;
    return dir == 0 ? (is_del ? A.del_src[i] : A.ins_src[i]) : (is_del ? A.del_dst[i] : A.ins_dst[i]);
}

// The whole workgroup drops the tombstones of vertex k's list in direction dir and makes room for its inserts.
__device__ inline void rebuild_by_workgroup(const RebuildArgs& A, int32_t k, int dir, RebuildShared& sh) {
    Adj a = dir ? A.in : A.out;
    int32_t* inscnt = dir ? A.inscnt1 : A.inscnt0;
    int32_t* delcnt = dir ? A.delcnt1 : A.delcnt0;
    const int64_t base = a.off[k];
    const int32_t deg0 = a.deg[k];
    const int32_t dc = delcnt[k], ic = inscnt[k];
    int32_t live = deg0;
    if (dc > 0 && dc <= RB_FEW) {
        // A few tombstones in a possibly very long list: find them with a read-only pass, then move the live entries
        // of the last dc positions into the holes in front of them.  Holes and fillers are matched in ascending
        // position order, so the resulting list order does not depend on thread scheduling.
        if (threadIdx.x == 0) sh.nh = 0;
        __syncthreads();
        for (int32_t p0 = threadIdx.x; p0 < deg0; p0 += RB_THREADS * 8) {      // eight independent loads, then the tests
            int32_t e8[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int32_t p = p0 + j * RB_THREADS;
                e8[j] = p < deg0 ? a.idx[base + p] : 0;
            }
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (e8[j] < 0) { const int at = atomicAdd(&sh.nh, 1); if (at < RB_FEW) sh.hole[at] = p0 + j * RB_THREADS; }
        }
        __syncthreads();
        const int nh = min(sh.nh, RB_FEW);            // equals dc for a validated batch
        const int32_t keep = deg0 - nh;
        int32_t my_hole = -1, my_rank = 0;
        if ((int)threadIdx.x < nh) {
            my_hole = sh.hole[threadIdx.x];
            for (int j = 0; j < nh; ++j) my_rank += sh.hole[j] < my_hole;
        }
        __syncthreads();
        if (my_hole >= 0) sh.hole[my_rank] = my_hole;                // ascending
        __syncthreads();
        // thread t looks at tail position keep + t; a live entry there is the r-th filler, r = t - holes before it
        if ((int)threadIdx.x < nh) {
            const int32_t p = keep + (int32_t)threadIdx.x;
            const int32_t e = a.idx[base + p];
            if (e >= 0) {
                int r = threadIdx.x;
                for (int j = 0; j < nh; ++j) r -= (sh.hole[j] >= keep && sh.hole[j] < p);
                const int32_t h = sh.hole[r];                        // r-th hole overall; all of these lie below keep
                a.idx[base + h] = e;
                if (a.wts) a.wts[base + h] = a.wts[base + p];
            }
        }
        live = keep;
    } else if (dc > 0) {
        uint32_t outpos = 0;
        for (int32_t start = 0; start < deg0; start += RB_THREADS * RB_EPT) {
            int32_t e[RB_EPT];
            float w[RB_EPT];
            uint32_t cnt = 0;
#pragma unroll
            for (int j = 0; j < RB_EPT; ++j) {
                int32_t p = start + (int32_t)threadIdx.x * RB_EPT + j;
                e[j] = p < deg0 ? a.idx[base + p] : -1;
                w[j] = (p < deg0 && a.wts) ? a.wts[base + p] : 0.f;
                cnt += e[j] >= 0;
            }
            uint32_t tot;
            uint32_t ex = block_excl_scan_u32(cnt, &tot, sh.wsum);   // barriers inside: all reads precede all writes
            uint32_t q = outpos + ex;
#pragma unroll
            for (int j = 0; j < RB_EPT; ++j) {
                if (e[j] >= 0) {
                    a.idx[base + q] = e[j];
                    if (a.wts) a.wts[base + q] = w[j];
                    ++q;
                }
            }
            outpos += tot;
        }
        live = (int32_t)outpos;
    }
    const int32_t need = live + ic;
    if (need > a.cap[k]) {
        const int32_t nc = new_cap_for(need);
        __syncthreads();
        if (threadIdx.x == 0) sh.newoff = (int64_t)atomicAdd((unsigned long long*)a.head, (unsigned long long)nc);
        __syncthreads();
        const int64_t no = sh.newoff;
        for (int32_t p = threadIdx.x; p < live; p += RB_THREADS) {
            a.idx[no + p] = a.idx[base + p];
            if (a.wts) a.wts[no + p] = a.wts[base + p];
        }
        if (threadIdx.x == 0) { a.off[k] = no; a.cap[k] = nc; }
    }
    // an in-list already counts its pending inserts: each is then written at its planned position behind the live
    // entries (append_kernel), so the order of an in-list does not depend on thread scheduling
    if (threadIdx.x == 0) { a.deg[k] = live + (dir ? ic : 0); inscnt[k] = 0; delcnt[k] = 0; }
    __syncthreads();                                   // the shared scratch may be reused for the next list
}

// One workgroup per (op, direction); only the first to stamp the key vertex works on its list.
__global__ void __launch_bounds__(RB_THREADS) rebuild_lists_kernel(RebuildArgs A) {
    __shared__ RebuildShared sh;
    __shared__ int32_t s_owner;
    const int dir = blockIdx.y;
    const int32_t k = rebuild_key(A, blockIdx.x, dir);
    int32_t* stamp = dir ? A.stamp1 : A.stamp0;
    if (threadIdx.x == 0) s_owner = atomicMax(&stamp[k], A.epoch) < A.epoch;
    __syncthreads();
    if (!s_owner) return;
    rebuild_by_workgroup(A, k, dir, sh);
}

// Large batches: a workgroup takes 16 (op, direction) items, one per wave.  The wave that stamps a key vertex first
// owns its list; a list of up to WAVE_LIST_MAX entries is squeezed (in list order) and, if needed, moved by that wave
// alone, the longer ones are then rebuilt one after the other by the whole workgroup.
__global__ void __launch_bounds__(RB_THREADS) rebuild_lists_packed_kernel(RebuildArgs A) {
    __shared__ RebuildShared sh;
    __shared__ int32_t s_long[RB_THREADS / 64];       // key vertex + 1, negative for the in-direction; 0: nothing left
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int64_t nops = A.n_ins + A.n_del;
    const int64_t item = (int64_t)blockIdx.x * (RB_THREADS / 64) + w;
    int32_t left = 0;
    if (item < 2 * nops) {
        const int dir = item >= nops;
        const int32_t k = rebuild_key(A, dir ? item - nops : item, dir);
        int32_t* stamp = dir ? A.stamp1 : A.stamp0;
        int32_t owner = 0;
        if (lane == 0) owner = atomicMax(&stamp[k], A.epoch) < A.epoch;
        owner = __shfl(owner, 0, 64);
        if (owner) {
            Adj a = dir ? A.in : A.out;
            const int32_t deg0 = a.deg[k];
            if (deg0 > WAVE_LIST_MAX) {
                left = dir ? -(k + 1) : k + 1;
            } else {
                int32_t* inscnt = dir ? A.inscnt1 : A.inscnt0;
                int32_t* delcnt = dir ? A.delcnt1 : A.delcnt0;
                const int64_t base = a.off[k];
                const int32_t dc = delcnt[k], ic = inscnt[k];
                int32_t live = deg0;
                if (dc > 0) {
                    // in-place squeeze: the entries of a trip are all read before any of them is written, and they
                    // are written at or below the positions just read
                    const unsigned long long below = (1ULL << lane) - 1ULL;
                    int32_t outpos = 0;
                    for (int32_t start = 0; start < deg0; start += 64) {
                        const int32_t p = start + lane;
                        const int32_t e = p < deg0 ? a.idx[base + p] : -1;
                        const float wt = (p < deg0 && a.wts) ? a.wts[base + p] : 0.f;
                        const unsigned long long m = __ballot(e >= 0);
                        if (e >= 0) {
                            const int32_t q = outpos + __popcll(m & below);
                            a.idx[base + q] = e;
                            if (a.wts) a.wts[base + q] = wt;
                        }
                        outpos += __popcll(m);
                    }
                    live = outpos;
                }
                const int32_t need = live + ic;
                if (need > a.cap[k]) {
                    const int32_t nc = new_cap_for(need);
                    long long no = 0;
                    if (lane == 0) no = (long long)atomicAdd((unsigned long long*)a.head, (unsigned long long)nc);
                    no = __shfl(no, 0, 64);
                    for (int32_t p = lane; p < live; p += 64) {
                        a.idx[no + p] = a.idx[base + p];
                        if (a.wts) a.wts[no + p] = a.wts[base + p];
                    }
                    if (lane == 0) { a.off[k] = no; a.cap[k] = nc; }
                }
                if (lane == 0) { a.deg[k] = live + (dir ? ic : 0); inscnt[k] = 0; delcnt[k] = 0; }
            }
        }
    }
    if (lane == 0) s_long[w] = left;
    __syncthreads();
    for (int t = 0; t < RB_THREADS / 64; ++t) {
        const int32_t code = s_long[t];                               // uniform over the workgroup
        if (code > 0) rebuild_by_workgroup(A, code - 1, 0, sh);
        else if (code < 0) rebuild_by_workgroup(A, -code - 1, 1, sh);
    }
}

// Out-lists take their inserts through a cursor (their order matters to no result: they only serve set expansion and
// lookups).  In-lists fix the order in which the gathers sum, so an inserted in-edge goes to the position the batch
// plan gave it: behind the live entries of its destination (whose degree already counts the inserts), by rank.
__global__ void append_kernel(Adj out, Adj in, int64_t n_ins, const int32_t* ins_src, const int32_t* ins_dst,
                              const float* ins_w, const int32_t* slot_of, const int32_t* ins_cnt, const int32_t* ins_rank) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_ins) return;
    const int32_t u = ins_src[i], v = ins_dst[i];
    const float w = ins_w ? ins_w[i] : 1.0f;
    int32_t p = atomicAdd(&out.deg[u], 1);
    out.idx[out.off[u] + p] = v;
    if (out.wts) out.wts[out.off[u] + p] = w;
    const int32_t q = in.deg[v] - ins_cnt[slot_of[v]] + ins_rank[i];
    in.idx[in.off[v] + q] = u;
    if (in.wts) in.wts[in.off[v] + q] = w;
}

void layout_adj(Bump& b, Adj& a, int64_t n, int64_t pool_cap, int weighted) {
    a.off = b.take<int64_t>(n);
    a.deg = b.take<int32_t>(n);
    a.cap = b.take<int32_t>(n);
    a.idx = b.take<int32_t>(pool_cap);
    a.wts = weighted ? b.take<float>(pool_cap) : nullptr;
    a.head = nullptr;   // set by graph_layout: the pool heads live in the shared counter block
    a.pool_cap = pool_cap;
}

}  // namespace

nrt_status graph_layout(Bump& b, nrt_graph* g) {
    const int64_t n = g->n;
    const int64_t pool_cap = g->e_capacity + g->e_capacity / 2 + 8 * n + 1024;
    layout_adj(b, g->out, n, pool_cap, g->weighted);
    layout_adj(b, g->in, n, pool_cap, g->weighted);
    g->scan_tmp_len = cdiv(n > g->e_capacity / NRT_CHUNK ? n : g->e_capacity / NRT_CHUNK, 1024) + 64;
    g->scan_tmp = b.take<uint64_t>(g->scan_tmp_len);
    for (int d = 0; d < 2; ++d) {
        g->stamp[d] = b.take<int32_t>(n);
        g->inscnt[d] = b.take<int32_t>(n);
        g->delcnt[d] = b.take<int32_t>(n);
    }
    g->dev_ctrs = b.take<int64_t>(NRT_NCTRS);
    g->out.head = g->dev_ctrs ? g->dev_ctrs + CTR_HEAD_OUT : nullptr;
    g->in.head = g->dev_ctrs ? g->dev_ctrs + CTR_HEAD_IN : nullptr;
    return NRT_OK;
}

static nrt_status build_direction(nrt_graph* g, Adj& a, const int64_t* indptr, const int32_t* indices, const float* w,
                                  int32_t* err, hipStream_t s) {
    const int64_t n = g->n;
    const int nb = (int)cdiv(n, 256);
    deg_from_indptr_kernel<<<nb, 256, 0, s>>>(indptr, n, a.deg);
    LAUNCH_CHECK();
    caps_kernel<<<nb, 256, 0, s>>>(a.deg, n, a.cap, (uint64_t*)a.off);
    LAUNCH_CHECK();
    NRT_TRY(k_exclusive_scan_u64((uint64_t*)a.off, n, g->scan_tmp, g->scan_tmp_len, (uint64_t*)a.head, s));
    copy_lists_kernel<<<(int)cdiv(n * 64, 256), 256, 0, s>>>(indptr, indices, w, n, a, err);
    LAUNCH_CHECK();
    return NRT_OK;
}

static nrt_status derive_direction(nrt_graph* g, Adj& other, const int64_t* indptr, const int32_t* indices,
                                   const float* w, int32_t* err, hipStream_t s) {
    const int64_t n = g->n;
    const int nb = (int)cdiv(n, 256);
    NRT_TRY(k_fill_u32((uint32_t*)other.deg, n, 0, s));
    if (g->e > 0) {
        int64_t grid = cdiv(g->e, 256);
        if (grid > 65536) grid = 65536;
        count_other_kernel<<<(int)grid, 256, 0, s>>>(indices, g->e, n, other.deg, err);
        LAUNCH_CHECK();
    }
    caps_kernel<<<nb, 256, 0, s>>>(other.deg, n, other.cap, (uint64_t*)other.off);
    LAUNCH_CHECK();
    NRT_TRY(k_exclusive_scan_u64((uint64_t*)other.off, n, g->scan_tmp, g->scan_tmp_len, (uint64_t*)other.head, s));
    int32_t* cursor = g->inscnt[0];   // zero between batches; restored to zero below
    transpose_fill_kernel<<<(int)cdiv(n * 64, 256), 256, 0, s>>>(indptr, indices, w, n, other, cursor);
    LAUNCH_CHECK();
    NRT_TRY(k_fill_u32((uint32_t*)cursor, n, 0, s));
    int64_t grid = cdiv(n, SORT_THREADS / 64);
    if (grid > 4096) grid = 4096;
    sort_lists_kernel<<<(int)grid, SORT_THREADS, 0, s>>>(other, n);
    LAUNCH_CHECK();
    return NRT_OK;
}

nrt_status graph_build(nrt_graph* g, const int64_t* csr_indptr, const int32_t* csr_indices, const float* csr_w,
                       const int64_t* csc_indptr, const int32_t* csc_indices, const float* csc_w, hipStream_t s) {
    const int64_t n = g->n;
    for (int d = 0; d < 2; ++d) {
        NRT_TRY(k_fill_u32((uint32_t*)g->stamp[d], n, 0, s));
        NRT_TRY(k_fill_u32((uint32_t*)g->inscnt[d], n, 0, s));
        NRT_TRY(k_fill_u32((uint32_t*)g->delcnt[d], n, 0, s));
    }
    NRT_TRY(k_fill_u64((uint64_t*)g->dev_ctrs, NRT_NCTRS, 0, s));
    int32_t* err = (int32_t*)(g->dev_ctrs + CTR_ERR);
    if (csr_indptr) NRT_TRY(build_direction(g, g->out, csr_indptr, csr_indices, csr_w, err, s));
    if (csc_indptr) NRT_TRY(build_direction(g, g->in, csc_indptr, csc_indices, csc_w, err, s));
    if (!csc_indptr) NRT_TRY(derive_direction(g, g->in, csr_indptr, csr_indices, csr_w, err, s));
    if (!csr_indptr) NRT_TRY(derive_direction(g, g->out, csc_indptr, csc_indices, csc_w, err, s));
    HIP_TRY(hipMemcpyAsync(g->host_pinned, g->dev_ctrs, NRT_NCTRS * sizeof(int64_t), hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    const int32_t* herr = (const int32_t*)(g->host_pinned + CTR_ERR);
    if (herr[0]) { nrt_set_error("graph has a vertex id outside [0, n)"); return NRT_ERR_INVALID_ARG; }
    if (herr[1]) { nrt_set_error("graph has an explicit self-loop"); return NRT_ERR_INVALID_ARG; }
    g->epoch = 2;
    return NRT_OK;
}

nrt_status graph_validate_batch(nrt_graph* g, const nrt_batch* b, BatchScratch& sc, const FillJobs* clears, hipStream_t s) {
    const int64_t nops = b->n_ins + b->n_del;
    FillJobs f;
    memset(&f, 0, sizeof(f));
    if (clears) f = *clears;
    f.add(g->dev_ctrs + CTR_ERR, 8);        // 8 int32 flags
    f.add(g->dev_ctrs + CTR_GROW, 4);
    if (nops > 0) f.add(sc.hash_keys, 2 * sc.hash_cap);
    NRT_TRY(k_multi_fill(f, s));
    if (b->n_feat > 0) {
        validate_feats_kernel<<<(int)cdiv(b->n_feat, 256), 256, 0, s>>>(g->n, b->n_feat, b->feat_ids, sc.feat_index,
                                                                       sc.feat_stamp, g->epoch, sc.err, sc.bm_feat);
        LAUNCH_CHECK();
    }
    if (nops == 0) return NRT_OK;
    ValArgs va;
    va.out = g->out; va.in = g->in;
    va.n = g->n; va.n_ins = b->n_ins; va.n_del = b->n_del;
    va.ins_src = b->ins_src; va.ins_dst = b->ins_dst; va.del_src = b->del_src; va.del_dst = b->del_dst;
    va.hash = sc.hash_keys; va.hash_cap = sc.hash_cap;
    va.pos_out = sc.pos_out; va.pos_in = sc.pos_in; va.del_w = sc.del_w; va.err = sc.err;
    va.inscnt0 = g->inscnt[0]; va.inscnt1 = g->inscnt[1]; va.delcnt0 = g->delcnt[0]; va.delcnt1 = g->delcnt[1];
    va.bm_dst = sc.bm_dst;
    if (nops > PACKED_MIN_OPS) validate_edges_packed_kernel<<<(unsigned)cdiv(nops, VAL_THREADS / 64), VAL_THREADS, 0, s>>>(va);
    else validate_edges_kernel<<<(unsigned)nops, VAL_THREADS, 0, s>>>(va);
    LAUNCH_CHECK();
    plan_growth_kernel<<<(int)cdiv(2 * nops, 256), 256, 0, s>>>(
        g->out, g->in, g->n, b->n_ins, b->n_del, b->ins_src, b->ins_dst, b->del_src, b->del_dst, g->stamp[0],
        g->stamp[1], g->epoch, g->inscnt[0], g->inscnt[1], g->delcnt[0], g->delcnt[1],
        (unsigned long long*)(g->dev_ctrs + CTR_GROW));
    LAUNCH_CHECK();
    return NRT_OK;
}

nrt_status graph_cancel_batch(nrt_graph* g, const nrt_batch* b, hipStream_t s) {
    const int64_t nops = b->n_ins + b->n_del;
    g->epoch += 2;   // stamps of the failed attempt must not look current to the next batch
    if (nops == 0) return NRT_OK;
    cancel_counts_kernel<<<(int)cdiv(nops, 256), 256, 0, s>>>(g->n, b->n_ins, b->n_del, b->ins_src, b->ins_dst,
                                                             b->del_src, b->del_dst, g->inscnt[0], g->inscnt[1],
                                                             g->delcnt[0], g->delcnt[1]);
    LAUNCH_CHECK();
    return NRT_OK;
}

nrt_status graph_mutate(nrt_graph* g, const nrt_batch* b, BatchScratch& sc, hipStream_t s) {
    const int64_t nops = b->n_ins + b->n_del;
    if (nops == 0) { g->epoch += 2; return NRT_OK; }
    if (b->n_ins > 0 && (!sc.plan_slot_of || !sc.plan_ins_cnt || !sc.plan_ins_rank)) {      // before anything changes
        nrt_set_error("internal: batch plan missing");
        return NRT_ERR_STATE;
    }
    if (b->n_del > 0) {
        tombstone_kernel<<<(int)cdiv(b->n_del, 256), 256, 0, s>>>(g->out, g->in, b->n_del, sc.pos_out, sc.pos_in);
        LAUNCH_CHECK();
    }
    RebuildArgs ra;
    ra.out = g->out; ra.in = g->in;
    ra.n_ins = b->n_ins; ra.n_del = b->n_del;
    ra.ins_src = b->ins_src; ra.ins_dst = b->ins_dst; ra.del_src = b->del_src; ra.del_dst = b->del_dst;
    ra.stamp0 = g->stamp[0]; ra.stamp1 = g->stamp[1]; ra.epoch = g->epoch + 1;
    ra.inscnt0 = g->inscnt[0]; ra.inscnt1 = g->inscnt[1]; ra.delcnt0 = g->delcnt[0]; ra.delcnt1 = g->delcnt[1];
    if (nops > PACKED_MIN_OPS) {
        rebuild_lists_packed_kernel<<<(unsigned)cdiv(2 * nops, RB_THREADS / 64), RB_THREADS, 0, s>>>(ra);
    } else {
        dim3 grid((unsigned)nops, 2, 1);
        rebuild_lists_kernel<<<grid, RB_THREADS, 0, s>>>(ra);
    }
    LAUNCH_CHECK();
    if (b->n_ins > 0) {
        append_kernel<<<(int)cdiv(b->n_ins, 256), 256, 0, s>>>(g->out, g->in, b->n_ins, b->ins_src, b->ins_dst, b->ins_w,
                                                               sc.plan_slot_of, sc.plan_ins_cnt, sc.plan_ins_rank);
        LAUNCH_CHECK();
    }
    g->epoch += 2;
    g->e += b->n_ins - b->n_del;
    return NRT_OK;
}
