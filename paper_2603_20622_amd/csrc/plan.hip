// Batch plan: the edge updates of a batch grouped by destination, in a fixed order.
//
// Section IV-B turns an inserted edge into a positive message and a deleted edge into a negative one for its
// destination.  Several updates of one batch may hit the same destination; so that their terms are summed in an order
// that does not depend on how the GPU schedules threads (and without floating-point atomics), the updates are sorted
// by (destination, position in the batch): destination slots in ascending vertex order, inside a slot inserts before
// deletes, each in the order the caller listed them.  One owner wave per destination then folds its terms
// (structural_fold_kernel and its GAT / A-GNN forms), and an inserted in-edge is appended at the position given by
// its rank, so the in-lists, whose order the gathers' sums follow, are reproducible too.
//
// Outputs: list[slot] = destination vertex (ascending), slot_of[v] = slot, off[slot] .. off[slot + 1] = its run in
// ord[] (update numbers: inserts 0 .. n_ins-1, deletes n_ins ..), ins_cnt[slot] = inserts in the run,
// ins_rank[i] = rank of insert i among the inserts of its destination, *count = number of slots.
// Updates with an id outside [0, n) are left out (the batch is about to be rejected).
#include "common.h"

namespace {

constexpr int PS_THREADS = 1024;
constexpr int PS_MAX = 2048;            // updates the single-workgroup form sorts in LDS

__device__ inline int32_t plan_dst(const PlanArgs& a, int64_t op) {
    return op < a.n_ins ? a.ins_dst[op] : a.del_dst[op - a.n_ins];
}
__device__ inline int32_t plan_src(const PlanArgs& a, int64_t op) {
    return op < a.n_ins ? a.ins_src[op] : a.del_src[op - a.n_ins];
}
__device__ inline bool plan_valid(const PlanArgs& a, int64_t op) {
    const int32_t u = plan_src(a, op), v = plan_dst(a, op);
    return u >= 0 && u < a.n && v >= 0 && v < a.n;
}

// ------------------------------------------------------------------ up to PS_MAX updates: one workgroup, one launch
// bitonic sort of the keys (destination << 32 | update number) in LDS, then runs of equal destinations are the slots
__global__ void __launch_bounds__(PS_THREADS) batch_plan_small_kernel(PlanArgs a) {
    __shared__ uint64_t key[PS_MAX];
    __shared__ int32_t s_off[PS_MAX + 1];
    __shared__ uint32_t wsum[PS_THREADS / 64];
    const int tid = threadIdx.x;
    const int nops = (int)(a.n_ins + a.n_del);
    int P = 64;
    while (P < nops) P <<= 1;                                   // sort size: power of two, at most PS_MAX
    for (int i = tid; i < P; i += PS_THREADS) {
        uint64_t k = ~0ULL;                                     // padding and rejected updates sort to the end
        if (i < nops && plan_valid(a, i)) k = ((uint64_t)(uint32_t)plan_dst(a, i) << 32) | (uint32_t)i;
        key[i] = k;
    }
    __syncthreads();
    for (int k = 2; k <= P; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int t = tid; t < (P >> 1); t += PS_THREADS) {
                const int lo = ((t & ~(j - 1)) << 1) | (t & (j - 1));
                const int hi = lo | j;
                const bool asc = (lo & k) == 0;
                const uint64_t x = key[lo], y = key[hi];
                if ((x > y) == asc) { key[lo] = y; key[hi] = x; }
            }
            __syncthreads();
        }
    }
    // two consecutive positions per thread; a position starts a slot when its destination differs from the one before
    const int p0 = 2 * tid;
    uint32_t lead[2];
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const int p = p0 + e;
        lead[e] = 0;
        if (p < P && key[p] != ~0ULL) lead[e] = (p == 0 || (key[p - 1] >> 32) != (key[p] >> 32)) ? 1u : 0u;
    }
    // inclusive scan of the slot starts over the workgroup
    const int lane = tid & 63, w = tid >> 6;
    uint32_t inc = lead[0] + lead[1];
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t o = __shfl_up(inc, d, 64);
        if (lane >= d) inc += o;
    }
    if (lane == 63) wsum[w] = inc;
    __syncthreads();
    uint32_t base = 0, nd = 0;
    for (int i = 0; i < PS_THREADS / 64; ++i) {
        const uint32_t t = wsum[i];
        if (i < w) base += t;
        nd += t;
    }
    uint32_t before = base + inc - (lead[0] + lead[1]);         // slots started before position p0
    int32_t slot[2];
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const int p = p0 + e;
        before += lead[e];
        slot[e] = (int32_t)before - 1;
        if (lead[e]) s_off[slot[e]] = p;
    }
    int n_valid = 0;                                            // valid keys are a prefix of the sorted array
    {
        int lo = 0, hi = P;                                     // first position holding padding
        while (lo < hi) { const int mid = (lo + hi) >> 1; if (key[mid] != ~0ULL) lo = mid + 1; else hi = mid; }
        n_valid = lo;
    }
    if (tid == 0) { s_off[nd] = n_valid; *a.count = (uint64_t)nd; }
    __syncthreads();
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const int p = p0 + e;
        if (p >= n_valid) continue;
        const uint64_t k = key[p];
        const int32_t v = (int32_t)(k >> 32), op = (int32_t)(k & 0xffffffffu);
        const int32_t s = slot[e], b = s_off[s], en = s_off[s + 1];
        a.ord[p] = op;
        if (lead[e]) {
            a.list[s] = v;
            a.slot_of[v] = s;
            a.off[s] = b;
            if (op >= a.n_ins) a.ins_cnt[s] = 0;                // the run starts with a delete: it holds no insert
        }
        if (p == n_valid - 1) a.off[nd] = n_valid;
        if (op < a.n_ins) {
            a.ins_rank[op] = p - b;
            const bool last_insert = p + 1 == en || (int64_t)(key[p + 1] & 0xffffffffu) >= a.n_ins;
            if (last_insert) a.ins_cnt[s] = p - b + 1;
        }
    }
    if (tid == 0 && n_valid == 0) a.off[0] = 0;
}

// ------------------------------------------------------------------ any number of updates
// runs sized by counting, filled through cursors (any order), then every update finds its rank inside its run
__global__ void plan_count_kernel(PlanArgs a) {
    const int64_t op = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (op >= a.n_ins + a.n_del || !plan_valid(a, op)) return;
    atomicAdd((unsigned long long*)&a.off64[a.slot_of[plan_dst(a, op)]], 1ULL);
}
__global__ void plan_fill_kernel(PlanArgs a) {
    const int64_t op = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (op >= a.n_ins + a.n_del || !plan_valid(a, op)) return;
    const int32_t s = a.slot_of[plan_dst(a, op)];
    const int32_t at = atomicAdd(&a.cursor[s], 1);
    a.tmp[(int64_t)a.off64[s] + at] = (int32_t)op;
}
__global__ void plan_rank_kernel(PlanArgs a) {
    const int64_t op = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (op >= a.n_ins + a.n_del || !plan_valid(a, op)) return;
    const int64_t nd = (int64_t)*a.count;
    const int32_t s = a.slot_of[plan_dst(a, op)];
    const int64_t b = (int64_t)a.off64[s];
    const int64_t e = s + 1 < nd ? (int64_t)a.off64[s + 1] : (int64_t)*a.total;
    int32_t rank = 0, n_ins_here = 0;
    int32_t first = 0x7fffffff;
    for (int64_t j = b; j < e; ++j) {
        const int32_t o = a.tmp[j];
        rank += o < (int32_t)op;
        n_ins_here += o < a.n_ins;
        first = min(first, o);
    }
    a.ord[b + rank] = (int32_t)op;
    if (op < a.n_ins) a.ins_rank[op] = rank;
    if (first == (int32_t)op) {                                  // the first update of the run writes what describes the run
        a.off[s] = (int32_t)b;
        a.ins_cnt[s] = n_ins_here;
        if (s + 1 == nd) a.off[nd] = (int32_t)e;
    }
}

// ------------------------------------------------------------------ structural terms, one owner per destination
// one wave per (destination slot, layer): SD^l[slot] = sum over the slot's updates, in plan order, of
// sign * c * p^{l-1}_src(old); the gather wave that owns the destination adds the row to the cached aggregate
__global__ void structural_fold_kernel(FoldArgs a) {
    const int lane = threadIdx.x & 63;
    const int l = blockIdx.y;
    const int64_t nd = (int64_t)*a.n_slots;
    const int64_t waves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    const int D = a.D[l];
    for (int64_t s = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6; s < nd; s += waves) {
        const int32_t b = a.off[s], e = a.off[s + 1];
        float* dst = a.SD[l] + s * D;
        for (int col = lane * 4; col < D; col += 256) {
            // a destination can collect hundreds of terms of one batch and they are added one after the other, so the sum
            // is compensated (Kahan): its error stays that of a single rounding instead of growing with the run's length
            float4 acc = make_float4(0.f, 0.f, 0.f, 0.f), comp = acc;
            for (int32_t j = b; j < e; ++j) {
                const int32_t op = a.ord[j];
                const bool is_del = op >= a.n_ins;
                const int64_t i = is_del ? op - a.n_ins : op;
                const int32_t u = is_del ? a.del_src[i] : a.ins_src[i];
                float c = is_del ? -1.0f : 1.0f;
                if (is_del && a.del_w) c *= a.del_w[i];
                if (!is_del && a.ins_w) c *= a.ins_w[i];
                if (a.indeg_old) c *= 1.0f / sqrtf((float)(a.indeg_old[u] + 1));
                int64_t row = a.compact_src[l] ? (int64_t)op : (int64_t)u;
                if (a.rel_R) {                                   // typed edge: the relation's message row of the source
                    row = (int64_t)u * a.rel_R + nrt_rel_of(is_del ? a.del_w[i] : a.ins_w[i], a.rel_R);
                    c = is_del ? -1.0f : 1.0f;
                }
                const float4 x = *reinterpret_cast<const float4*>(a.Hprev[l] + row * D + col);
                const float4 y = make_float4(fmaf(c, x.x, -comp.x), fmaf(c, x.y, -comp.y), fmaf(c, x.z, -comp.z), fmaf(c, x.w, -comp.w));
                const float4 t = make_float4(acc.x + y.x, acc.y + y.y, acc.z + y.z, acc.w + y.w);
                comp = make_float4((t.x - acc.x) - y.x, (t.y - acc.y) - y.y, (t.z - acc.z) - y.z, (t.w - acc.w) - y.w);
                acc = t;
            }
            *reinterpret_cast<float4*>(dst + col) = acc;
        }
    }
}

}  // namespace

nrt_status k_batch_plan(const PlanArgs& a, uint64_t* scan_tmp, int64_t scan_tmp_len, hipStream_t s) {
    const int64_t nops = a.n_ins + a.n_del;
    if (nops <= 0) return NRT_OK;
    if (nops <= PS_MAX) {
        batch_plan_small_kernel<<<1, PS_THREADS, 0, s>>>(a);
        LAUNCH_CHECK();
        return NRT_OK;
    }
    // slots from the bitmap of destinations (sorted list, vertex -> slot), then count / scan / fill / rank
    NRT_TRY(k_compact(nullptr, a.dst_bitmap, nullptr, a.scratch_bm, a.n, a.list, a.slot_of, a.cmp_state, a.cmp_state_len, a.count, s));
    const int grid = (int)cdiv(nops, 256);
    plan_count_kernel<<<grid, 256, 0, s>>>(a);
    LAUNCH_CHECK();
    NRT_TRY(k_exclusive_scan_u64(a.off64, nops, scan_tmp, scan_tmp_len, a.total, s));
    plan_fill_kernel<<<grid, 256, 0, s>>>(a);
    LAUNCH_CHECK();
    plan_rank_kernel<<<grid, 256, 0, s>>>(a);
    LAUNCH_CHECK();
    return NRT_OK;
}

nrt_status k_structural_fold(const FoldArgs& a, hipStream_t s) {
    const int64_t nops = a.n_ins + a.n_del;
    if (nops <= 0 || a.n_layers <= 0) return NRT_OK;
    int64_t g = cdiv(nops, 4);                                   // at most one slot per update; four waves per workgroup
    if (g > 2048) g = 2048;
    structural_fold_kernel<<<dim3((unsigned)g, (unsigned)a.n_layers, 1), 256, 0, s>>>(a);
    LAUNCH_CHECK();
    return NRT_OK;
}
