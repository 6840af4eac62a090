// Delta-message gather and fold (the message and aggregation steps of Algorithm 1, with the aggregate cached in context-free form).
//
// For every affected destination v the cached sum S[v] = sum_u c_uv p_u receives the changes of its
// affected in-neighbours: S[v] += sum_{u in N_new(v), u changed} c_uv * dp_u, where dp_u is the change of
// the source payload (already formed by the previous layer's write-back).  The terms of inserted and
// deleted edges are folded beforehand on the old caches (k_structural_fold, plan.hip): +c p_u(old) for an inserted
// edge, -c p_u(old) for a deleted one, so that an inserted edge whose source also changed sums to
// c p_u(new) (Section IV-B: insert = positive message, delete = negative, update = both).
//
// The same kernel, with no source filter and rows read straight from h^{l-1}, is the full-neighbour
// aggregation of Eq. 1 used by nrt_cache_init.
//
// Mapping to the machine: destinations are walked through their in-lists (no atomics, no sort: each
// destination row is owned by one wave).  An in-list of more than NRT_CHUNK entries is cut into items of
// NRT_CHUNK entries that write partial rows; a second small kernel sums them in item order, which keeps a
// 100k-degree hub from serialising on one wave and keeps the result order-deterministic.  Two kernels serve the
// layers: gather_kernel (software pipeline over 64-entry steps, built for layers where most in-list entries
// contribute and the row traffic dominates) and gather_sparse_kernel (short per-entry path with an LDS filter,
// for layers where few sources changed); the device counters decide which of the two runs.
#include "common.h"

namespace {

constexpr int WAVES_PER_BLOCK = 4;

__device__ inline float4 f4_fma(float c, float4 x, float4 a) {
    a.x = fmaf(c, x.x, a.x); a.y = fmaf(c, x.y, a.y); a.z = fmaf(c, x.z, a.z); a.w = fmaf(c, x.w, a.w);
    return a;
}
// Element offset of a row: row ids are non-negative, so the product is one unsigned 32x32->64 multiply.
__device__ inline int64_t row_off(int32_t row, int D) { return (int64_t)((uint64_t)(uint32_t)row * (uint32_t)D); }
__device__ inline float4 f4_add(float4 a, float4 b) { return make_float4(a.x + b.x, a.y + b.y, a.z + b.z, a.w + b.w); }
__device__ inline float4 f4_shfl_xor(float4 a, int m) {
    return make_float4(__shfl_xor(a.x, m, 64), __shfl_xor(a.y, m, 64), __shfl_xor(a.z, m, 64), __shfl_xor(a.w, m, 64));
}
__device__ inline float gcn_scale(int32_t indeg) { return 1.0f / sqrtf((float)(indeg + 1)); }

// ------------------------------------------------------------------ records and hub items
// One thread per destination slot (strided over a fixed grid; the count lives on the device): its record,
// and for a hub its entry in the hub list and its run of items.  Hub and item numbers are handed out with one
// atomic per workgroup (a block-wide prefix sum inside), not one per hub.
constexpr int REC_THREADS = 1024;
constexpr int REC_EPT = 4;          // slots per thread per round: few, large workgroups keep the shared atomics rare

__device__ inline uint64_t rec_block_scan(uint64_t v, uint64_t* total, uint64_t* wsum) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    uint64_t inc = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        uint64_t o = __shfl_up((unsigned long long)inc, d, 64);
        if (lane >= d) inc += o;
    }
    if (lane == 63) wsum[w] = inc;
    __syncthreads();
    uint64_t base = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < REC_THREADS / 64; ++i) {
        const uint64_t t = wsum[i];
        if (i < w) base += t;
        tot += t;
    }
    __syncthreads();
    *total = tot;
    return base + inc - v;
}

__global__ void __launch_bounds__(REC_THREADS)
dst_records_kernel(const int32_t* list, int64_t n_all, Adj in, DstRec* recs, HubWork hubs, LayerCtrs* lc,
                   const uint64_t* plain_if_zero) {
    __shared__ uint64_t wsum[REC_THREADS / 64];
    __shared__ unsigned long long s_hbase, s_ibase;
    const int64_t count = list ? (int64_t)lc->count : n_all;
    const bool no_items = plain_if_zero && *plain_if_zero == 0;
    const int64_t per_round = (int64_t)REC_THREADS * REC_EPT;
    const int64_t stride = (int64_t)gridDim.x * per_round;
    uint64_t degsum = 0;
    for (int64_t i0 = (int64_t)blockIdx.x * per_round; i0 < count; i0 += stride) {   // workgroup-uniform trip count
        DstRec r[REC_EPT];
        uint64_t nch[REC_EPT];
        uint64_t mine = 0;
#pragma unroll
        for (int e = 0; e < REC_EPT; ++e) {
            const int64_t i = i0 + (int64_t)e * REC_THREADS + threadIdx.x;
            nch[e] = 0;
            r[e].off = 0; r[e].deg = 0; r[e].v = 0;
            if (i < count) {
                const int32_t v = list ? list[i] : (int32_t)i;
                r[e].off = in.off[v];
                r[e].deg = in.deg[v];
                r[e].v = v;
            }
        }
#pragma unroll
        for (int e = 0; e < REC_EPT; ++e) {
            const int64_t i = i0 + (int64_t)e * REC_THREADS + threadIdx.x;
            if (i < count) {
                recs[i] = r[e];
                degsum += (uint64_t)r[e].deg;
                if (r[e].deg > NRT_CHUNK && !no_items) nch[e] = (uint64_t)((r[e].deg + NRT_CHUNK - 1) / NRT_CHUNK);
                mine += nch[e] ? ((1ULL << 32) | nch[e]) : 0ULL;     // high 32 bits: hubs, low 32 bits: items
            }
        }
        uint64_t tot;
        uint64_t ex = rec_block_scan(mine, &tot, wsum);
        if (threadIdx.x == 0 && tot) {
            s_hbase = atomicAdd((unsigned long long*)&lc->n_hubs, (unsigned long long)(tot >> 32));
            s_ibase = atomicAdd((unsigned long long*)&lc->n_items, (unsigned long long)(tot & 0xffffffffu));
        }
        __syncthreads();
        // items of a hub: a hub of a hundred thousand in-edges has hundreds of them, and one thread writing them
        // alone would set the kernel's time, so the wave writes those together
        const int lane = threadIdx.x & 63;
#pragma unroll
        for (int e = 0; e < REC_EPT; ++e) {
            const int64_t i = i0 + (int64_t)e * REC_THREADS + threadIdx.x;
            const int64_t h = (int64_t)(s_hbase + (ex >> 32));
            const int64_t first = (int64_t)(s_ibase + (ex & 0xffffffffu));
            const bool is_hub = nch[e] != 0 && h < hubs.hub_cap;
            if (nch[e]) ex += (1ULL << 32) | nch[e];
            if (is_hub) {
                hubs.hub_slot[h] = (int32_t)i;
                hubs.hub_first[h] = (uint64_t)first;
            }
            if (is_hub && nch[e] <= 8) {                          // the many small hubs: their own lane writes the few items
                for (int32_t c = 0; c < (int32_t)nch[e]; ++c) {
                    if (first + c < hubs.item_cap) {
                        hubs.item_hub[first + c] = (int32_t)h;
                        hubs.item_chunk[first + c] = c;
                    }
                }
            }
            unsigned long long m = __ballot(is_hub && nch[e] > 8);  // the few long ones: the whole wave writes
            while (m) {
                const int from = __ffsll((long long)m) - 1;
                m &= m - 1;
                const int32_t hh = (int32_t)__shfl((long long)h, from, 64);
                const int64_t ff = (int64_t)__shfl((long long)first, from, 64);
                const int32_t nn = (int32_t)__shfl((long long)nch[e], from, 64);
                for (int32_t c = lane; c < nn; c += 64) {
                    if (ff + c < hubs.item_cap) {
                        hubs.item_hub[ff + c] = hh;
                        hubs.item_chunk[ff + c] = c;
                    }
                }
            }
        }
        __syncthreads();
    }
    uint64_t bt;
    rec_block_scan(degsum, &bt, wsum);
    if (threadIdx.x == 0 && bt) atomicAdd((unsigned long long*)&lc->in_edges[blockIdx.x & 15], (unsigned long long)bt);
}

// ------------------------------------------------------------------ gather
// Work units: [0, n_items) are the hub items, NRT_CHUNK in-list entries each, whose partial row goes to
// partial[item] (heavy units first, so they start early); [n_items, n_items + n_dst) are the destinations
// themselves (those with at most NRT_CHUNK in-edges are served here, hubs are skipped).  All sizes are read on
// the device; a fixed grid strides over chunks of `upw` consecutive units.  A wave owns one chunk at a time and walks them as a sequence of
// steps of 64 in-list entries (one per lane) through a four-stage software pipeline, so that the four
// dependent memory accesses of a step (in-list entry -> bitmap word of changed sources -> slot of the
// source's delta row -> the row itself) overlap with the accesses of the neighbouring steps instead of
// being paid one after the other for every destination:
//   A  load the in-list entries of step t+3
//   B  load the bitmap words for step t+2
//   C  test the bits, load the slots of the survivors of step t+1 (and the old aggregate row if the step
//      closes its destination)
//   D  walk the ballot of survivors of step t with scalar bit operations: each survivor's slot is broadcast
//      with a lane read, so the row address is wave-uniform and the row load is one coalesced instruction
//      (rows narrower than 256 floats put RPI = 2 or 4 survivors into one load, one per LPR-lane sub-group);
//      on the last step of a unit reduce the sub-groups and write the row.
// Rebuild the aggregate row of v from its whole in-neighbourhood with current values (the full-neighbour
// definition, Eq. 1): the fallback when an incremental fold has cancelled the leading digits of a row.  (Only the
// un-normalised models carry that guard; typed edges never reach this function, k_gather refuses the combination.)
template <int LPR, int NV>
__device__ inline void full_row(const GatherArgs& a, int32_t v, int64_t off, int32_t deg, int lane, float4 (&acc)[NV]) {
    constexpr int RPI = 64 / LPR;
    const int sub = lane / LPR, gl = lane % LPR, D = a.D;
    const float* Pl = a.Pfull + gl * 4;
#pragma unroll
    for (int q = 0; q < NV; ++q) acc[q] = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int32_t j0 = 0; j0 < deg; j0 += 64) {
        const int32_t jj = j0 + lane;
        const int32_t u = jj < deg ? a.in.idx[off + jj] : -1;
        float c = 1.0f;
        if (u >= 0 && a.use_weights) c = a.in.wts[off + jj];
        if (u >= 0 && a.full_scale_gcn) c *= gcn_scale(a.in.deg[u]);
        unsigned long long m = __ballot(u >= 0);
        while (m) {
            int32_t rr = -1;
            float cc = 0.f;
#pragma unroll
            for (int t = 0; t < RPI; ++t) {
                if (m) {
                    const int bit = __ffsll((long long)m) - 1;
                    m &= m - 1;
                    const int32_t rs = __builtin_amdgcn_readlane(u, bit);
                    const float cs = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, c), bit));
                    if (sub == t) { rr = rs; cc = cs; }
                }
            }
#pragma unroll
            for (int q = 0; q < NV; ++q)
                if (rr >= 0 && gl * 4 + q * LPR * 4 < D)
                    acc[q] = f4_fma(cc, *reinterpret_cast<const float4*>(Pl + row_off(rr, D) + q * LPR * 4), acc[q]);
        }
    }
    if (a.self_pair && sub == 0) {
        const float cs = a.full_scale_gcn ? gcn_scale(deg) : 1.0f;
#pragma unroll
        for (int q = 0; q < NV; ++q)
            if (gl * 4 + q * LPR * 4 < D)
                acc[q] = f4_fma(cs, *reinterpret_cast<const float4*>(Pl + (int64_t)v * D + q * LPR * 4), acc[q]);
    }
#pragma unroll
    for (int q = 0; q < NV; ++q)
#pragma unroll
        for (int mm = LPR; mm < 64; mm <<= 1) acc[q] = f4_add(acc[q], f4_shfl_xor(acc[q], mm));
}

// largest |component| over the lanes of a wave (lanes outside `use` contribute 0)
template <int NV>
__device__ inline float wave_absmax(const float4 (&x)[NV], bool use) {
    float m = 0.f;
    if (use) {
#pragma unroll
        for (int q = 0; q < NV; ++q) m = fmaxf(m, fmaxf(fmaxf(fabsf(x[q].x), fabsf(x[q].y)), fmaxf(fabsf(x[q].z), fabsf(x[q].w))));
    }
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) m = fmaxf(m, __shfl_xor(m, s, 64));
    return m;
}
constexpr float GUARD_RATIO = 16.0f;     // rebuild a row when the fold is 16x larger than what it leaves behind

// The host cannot know how many sources changed without a synchronisation, so both gather kernels are launched
// and each asks the device counters whether the layer is its to serve.
__device__ inline bool layer_is_sparse(const GatherArgs& a) {
    if (a.sparse_ok == 2) return true;          // the host launched only the sparse kernel (it is correct at any density)
    return a.sparse_ok && a.n_src_dev && (int64_t)(*a.n_src_dev) * 16 <= a.n_vertices;
}

// true when this launch is not the one that serves the layer (see GatherArgs::auto_role)
__device__ inline bool layer_goes_to_other_role(const GatherArgs& a) {
    if (!a.auto_role) return false;
    const bool recompute = 4 * (int64_t)(*a.auto_src_dev) > a.n_vertices;
    return a.auto_role == 1 ? recompute : !recompute;
}

// Step flags kept in the per-wave step table.
enum { SF_FIRST = 1, SF_LAST = 2, SF_PART = 4, SF_SELF = 8, SF_DD = 16 };

// COEF: 0 every term has coefficient 1; 1 edge weights and / or the GCN source scale; 2 typed edges: the weight is a
// relation id that picks one of the source's rel_R rows (coefficient 1)
template <int LPR, int NV, bool FILTER, int COEF>
__global__ void __launch_bounds__(WAVES_PER_BLOCK * 64) gather_kernel(GatherArgs a) {
    constexpr int RPI = 64 / LPR;
    constexpr int MAX_UPW = 8;                       // units per wave; 8 units * 4 steps fit the 64-lane step table
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int sub = lane / LPR, gl = lane % LPR;
    const int D = a.D;
    if (layer_goes_to_other_role(a)) return;
    if (a.n_src_dev && *a.n_src_dev == 0 && !a.sd) return;   // nothing changed upstream of this layer
    if (FILTER && NV == 1 && layer_is_sparse(a)) return;     // served by gather_sparse_kernel
    const int64_t n_dst = (int64_t)a.lc->count;
    int64_t n_items = (int64_t)a.lc->n_items;
    if (n_items > a.hubs.item_cap) n_items = a.hubs.item_cap;
    const int64_t total = n_dst + n_items;
    int upw = (int)(total / 16384);                        // units per wave: keep ~16k waves when there is enough work
                                                           // (more units per wave = fewer pipeline fill/drain bubbles)
    upw = upw < 1 ? 1 : (upw > MAX_UPW ? MAX_UPW : upw);
    const int64_t n_chunks = (total + upw - 1) / upw;
    const int64_t n_waves = (int64_t)gridDim.x * WAVES_PER_BLOCK;
    const float* Pl = a.P + gl * 4;
    long long pairs = 0;

    auto take = [&](unsigned long long& m, int32_t rv, float cv) {
        int32_t rr = -1;
        float cc = 1.0f;
#pragma unroll
        for (int t = 0; t < RPI; ++t) {
            if (m) {
                const int bit = __ffsll((long long)m) - 1;
                m &= m - 1;
                const int32_t rs = __builtin_amdgcn_readlane(rv, bit);
                if (sub == t) rr = rs;
                if (COEF) {
                    const float cs = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, cv), bit));
                    if (sub == t) cc = cs;
                }
            }
        }
        return make_int2(rr, __builtin_bit_cast(int, cc));
    };

    for (int64_t chunk_id = (int64_t)blockIdx.x * WAVES_PER_BLOCK + w; chunk_id < n_chunks; chunk_id += n_waves) {
        const int64_t unit0 = chunk_id * upw;
        const int nu = (int)min((int64_t)upw, total - unit0);

        // ---- lane i < nu describes unit i of this chunk
        int64_t u_base = 0, u_out = 0;
        int32_t u_cnt = -1, u_v = 0, u_deg = 0, u_flags = 0;
        if (lane < nu) {
            const int64_t unit = unit0 + lane;
            DstRec rec;
            int32_t chunk = 0;
            if (unit >= n_items) {                     // hub items come first: the heavy units start early
                rec = a.recs[unit - n_items];
                u_cnt = rec.deg > NRT_CHUNK ? -1 : rec.deg;
                u_out = (int64_t)rec.v * D;
                u_flags = SF_SELF;
            } else {
                chunk = a.hubs.item_chunk[unit];
                rec = a.recs[a.hubs.hub_slot[a.hubs.item_hub[unit]]];
                u_cnt = min(NRT_CHUNK, rec.deg - chunk * NRT_CHUNK);
                u_out = unit * D;
                u_flags = SF_PART | (chunk == 0 ? SF_SELF : 0);
            }
            u_base = rec.off + (int64_t)chunk * NRT_CHUNK;
            u_v = rec.v;
            u_deg = rec.deg;
        }
        // ---- step table: lane t describes step t (64 in-list entries) of the chunk
        const int u_steps = u_cnt < 0 ? 0 : (u_cnt + 63 > 63 ? (u_cnt + 63) >> 6 : 1);     // at least one step per served unit
        int my_unit = 0, my_first = 0, n_steps = 0;
#pragma unroll
        for (int i = 0; i < MAX_UPW; ++i) {
            const int sc = __builtin_amdgcn_readlane(u_steps, i);      // 0 for lanes past nu (u_cnt = -1)
            if (lane >= n_steps) { my_unit = i; my_first = n_steps; }
            n_steps += sc;
        }
        const int addr = my_unit << 2;
        const int32_t t_cnt = __builtin_amdgcn_ds_bpermute(addr, u_cnt);
        const int32_t t_j = (lane - my_first) << 6;
        const int32_t t_n = min(64, t_cnt - t_j);
        const int64_t t_base = ((int64_t)(((uint64_t)(uint32_t)__builtin_amdgcn_ds_bpermute(addr, (int32_t)(u_base >> 32)) << 32) |
                                          (uint32_t)__builtin_amdgcn_ds_bpermute(addr, (int32_t)(u_base & 0xffffffff)))) + t_j;
        const int32_t t_out_lo = __builtin_amdgcn_ds_bpermute(addr, (int32_t)(u_out & 0xffffffff));
        const int32_t t_out_hi = __builtin_amdgcn_ds_bpermute(addr, (int32_t)(u_out >> 32));
        const int32_t t_v = __builtin_amdgcn_ds_bpermute(addr, u_v);
        const int32_t t_deg = __builtin_amdgcn_ds_bpermute(addr, u_deg);
        int32_t t_flags = __builtin_amdgcn_ds_bpermute(addr, u_flags);
        t_flags = (t_flags & SF_PART) | (t_j == 0 ? SF_FIRST | (t_flags & SF_SELF) : 0) | (t_j + 64 >= t_cnt ? SF_LAST : 0);
        const int32_t t_base_lo = (int32_t)(t_base & 0xffffffff), t_base_hi = (int32_t)(t_base >> 32);

        // ---- four-stage pipeline over the steps
        int32_t uB = -1, uC = -1, slD = -1;
        float wB = 1.f, wC = 1.f, cD = 1.f;
        uint32_t xC = 0;                 // bitmap word (FILTER) or in-degree of the source (GCN scale)
        float4 acc[NV], oldD[NV];
#pragma unroll
        for (int q = 0; q < NV; ++q) { acc[q] = make_float4(0.f, 0.f, 0.f, 0.f); oldD[q] = acc[q]; }

        auto fetch_add = [&](int2 p0, int2 p1, int2 p2, int2 p3) {
            const float c0 = __builtin_bit_cast(float, p0.y), c1 = __builtin_bit_cast(float, p1.y);
            const float c2 = __builtin_bit_cast(float, p2.y), c3 = __builtin_bit_cast(float, p3.y);
#pragma unroll
            for (int q = 0; q < NV; ++q) {
                const bool live = gl * 4 + q * LPR * 4 < D;
                float4 x0 = make_float4(0.f, 0.f, 0.f, 0.f), x1 = x0, x2 = x0, x3 = x0;
                if (p0.x >= 0 && live) x0 = *reinterpret_cast<const float4*>(Pl + row_off(p0.x, D) + q * LPR * 4);
                if (p1.x >= 0 && live) x1 = *reinterpret_cast<const float4*>(Pl + row_off(p1.x, D) + q * LPR * 4);
                if (p2.x >= 0 && live) x2 = *reinterpret_cast<const float4*>(Pl + row_off(p2.x, D) + q * LPR * 4);
                if (p3.x >= 0 && live) x3 = *reinterpret_cast<const float4*>(Pl + row_off(p3.x, D) + q * LPR * 4);
                acc[q] = COEF ? f4_fma(c0, x0, acc[q]) : f4_add(acc[q], x0);
                acc[q] = COEF ? f4_fma(c1, x1, acc[q]) : f4_add(acc[q], x1);
                acc[q] = COEF ? f4_fma(c2, x2, acc[q]) : f4_add(acc[q], x2);
                acc[q] = COEF ? f4_fma(c3, x3, acc[q]) : f4_add(acc[q], x3);
            }
        };

        auto fetch_add2 = [&](int2 p0, int2 p1) {
            const float c0 = __builtin_bit_cast(float, p0.y), c1 = __builtin_bit_cast(float, p1.y);
#pragma unroll
            for (int q = 0; q < NV; ++q) {
                const bool live = gl * 4 + q * LPR * 4 < D;
                float4 x0 = make_float4(0.f, 0.f, 0.f, 0.f), x1 = x0;
                if (p0.x >= 0 && live) x0 = *reinterpret_cast<const float4*>(Pl + row_off(p0.x, D) + q * LPR * 4);
                if (p1.x >= 0 && live) x1 = *reinterpret_cast<const float4*>(Pl + row_off(p1.x, D) + q * LPR * 4);
                acc[q] = COEF ? f4_fma(c0, x0, acc[q]) : f4_add(acc[q], x0);
                acc[q] = COEF ? f4_fma(c1, x1, acc[q]) : f4_add(acc[q], x1);
            }
        };

        for (int i = 0; i < n_steps + 3; ++i) {
            // ---- stage A: in-list entries of step i
            int32_t uA = -1;
            float wA = 1.f;
            if (i < n_steps) {
                const int n = __builtin_amdgcn_readlane(t_n, i);
                const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane(t_base_lo, i);
                const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane(t_base_hi, i);
                const int64_t base = (int64_t)(((uint64_t)hi << 32) | lo);
                if (lane < n) {
                    uA = a.in.idx[base + lane];
                    if (COEF && a.use_weights) wA = a.in.wts[base + lane];
                }
            }
            // ---- stage B (step i-1): bitmap word, or source degree for the GCN scale
            uint32_t xB = 0;
            if (FILTER) { if (uB >= 0) xB = a.src_bitmap[(uint32_t)uB >> 5]; }
            else if (COEF && a.src_scale_gcn) { if (uB >= 0) xB = (uint32_t)a.in.deg[(uint32_t)uB]; }
            // ---- stage C (step i-2): survivors and their slots; old aggregate row if the step closes its unit
            int32_t slC = -1;
            float cC = wC;
            float4 oldC[NV];
#pragma unroll
            for (int q = 0; q < NV; ++q) oldC[q] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (FILTER) {
                if (uC >= 0 && ((xC >> (uC & 31)) & 1u)) slC = a.src_slot[(uint32_t)uC];
            } else {
                slC = uC;
                if (COEF && a.src_scale_gcn && uC >= 0) cC *= gcn_scale((int32_t)xC);
            }
            if (COEF == 2) {                                     // typed edge: the relation's row of the source, coefficient 1
                if (slC >= 0) slC = slC * a.rel_R + nrt_rel_of(cC, a.rel_R);
                cC = 1.0f;
            }
            if (i >= 2 && i - 2 < n_steps && a.accumulate) {
                const int f = __builtin_amdgcn_readlane(t_flags, i - 2);
                if ((f & (SF_LAST | SF_PART)) == SF_LAST) {
                    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane(t_out_lo, i - 2);
                    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane(t_out_hi, i - 2);
                    const float* op = a.S + (int64_t)(((uint64_t)hi << 32) | lo) + gl * 4;
#pragma unroll
                    for (int q = 0; q < NV; ++q)
                        if (sub == 0 && gl * 4 + q * LPR * 4 < D) oldC[q] = *reinterpret_cast<const float4*>(op + q * LPR * 4);
                }
            }
            // ---- stage D (step i-3): stream the rows of the survivors
            if (i >= 3) {
                const int f = __builtin_amdgcn_readlane(t_flags, i - 3);
                unsigned long long m = __ballot(slD >= 0);
                pairs += __popcll(m);
                while (m) {
                    if (__popcll(m) <= 2 * RPI) {            // the common case on sparse layers: one short round
                        const int2 p0 = take(m, slD, cD);
                        const int2 p1 = take(m, slD, cD);
                        fetch_add2(p0, p1);
                    } else {
                        const int2 p0 = take(m, slD, cD);
                        const int2 p1 = take(m, slD, cD);
                        const int2 p2 = take(m, slD, cD);
                        const int2 p3 = take(m, slD, cD);
                        fetch_add(p0, p1, p2, p3);
                    }
                }
                if ((f & SF_SELF) && a.self_pair) {
                    const int32_t v = __builtin_amdgcn_readlane(t_v, i - 3);
                    bool sok = true;
                    if (FILTER) sok = (a.src_bitmap[v >> 5] >> (v & 31)) & 1u;
                    if (sok) {
                        const int32_t rs = FILTER ? a.src_slot[v] : v;
                        const float cs = (COEF && a.src_scale_gcn) ? gcn_scale(__builtin_amdgcn_readlane(t_deg, i - 3)) : 1.0f;
                        fetch_add(make_int2(sub == 0 ? rs : -1, __builtin_bit_cast(int, cs)), make_int2(-1, 0),
                                  make_int2(-1, 0), make_int2(-1, 0));
                        pairs += 1;
                    }
                }
                if ((f & SF_SELF) && a.sd) {                 // structural terms of the batch for this destination
                    const int32_t v = __builtin_amdgcn_readlane(t_v, i - 3);
                    if ((a.dd_bitmap[v >> 5] >> (v & 31)) & 1u) {
                        const float* sp = a.sd + (int64_t)a.dd_slot[v] * D + gl * 4;
#pragma unroll
                        for (int q = 0; q < NV; ++q)
                            if (sub == 0 && gl * 4 + q * LPR * 4 < D)
                                acc[q] = f4_add(acc[q], *reinterpret_cast<const float4*>(sp + q * LPR * 4));
                    }
                }
                if (f & SF_LAST) {
                    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane(t_out_lo, i - 3);
                    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane(t_out_hi, i - 3);
                    float* op = ((f & SF_PART) ? a.hubs.partial : a.S) + (int64_t)(((uint64_t)hi << 32) | lo) + gl * 4;
                    const bool fold = !(f & SF_PART) && a.accumulate;
#pragma unroll
                    for (int q = 0; q < NV; ++q)
#pragma unroll
                        for (int mm = LPR; mm < 64; mm <<= 1) acc[q] = f4_add(acc[q], f4_shfl_xor(acc[q], mm));
                    float4 y[NV];
#pragma unroll
                    for (int q = 0; q < NV; ++q) y[q] = fold ? f4_add(acc[q], oldD[q]) : acc[q];
                    if (fold && a.guard) {
                        const float big = wave_absmax<NV>(acc, sub == 0), left = wave_absmax<NV>(y, sub == 0);
                        if (big > GUARD_RATIO * left) {          // the fold cancelled the row: rebuild it in full
                            const int32_t v = __builtin_amdgcn_readlane(t_v, i - 3);
                            const int32_t dg = __builtin_amdgcn_readlane(t_deg, i - 3);
                            const uint32_t blo = (uint32_t)__builtin_amdgcn_readlane(t_base_lo, i - 3);
                            const uint32_t bhi = (uint32_t)__builtin_amdgcn_readlane(t_base_hi, i - 3);
                            const int64_t off = (int64_t)(((uint64_t)bhi << 32) | blo) - __builtin_amdgcn_readlane(t_j, i - 3);
                            full_row<LPR, NV>(a, v, off, dg, lane, y);
                        }
                    }
#pragma unroll
                    for (int q = 0; q < NV; ++q) {
                        if (sub == 0 && gl * 4 + q * LPR * 4 < D) *reinterpret_cast<float4*>(op + q * LPR * 4) = y[q];
                        acc[q] = make_float4(0.f, 0.f, 0.f, 0.f);
                    }
                }
            }
            // ---- rotate
            slD = slC; cD = cC;
#pragma unroll
            for (int q = 0; q < NV; ++q) oldD[q] = oldC[q];
            uC = uB; wC = wB; xC = xB;
            uB = uA; wB = wA;
        }
    }
    if (a.pair_ctr && lane == 0 && pairs) atomicAdd(&a.pair_ctr[blockIdx.x & 1023], (unsigned long long)pairs);
}

// ------------------------------------------------------------------ gather over sparsely changed sources
// When only a small part of the vertices changed, most in-list entries fail the bitmap test and the cost of a
// destination is the instructions spent per scanned entry, not the bytes of the few delta rows.  This variant
// keeps the per-entry work short: a wave takes four consecutive units at a time, one per 16-lane group, and
//   scan   every lane reads four in-list entries of its group's unit (64 entries per unit and trip), then the
//          bitmap words, then the slots of the survivors: three batches of independent loads;
//   pack   the survivors of each group are written, in in-list order, to the group's queue in LDS;
//   rows   the queues are drained four slots per LDS read; each LPR-lane sub-group streams the rows of one
//          unit (RPI = 64 / LPR units at a time), so row addresses come from LDS, not from lane reads;
//   fold   the old aggregate rows (requested before the scan when they fit the registers) are added and stored.
// The order of additions is fixed by the in-lists, so the result does not depend on the schedule.
constexpr int SQ_CAP = 72;      // queue entries per group: 64 scanned entries + the self term, padded to 16 bytes
constexpr int SP_WAVES = 8;     // waves per workgroup: they share one copy of the coarse filter in LDS
constexpr int SP_BLOCKS = 768;  // persistent grid: three workgroups per compute unit

// A random probe of the changed-source bitmap from HBM/L2 pulls a whole cache line per in-list entry; with a
// bitmap far larger than the vector L1 that line traffic, not arithmetic, bounds the scan.  Each workgroup
// therefore keeps a coarse copy in LDS (one bit per 2^shift vertices, at most COARSE_WORDS words) and only the
// entries that pass it go on to the exact bitmap.  coarse_bitmap_kernel builds the copy once per layer.
__global__ void coarse_bitmap_kernel(const uint32_t* fine, int64_t n, int shift, uint32_t* coarse, int64_t n_words) {
    const int64_t cw = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (cw >= n_words) return;
    const int64_t fine_words = (n + 31) >> 5;
    uint32_t out = 0;
    for (int i = 0; i < 32; ++i) {
        const int64_t v0 = (cw * 32 + i) << shift;            // first vertex of the bit's group
        if (v0 >= n) break;
        uint32_t any = 0;
        if (shift <= 5) {
            const uint32_t word = fine[v0 >> 5];
            const uint32_t mask = shift == 5 ? 0xffffffffu : (((1u << (1 << shift)) - 1u) << (v0 & 31));
            any = word & mask;
        } else {
            const int64_t w0 = v0 >> 5, nw = (int64_t)1 << (shift - 5);
            for (int64_t k = 0; k < nw && w0 + k < fine_words; ++k) any |= fine[w0 + k];
        }
        if (any) out |= 1u << i;
    }
    coarse[cw] = out;
}

template <int LPR, int COEF>
__global__ void __launch_bounds__(SP_WAVES * 64) gather_sparse_kernel(GatherArgs a) {
    constexpr int RPI = 64 / LPR;          // units served by one row load
    constexpr int NPASS = 4 / RPI;         // row passes over the four units of a round
    constexpr bool PREFETCH = NPASS <= 2;  // old aggregate rows requested before the scan
    __shared__ __attribute__((aligned(16))) int32_t s_slot[SP_WAVES][4][SQ_CAP];
    __shared__ __attribute__((aligned(16))) float s_coef[SP_WAVES][4][COEF ? SQ_CAP : 4];
    __shared__ uint32_t s_coarse[NRT_COARSE_WORDS];
    if (layer_goes_to_other_role(a) || !layer_is_sparse(a)) return;
    if (*a.n_src_dev == 0 && !a.sd) return;
    for (int i = threadIdx.x; i < a.coarse_words; i += SP_WAVES * 64) s_coarse[i] = a.coarse[i];
    __syncthreads();
    const int csh = a.coarse_shift;
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int g = lane >> 4, l16 = lane & 15;          // scan role
    const int sub = lane / LPR, gl = lane % LPR;       // row role
    const int D = a.D;
    const bool live = gl * 4 < D;
    const int64_t n_dst = (int64_t)a.lc->count;
    int64_t n_items = (int64_t)a.lc->n_items;
    if (n_items > a.hubs.item_cap) n_items = a.hubs.item_cap;
    const int64_t total = n_dst + n_items;
    const int64_t n_rounds = (total + 3) >> 2;
    const int64_t n_waves = (int64_t)gridDim.x * SP_WAVES;
    const float* Pl = a.P + gl * 4;
    int32_t* q_mine = &s_slot[w][g][0];
    float* c_mine = &s_coef[w][g][0];
    const uint32_t below = (1u << l16) - 1u;
    long long pairs = 0;

    for (int64_t r = (int64_t)blockIdx.x * SP_WAVES + w; r < n_rounds; r += n_waves) {
        // ---- scan role: the unit of this lane's group
        const int64_t unit = r * 4 + g;
        int64_t u_base = 0, u_out = 0;
        int32_t u_cnt = 0, u_v = 0, u_deg = 0, u_flags = 0;     // flags == 0: nothing to serve, nothing to write
        if (unit < total) {
            DstRec rec;
            int32_t chunk = 0;
            if (unit >= n_items) {
                rec = a.recs[unit - n_items];
                if (rec.deg <= NRT_CHUNK) { u_cnt = rec.deg; u_flags = SF_SELF | SF_LAST; }   // hubs are served through their items
                u_out = (int64_t)rec.v * D;
            } else {
                chunk = a.hubs.item_chunk[unit];
                rec = a.recs[a.hubs.hub_slot[a.hubs.item_hub[unit]]];
                u_cnt = min(NRT_CHUNK, rec.deg - chunk * NRT_CHUNK);
                u_out = unit * D;
                u_flags = SF_PART | SF_LAST | (chunk == 0 ? SF_SELF : 0);
            }
            u_base = rec.off + (int64_t)chunk * NRT_CHUNK;
            u_v = rec.v;
            u_deg = rec.deg;
            // destination of an updated edge: its structural terms join the fold (tested here, with the record, so
            // that the fold itself waits for no load in the common case)
            if (a.sd && (u_flags & SF_SELF) && ((a.dd_bitmap[rec.v >> 5] >> (rec.v & 31)) & 1u)) u_flags |= SF_DD;
        }
        // ---- row role: accumulators, and the old rows while the scan runs
        float4 acc[NPASS], old[NPASS];
#pragma unroll
        for (int ps = 0; ps < NPASS; ++ps) {
            acc[ps] = make_float4(0.f, 0.f, 0.f, 0.f);
            old[ps] = acc[ps];
            if (PREFETCH) {
                const int from = (ps * RPI + sub) << 4;
                const int32_t fl = __shfl(u_flags, from, 64);
                const int32_t vr = __shfl(u_v, from, 64);
                if ((fl & (SF_LAST | SF_PART)) == SF_LAST && live)
                    old[ps] = *reinterpret_cast<const float4*>(a.S + row_off(vr, D) + gl * 4);
            }
        }
        int32_t maxcnt = max(max(__builtin_amdgcn_readlane(u_cnt, 0), __builtin_amdgcn_readlane(u_cnt, 16)),
                             max(__builtin_amdgcn_readlane(u_cnt, 32), __builtin_amdgcn_readlane(u_cnt, 48)));
        int32_t hits = 0;                                        // per group, over the whole unit
        int32_t j = 0;
        do {
            // ---- scan: entries, bitmap words, slots
            int32_t e[5];
            float wv[5];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int32_t jj = j + k * 16 + l16;
                e[k] = -1;
                wv[k] = 1.0f;
                if (jj < u_cnt) {
                    e[k] = a.in.idx[u_base + jj];
                    if (COEF) wv[k] = a.in.wts[u_base + jj];
                }
            }
            e[4] = (j == 0 && l16 == 0 && a.self_pair && (u_flags & SF_SELF)) ? u_v : -1;
            wv[4] = 1.0f;
            uint32_t bw[5];
#pragma unroll
            for (int k = 0; k < 5; ++k) {                       // coarse filter in LDS
                bw[k] = 0u;
                if (e[k] >= 0) {
                    const uint32_t cbit = (uint32_t)e[k] >> csh;
                    bw[k] = (s_coarse[cbit >> 5] >> (cbit & 31)) & 1u;
                }
            }
#pragma unroll
            for (int k = 0; k < 5; ++k) bw[k] = bw[k] ? a.src_bitmap[(uint32_t)e[k] >> 5] : 0u;
            int32_t sl[5];
#pragma unroll
            for (int k = 0; k < 5; ++k) sl[k] = ((bw[k] >> (e[k] & 31)) & 1u) ? a.src_slot[(uint32_t)e[k]] : -1;
            if (COEF == 2) {                                     // typed edge: the relation's row of the source, coefficient 1
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    if (sl[k] >= 0) sl[k] = sl[k] * a.rel_R + nrt_rel_of(wv[k], a.rel_R);
                    wv[k] = 1.0f;
                }
            }
            // ---- pack the survivors of each group, in in-list order
            int32_t nq = 0;
#pragma unroll
            for (int k = 0; k < 5; ++k) {
                const bool hit = sl[k] >= 0;
                const unsigned long long b = __ballot(hit);
                pairs += __popcll(b);
                const uint32_t gb = (uint32_t)(b >> (g << 4)) & 0xffffu;
                if (hit) {
                    const int pos = nq + __popc(gb & below);
                    q_mine[pos] = sl[k];
                    if (COEF) c_mine[pos] = wv[k];
                }
                nq += __popc(gb);
            }
            hits += nq;
            __builtin_amdgcn_wave_barrier();
            // ---- rows: RPI units per pass, four queue entries per trip
#pragma unroll
            for (int ps = 0; ps < NPASS; ++ps) {
                const int uu = ps * RPI + sub;
                const int32_t n_u = __shfl(nq, uu << 4, 64);
                int32_t n_max = 0;
#pragma unroll
                for (int t = 0; t < RPI; ++t) n_max = max(n_max, __builtin_amdgcn_readlane(nq, (ps * RPI + t) << 4));
                const int32_t* qu = &s_slot[w][uu][0];
                const float* cu = &s_coef[w][COEF ? uu : 0][0];
                for (int32_t t = 0; t < n_max; t += 4) {
                    const int4 s4 = *reinterpret_cast<const int4*>(qu + t);
                    float4 c4 = make_float4(1.f, 1.f, 1.f, 1.f);
                    if (COEF) {                                  // entries past the queue's end are stale: keep them finite
                        c4 = *reinterpret_cast<const float4*>(cu + t);
                        if (t + 0 >= n_u) c4.x = 0.f;
                        if (t + 1 >= n_u) c4.y = 0.f;
                        if (t + 2 >= n_u) c4.z = 0.f;
                        if (t + 3 >= n_u) c4.w = 0.f;
                    }
                    float4 x0 = make_float4(0.f, 0.f, 0.f, 0.f), x1 = x0, x2 = x0, x3 = x0;
                    if (t + 0 < n_u && live) x0 = *reinterpret_cast<const float4*>(Pl + row_off(s4.x, D));
                    if (t + 1 < n_u && live) x1 = *reinterpret_cast<const float4*>(Pl + row_off(s4.y, D));
                    if (t + 2 < n_u && live) x2 = *reinterpret_cast<const float4*>(Pl + row_off(s4.z, D));
                    if (t + 3 < n_u && live) x3 = *reinterpret_cast<const float4*>(Pl + row_off(s4.w, D));
                    acc[ps] = COEF ? f4_fma(c4.x, x0, acc[ps]) : f4_add(acc[ps], x0);
                    acc[ps] = COEF ? f4_fma(c4.y, x1, acc[ps]) : f4_add(acc[ps], x1);
                    acc[ps] = COEF ? f4_fma(c4.z, x2, acc[ps]) : f4_add(acc[ps], x2);
                    acc[ps] = COEF ? f4_fma(c4.w, x3, acc[ps]) : f4_add(acc[ps], x3);
                }
            }
            __builtin_amdgcn_wave_barrier();
            j += 64;
        } while (j < maxcnt);

        // ---- fold and store
#pragma unroll
        for (int ps = 0; ps < NPASS; ++ps) {
            const int from = (ps * RPI + sub) << 4;
            const int32_t fl = __shfl(u_flags, from, 64);
            const int32_t vr = __shfl(u_v, from, 64);
            const int32_t nh = __shfl(hits, from, 64);
            const int64_t out = (int64_t)(((uint64_t)(uint32_t)__shfl((int32_t)(u_out >> 32), from, 64) << 32) |
                                          (uint32_t)__shfl((int32_t)(u_out & 0xffffffff), from, 64));
            float4 y = acc[ps];
            bool touched = nh > 0;
            if (fl & SF_DD) {
                touched = true;
                if (live) y = f4_add(y, *reinterpret_cast<const float4*>(a.sd + (int64_t)a.dd_slot[vr] * D + gl * 4));
            }
            const bool part = fl & SF_PART;
            if (part && live) *reinterpret_cast<float4*>(a.hubs.partial + out + gl * 4) = y;
            const bool fold = !part && (fl & SF_LAST) && touched && live;      // no early exit: the votes below need every lane
            if (!PREFETCH && fold) old[ps] = *reinterpret_cast<const float4*>(a.S + out + gl * 4);
            float4 z = f4_add(y, old[ps]);
            if (a.guard) {
                float big = 0.f, left = 0.f;
                if (fold) {
                    big = fmaxf(fmaxf(fabsf(y.x), fabsf(y.y)), fmaxf(fabsf(y.z), fabsf(y.w)));
                    left = fmaxf(fmaxf(fabsf(z.x), fabsf(z.y)), fmaxf(fabsf(z.z), fabsf(z.w)));
                }
#pragma unroll
                for (int sft = 1; sft < LPR; sft <<= 1) {
                    big = fmaxf(big, __shfl_xor(big, sft, 64));
                    left = fmaxf(left, __shfl_xor(left, sft, 64));
                }
                unsigned long long trig = __ballot(gl == 0 && big > GUARD_RATIO * left);
                while (trig) {                                   // rebuild the cancelled rows, one unit at a time
                    const int bit = __ffsll((long long)trig) - 1;
                    trig &= trig - 1;
                    const int src = (ps * RPI + bit / LPR) << 4;
                    const int32_t fv = __builtin_amdgcn_readlane(u_v, src);
                    const int32_t fd = __builtin_amdgcn_readlane(u_deg, src);
                    const uint32_t blo = (uint32_t)__builtin_amdgcn_readlane((int32_t)(u_base & 0xffffffff), src);
                    const uint32_t bhi = (uint32_t)__builtin_amdgcn_readlane((int32_t)(u_base >> 32), src);
                    float4 full[1];
                    full_row<LPR, 1>(a, fv, (int64_t)(((uint64_t)bhi << 32) | blo), fd, lane, full);
                    if (sub == bit / LPR) z = full[0];
                }
            }
            if (fold) *reinterpret_cast<float4*>(a.S + out + gl * 4) = z;
        }
    }
    if (a.pair_ctr && lane == 0 && pairs) atomicAdd(&a.pair_ctr[blockIdx.x & 1023], (unsigned long long)pairs);
}

// one wave per hub (strided): sum its partial rows in item order into the cached aggregate
__global__ void combine_kernel(GatherArgs a) {
    if (a.n_src_dev && *a.n_src_dev == 0 && !a.sd) return;
    if (a.auto_role == 1 && layer_goes_to_other_role(a)) {   // the layer was recomputed: partial rows are whole sums
        a.accumulate = 0;
        a.guard = 0;
    }
    const int lane = threadIdx.x & 63;
    int64_t nh = (int64_t)a.lc->n_hubs;
    if (nh > a.hubs.hub_cap) nh = a.hubs.hub_cap;
    const int64_t waves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    const int D = a.D;
    // rows narrower than 256 floats leave lanes free: LW lanes cover a row, the 64 / LW sub-groups take every
    // (64 / LW)-th partial row, eight loads in flight each, and are reduced with lane exchanges at the end
    const int LW = D <= 64 ? 16 : (D <= 128 ? 32 : 64);
    const int G = 64 / LW, sub = lane / LW, gl = lane % LW;
    for (int64_t h = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6; h < nh; h += waves) {
        const DstRec rec = a.recs[a.hubs.hub_slot[h]];
        const int32_t nch = (rec.deg + NRT_CHUNK - 1) / NRT_CHUNK;
        const int64_t first = (int64_t)a.hubs.hub_first[h];
        float big = 0.f, left = 0.f;
        for (int col = gl * 4; col < D; col += 256) {
            const float* p = a.hubs.partial + first * D + col;
            float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
            for (int32_t c0 = sub; c0 < nch; c0 += 8 * G) {
                float4 x[8];
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const int32_t c = c0 + k * G;
                    x[k] = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (c < nch) x[k] = *reinterpret_cast<const float4*>(p + (int64_t)c * D);
                }
#pragma unroll
                for (int k = 0; k < 8; ++k) acc = f4_add(acc, x[k]);
            }
            for (int mm = LW; mm < 64; mm <<= 1) acc = f4_add(acc, f4_shfl_xor(acc, mm));
            float4* dst = reinterpret_cast<float4*>(a.S + (int64_t)rec.v * D + col);
            float4 y = acc;
            if (sub == 0) {
                if (a.accumulate) y = f4_add(acc, *dst);
                *dst = y;
                if (a.accumulate && a.guard) {
                    big = fmaxf(big, fmaxf(fmaxf(fabsf(acc.x), fabsf(acc.y)), fmaxf(fabsf(acc.z), fabsf(acc.w))));
                    left = fmaxf(left, fmaxf(fmaxf(fabsf(y.x), fabsf(y.y)), fmaxf(fabsf(y.z), fabsf(y.w))));
                }
            }
        }
        if (a.accumulate && a.guard) {
#pragma unroll
            for (int s = 32; s >= 1; s >>= 1) { big = fmaxf(big, __shfl_xor(big, s, 64)); left = fmaxf(left, __shfl_xor(left, s, 64)); }
            if (big > GUARD_RATIO * left) {                  // cancelled: rebuild the hub's row in full
                if (D <= 256) {
                    float4 full[1];
                    full_row<64, 1>(a, rec.v, rec.off, rec.deg, lane, full);
                    if (lane * 4 < D) *reinterpret_cast<float4*>(a.S + (int64_t)rec.v * D + lane * 4) = full[0];
                } else {
                    float4 full[4];
                    full_row<64, 4>(a, rec.v, rec.off, rec.deg, lane, full);
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        if (lane * 4 + q * 256 < D) *reinterpret_cast<float4*>(a.S + (int64_t)rec.v * D + lane * 4 + q * 256) = full[q];
                }
            }
        }
    }
}

// ------------------------------------------------------------------ layer-0 delta payloads
// one wave per source of change at layer 1: replaced features and (GCN) re-normalised payloads
__global__ void layer0_delta_kernel(DeltaArgs a) {
    const int64_t s = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int lane = threadIdx.x & 63;
    if (s >= (int64_t)*a.n_dev) return;
    const int32_t v = a.list[s];
    const bool isfeat = (a.feat_bitmap[v >> 5] >> (v & 31)) & 1u;
    float cn = 1.0f, co = 1.0f;
    if (a.indeg_new) { cn = gcn_scale(a.indeg_new[v]); co = gcn_scale(a.indeg_old[v]); }
    float* h = a.H0 + (int64_t)v * a.D;
    const float* fresh = isfeat ? a.feat_rows + (int64_t)a.feat_index[v] * a.D : h;
    float* dp = a.DP + s * a.D;
    for (int k = lane * 4; k < a.D; k += 256) {
        const float4 xo = *reinterpret_cast<const float4*>(h + k);
        const float4 xn = isfeat ? *reinterpret_cast<const float4*>(fresh + k) : xo;
        float4 d;
        d.x = xn.x * cn - xo.x * co; d.y = xn.y * cn - xo.y * co; d.z = xn.z * cn - xo.z * co; d.w = xn.w * cn - xo.w * co;
        *reinterpret_cast<float4*>(dp + k) = a.store_old ? xo : d;
        if (isfeat) *reinterpret_cast<float4*>(h + k) = xn;
    }
}

}  // namespace

nrt_status k_dst_records(const int32_t* list, int64_t bound, const Adj& in, DstRec* recs, const HubWork& hubs,
                         LayerCtrs* lc, bool all_vertices, const uint64_t* plain_if_zero, hipStream_t s) {
    if (bound <= 0) return NRT_OK;
    int64_t g = cdiv(bound, (int64_t)REC_THREADS * REC_EPT);
    if (g > 1024) g = 1024;
    dst_records_kernel<<<(int)g, REC_THREADS, 0, s>>>(all_vertices ? nullptr : list, bound, in, recs, hubs, lc, plain_if_zero);
    LAUNCH_CHECK();
    return NRT_OK;
}

template <int LPR, int NV>
static void launch_gather(const GatherArgs& a, hipStream_t s) {
    // a fixed grid strides over the work (sizes are read on the device); sized to the previous batch's work when known
    int nb = 8192, sp_blocks = SP_BLOCKS;
    if (a.units_hint > 0) {
        const int64_t want = cdiv(a.units_hint + a.units_hint / 4 + 64, WAVES_PER_BLOCK);
        nb = (int)(want < 128 ? 128 : (want > 8192 ? 8192 : want));
        const int64_t want_sp = cdiv(a.units_hint + a.units_hint / 4 + 64, 4 * SP_WAVES);
        sp_blocks = (int)(want_sp < 64 ? 64 : (want_sp > SP_BLOCKS ? SP_BLOCKS : want_sp));
    }
    const int threads = WAVES_PER_BLOCK * 64;
    const bool filter = a.src_bitmap != nullptr;
    const int coef = a.rel_R ? 2 : ((a.use_weights || a.src_scale_gcn) ? 1 : 0);
    auto sparse = [&]() {
        if (coef == 2) gather_sparse_kernel<LPR, 2><<<sp_blocks, SP_WAVES * 64, 0, s>>>(a);
        else if (coef) gather_sparse_kernel<LPR, 1><<<sp_blocks, SP_WAVES * 64, 0, s>>>(a);
        else gather_sparse_kernel<LPR, 0><<<sp_blocks, SP_WAVES * 64, 0, s>>>(a);
    };
    if (NV == 1 && a.sparse_ok == 2) {
        sparse();
        return;
    }
    if (filter) {
        if (coef == 2) gather_kernel<LPR, NV, true, 2><<<nb, threads, 0, s>>>(a);
        else if (coef) gather_kernel<LPR, NV, true, 1><<<nb, threads, 0, s>>>(a);
        else gather_kernel<LPR, NV, true, 0><<<nb, threads, 0, s>>>(a);
    } else {
        if (coef == 2) gather_kernel<LPR, NV, false, 2><<<nb, threads, 0, s>>>(a);
        else if (coef) gather_kernel<LPR, NV, false, 1><<<nb, threads, 0, s>>>(a);
        else gather_kernel<LPR, NV, false, 0><<<nb, threads, 0, s>>>(a);
    }
    if (NV == 1 && a.sparse_ok) {
        ++nrt_launch_count;                     // the second launch of this call
        sparse();
    }
}

nrt_status k_gather(const GatherArgs& a, hipStream_t s) {
    if (a.rel_R && (a.guard || a.self_pair || a.src_scale_gcn)) {
        nrt_set_error("gather: typed edges combine with neither the cancellation guard nor the GCN terms");
        return NRT_ERR_INVALID_ARG;
    }
    if (a.D <= 64) launch_gather<16, 1>(a, s);
    else if (a.D <= 128) launch_gather<32, 1>(a, s);
    else if (a.D <= 256) launch_gather<64, 1>(a, s);
    else if (a.D <= 512) launch_gather<64, 2>(a, s);
    else launch_gather<64, 4>(a, s);
    LAUNCH_CHECK();
    return NRT_OK;
}

nrt_status k_coarse_bitmap(const uint32_t* fine, int64_t n, int shift, uint32_t* coarse, int64_t n_words, hipStream_t s) {
    if (n_words <= 0) return NRT_OK;
    coarse_bitmap_kernel<<<(int)cdiv(n_words, 256), 256, 0, s>>>(fine, n, shift, coarse, n_words);
    LAUNCH_CHECK();
    return NRT_OK;
}

nrt_status k_combine_partials(const GatherArgs& a, hipStream_t s) {
    int nb = 2048;                              // one wave per hub, strided
    if (a.units_hint > 0) {
        const int64_t want = cdiv(a.hubs_hint + a.hubs_hint / 4 + 16, 4);
        nb = (int)(want < 16 ? 16 : (want > 2048 ? 2048 : want));
    }
    combine_kernel<<<nb, 256, 0, s>>>(a);
    LAUNCH_CHECK();
    return NRT_OK;
}

nrt_status k_layer0_delta(const DeltaArgs& a, hipStream_t s) {
    if (a.bound <= 0) return NRT_OK;
    layer0_delta_kernel<<<(int)cdiv(a.bound * 64, 256), 256, 0, s>>>(a);
    LAUNCH_CHECK();
    return NRT_OK;
}
