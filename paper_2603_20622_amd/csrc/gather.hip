// Delta-message gather and fold (Algorithm 1 lines 1-6 with the aggregate cached in context-free form).
//
// For every affected destination v the cached sum S[v] = sum_u c_uv p_u receives the changes of its
// affected in-neighbours: S[v] += sum_{u in N_new(v), u changed} c_uv * dp_u, where dp_u is the change of
// the source payload (already formed by the previous layer's write-back).  The terms of inserted and
// deleted edges are folded beforehand on the old caches (k_structural_fold): +c p_u(old) for an inserted
// edge, -c p_u(old) for a deleted one, so that an inserted edge whose source also changed sums to
// c p_u(new) (Section IV-B: insert = positive message, delete = negative, update = both).
//
// The same kernel, with no source filter and rows read straight from h^{l-1}, is the full-neighbour
// aggregation of Eq. 1 used by nrt_cache_init.
//
// Mapping to the machine: destinations are walked through their in-lists (no atomics, no sort: each
// destination row is owned by one wave).  An in-list is cut into items of NRT_CHUNK entries; a wave stages the
// ids of one item, filters them against the bitmap of changed sources with a ballot/prefix-count, keeps the
// surviving (row, coefficient) pairs in LDS and then streams the rows: one 16-byte load per lane, so a
// 256-float row is one fully coalesced 1 KiB wave load (narrower rows put 2 or 4 neighbours in one load).
// Destinations with more than one item write partial rows that a second small kernel sums in item order,
// which keeps a 100k-degree hub from serialising on one wave and keeps the result order-deterministic.
#include "common.h"

namespace {

constexpr int WAVES_PER_BLOCK = 4;

__device__ inline float4 f4_fma(float c, float4 x, float4 a) {
    a.x = fmaf(c, x.x, a.x); a.y = fmaf(c, x.y, a.y); a.z = fmaf(c, x.z, a.z); a.w = fmaf(c, x.w, a.w);
    return a;
}
__device__ inline float4 f4_add(float4 a, float4 b) { return make_float4(a.x + b.x, a.y + b.y, a.z + b.z, a.w + b.w); }
__device__ inline float4 f4_shfl_xor(float4 a, int m) {
    return make_float4(__shfl_xor(a.x, m, 64), __shfl_xor(a.y, m, 64), __shfl_xor(a.z, m, 64), __shfl_xor(a.w, m, 64));
}
__device__ inline float gcn_scale(int32_t indeg) { return 1.0f / sqrtf((float)(indeg + 1)); }

// ------------------------------------------------------------------ items
__global__ void item_count_kernel(const int32_t* dst_list, int64_t n_dst, const int32_t* indeg, uint64_t* item_off,
                                  unsigned long long* inedge_sum) {
    const int64_t s = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    unsigned long long d = 0;
    if (s < n_dst) {
        const int32_t v = dst_list ? dst_list[s] : (int32_t)s;
        d = (unsigned long long)indeg[v];
        const uint64_t nch = d > NRT_CHUNK ? (d + NRT_CHUNK - 1) / NRT_CHUNK : 1;
        item_off[s] = nch | ((nch > 1 ? nch : 0) << 32);
    }
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) d += __shfl_xor(d, m, 64);
    if ((threadIdx.x & 63) == 0 && d) atomicAdd(inedge_sum, d);
}
__global__ void item_fill_kernel(const int32_t* dst_list, int64_t n_dst, const int32_t* indeg, const uint64_t* item_off,
                                 int32_t* item_slot, int32_t* item_chunk, int32_t* multi_list,
                                 unsigned long long* n_multi) {
    const int64_t s = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (s >= n_dst) return;
    const int32_t v = dst_list ? dst_list[s] : (int32_t)s;
    const int32_t d = indeg[v];
    const int32_t nch = d > NRT_CHUNK ? (d + NRT_CHUNK - 1) / NRT_CHUNK : 1;
    const uint32_t first = (uint32_t)(item_off[s] & 0xffffffffu);
    for (int32_t c = 0; c < nch; ++c) {
        item_slot[first + c] = (int32_t)s;
        item_chunk[first + c] = c;
    }
    if (nch > 1) multi_list[atomicAdd(n_multi, 1ULL)] = (int32_t)s;
}

// ------------------------------------------------------------------ gather
template <int LPR>   // lanes per row
__global__ void __launch_bounds__(WAVES_PER_BLOCK * 64) gather_kernel(GatherArgs a) {
    constexpr int RPI = 64 / LPR;   // rows fetched by one wave-wide load
    __shared__ int32_t s_row[WAVES_PER_BLOCK][NRT_CHUNK + 1];
    __shared__ float s_coef[WAVES_PER_BLOCK][NRT_CHUNK + 1];
    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int64_t item = (int64_t)blockIdx.x * WAVES_PER_BLOCK + w;
    const int64_t n_items = (int64_t)(*a.n_items_dev & 0xffffffffu);
    if (item >= n_items) return;
    const int32_t s = a.item_slot[item];
    const int32_t chunk = a.item_chunk[item];
    const int32_t v = a.dst_list ? a.dst_list[s] : s;
    const int32_t deg = a.in.deg[v];
    const int64_t base = a.in.off[v] + (int64_t)chunk * NRT_CHUNK;
    const int32_t cnt = min(NRT_CHUNK, deg - chunk * NRT_CHUNK);
    int32_t* rows = s_row[w];
    float* coefs = s_coef[w];

    // stage the surviving (row, coefficient) pairs of this item
    int nvalid = 0;
    for (int j = 0; j < cnt; j += 64) {
        const int jj = j + lane;
        bool ok = jj < cnt;
        int32_t u = 0;
        if (ok) {
            u = a.in.idx[base + jj];
            if (a.src_bitmap) ok = (a.src_bitmap[u >> 5] >> (u & 31)) & 1u;
        }
        const unsigned long long m = __ballot(ok);
        if (ok) {
            const int pos = nvalid + __popcll(m & ((1ULL << lane) - 1ULL));
            float c = a.use_weights ? a.in.wts[base + jj] : 1.0f;
            if (a.src_scale_gcn) c *= gcn_scale(a.in.deg[u]);
            rows[pos] = a.src_bitmap ? a.src_slot[u] : u;
            coefs[pos] = c;
        }
        nvalid += __popcll(m);
    }
    if (a.self_pair && chunk == 0) {
        bool ok = true;
        if (a.src_bitmap) ok = (a.src_bitmap[v >> 5] >> (v & 31)) & 1u;
        if (ok) {
            if (lane == 0) {
                rows[nvalid] = a.src_bitmap ? a.src_slot[v] : v;
                coefs[nvalid] = a.src_scale_gcn ? gcn_scale(deg) : 1.0f;
            }
            nvalid += 1;
        }
    }
    if (a.pair_ctr && lane == 0 && nvalid) atomicAdd(&a.pair_ctr[blockIdx.x & 1023], (unsigned long long)nvalid);
    __builtin_amdgcn_wave_barrier();
    __threadfence_block();

    const uint64_t off = a.item_off[s];
    const bool multi = deg > NRT_CHUNK;
    const int sub = lane / LPR;
    const int D = a.D;
    for (int cb = 0; cb < D; cb += LPR * 4) {
        const int col = cb + (lane % LPR) * 4;
        const bool live = col < D;
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        float4 old = acc;
        float* dstp = multi ? a.partial + ((int64_t)(off >> 32) + chunk) * D + col : a.S + (int64_t)v * D + col;
        if (live && !multi && a.accumulate) old = *reinterpret_cast<const float4*>(dstp);
        if (live) {
            const float* P = a.P + col;
            int i = sub;
            for (; i + 3 * RPI < nvalid; i += 4 * RPI) {
                const int32_t r0 = rows[i], r1 = rows[i + RPI], r2 = rows[i + 2 * RPI], r3 = rows[i + 3 * RPI];
                const float c0 = coefs[i], c1 = coefs[i + RPI], c2 = coefs[i + 2 * RPI], c3 = coefs[i + 3 * RPI];
                const float4 x0 = *reinterpret_cast<const float4*>(P + (int64_t)r0 * D);
                const float4 x1 = *reinterpret_cast<const float4*>(P + (int64_t)r1 * D);
                const float4 x2 = *reinterpret_cast<const float4*>(P + (int64_t)r2 * D);
                const float4 x3 = *reinterpret_cast<const float4*>(P + (int64_t)r3 * D);
                acc = f4_fma(c0, x0, acc);
                acc = f4_fma(c1, x1, acc);
                acc = f4_fma(c2, x2, acc);
                acc = f4_fma(c3, x3, acc);
            }
            for (; i < nvalid; i += RPI) {
                const float4 x0 = *reinterpret_cast<const float4*>(P + (int64_t)rows[i] * D);
                acc = f4_fma(coefs[i], x0, acc);
            }
        }
#pragma unroll
        for (int m = LPR; m < 64; m <<= 1) acc = f4_add(acc, f4_shfl_xor(acc, m));
        if (live && sub == 0) {
            if (!multi && a.accumulate) acc = f4_add(acc, old);
            *reinterpret_cast<float4*>(dstp) = acc;
        }
    }
}

// one wave per multi-item destination: sum its partial rows in item order
__global__ void combine_kernel(GatherArgs a, const int32_t* multi_list, int64_t n_multi) {
    const int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int lane = threadIdx.x & 63;
    if (i >= n_multi) return;
    const int32_t s = multi_list[i];
    const int32_t v = a.dst_list ? a.dst_list[s] : s;
    const int32_t deg = a.in.deg[v];
    const int32_t nch = (deg + NRT_CHUNK - 1) / NRT_CHUNK;
    const int64_t pfirst = (int64_t)(a.item_off[s] >> 32);
    const int D = a.D;
    for (int col = lane * 4; col < D; col += 256) {
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int32_t c = 0; c < nch; ++c)
            acc = f4_add(acc, *reinterpret_cast<const float4*>(a.partial + (pfirst + c) * D + col));
        float4* dst = reinterpret_cast<float4*>(a.S + (int64_t)v * D + col);
        if (a.accumulate) acc = f4_add(acc, *dst);
        *dst = acc;
    }
}

// ------------------------------------------------------------------ structural fold
// one wave per updated edge: S[dst] += sign * c * p_src(old)
__global__ void structural_fold_kernel(FoldArgs a) {
    const int64_t op = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int lane = threadIdx.x & 63;
    if (op >= a.n_ins + a.n_del) return;
    const bool is_del = op >= a.n_ins;
    const int64_t i = is_del ? op - a.n_ins : op;
    const int32_t u = is_del ? a.del_src[i] : a.ins_src[i];
    const int32_t v = is_del ? a.del_dst[i] : a.ins_dst[i];
    float c = is_del ? -1.0f : 1.0f;
    if (is_del && a.del_w) c *= a.del_w[i];
    if (!is_del && a.ins_w) c *= a.ins_w[i];
    if (a.indeg_old) c *= gcn_scale(a.indeg_old[u]);
    const float* src = a.Hprev + (int64_t)u * a.D;
    float* dst = a.S + (int64_t)v * a.D;
    for (int k = lane; k < a.D; k += 64) unsafeAtomicAdd(dst + k, c * src[k]);
}

// ------------------------------------------------------------------ layer-0 delta payloads
// one wave per source of change at layer 1: replaced features and (GCN) re-normalised payloads
__global__ void layer0_delta_kernel(DeltaArgs a) {
    const int64_t s = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int lane = threadIdx.x & 63;
    if (s >= a.n) return;
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
        *reinterpret_cast<float4*>(dp + k) = d;
        if (isfeat) *reinterpret_cast<float4*>(h + k) = xn;
    }
}

}  // namespace

nrt_status k_build_items(const int32_t* dst_list, int64_t n_dst, const int32_t* indeg, uint64_t* item_off,
                         int32_t* item_slot, int32_t* item_chunk, int32_t* multi_list, uint64_t* scan_tmp,
                         int64_t scan_tmp_len, int64_t* dev_ctrs, hipStream_t s) {
    NRT_TRY(k_fill_u64((uint64_t*)(dev_ctrs + CTR_ITEMS), 3, 0, s));
    if (n_dst <= 0) return NRT_OK;
    const int nb = (int)cdiv(n_dst, 256);
    item_count_kernel<<<nb, 256, 0, s>>>(dst_list, n_dst, indeg, item_off, (unsigned long long*)(dev_ctrs + CTR_INEDGES));
    LAUNCH_CHECK();
    NRT_TRY(k_exclusive_scan_u64(item_off, n_dst, scan_tmp, scan_tmp_len, (uint64_t*)(dev_ctrs + CTR_ITEMS), s));
    item_fill_kernel<<<nb, 256, 0, s>>>(dst_list, n_dst, indeg, item_off, item_slot, item_chunk, multi_list,
                                        (unsigned long long*)(dev_ctrs + CTR_MULTI));
    LAUNCH_CHECK();
    return NRT_OK;
}

nrt_status k_gather(const GatherArgs& a, int64_t n_items, hipStream_t s) {
    if (n_items <= 0) return NRT_OK;
    const int nb = (int)cdiv(n_items, WAVES_PER_BLOCK);
    if (a.D <= 64) gather_kernel<16><<<nb, WAVES_PER_BLOCK * 64, 0, s>>>(a);
    else if (a.D <= 128) gather_kernel<32><<<nb, WAVES_PER_BLOCK * 64, 0, s>>>(a);
    else gather_kernel<64><<<nb, WAVES_PER_BLOCK * 64, 0, s>>>(a);
    LAUNCH_CHECK();
    return NRT_OK;
}

nrt_status k_combine_partials(const GatherArgs& a, const int32_t* multi_list, int64_t n_multi, hipStream_t s) {
    if (n_multi <= 0) return NRT_OK;
    combine_kernel<<<(int)cdiv(n_multi * 64, 256), 256, 0, s>>>(a, multi_list, n_multi);
    LAUNCH_CHECK();
    return NRT_OK;
}

nrt_status k_structural_fold(const FoldArgs& a, hipStream_t s) {
    const int64_t nops = a.n_ins + a.n_del;
    if (nops <= 0) return NRT_OK;
    structural_fold_kernel<<<(int)cdiv(nops * 64, 256), 256, 0, s>>>(a);
    LAUNCH_CHECK();
    return NRT_OK;
}

nrt_status k_layer0_delta(const DeltaArgs& a, hipStream_t s) {
    if (a.n <= 0) return NRT_OK;
    layer0_delta_kernel<<<(int)cdiv(a.n * 64, 256), 256, 0, s>>>(a);
    LAUNCH_CHECK();
    return NRT_OK;
}
