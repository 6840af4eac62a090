// A-GNN (Table II): the message of an edge <u,v> is w * cos(h_v, h_u) * h_u, summed over the in-neighbours.
// G-GCN (Table II) shares every kernel of this file (template flag GATE): its message is sigmoid(W_1 h_u + W_2 h_v) * h_u
// element by element, with the two projections cached per vertex (and the old W_1 h_u of the changed vertices kept
// compact next to their old rows).
//
// The coefficient reads the destination's own embedding, so the model is one of the paper's constrained ones
// (Section III-D): a destination whose own h^{l-1} changed is summed again over its whole in-neighbourhood; every
// other affected destination only exchanges the terms of its changed in-neighbours, c_new h_new - c_old h_old, where
// the old term is recomputed from the old row and the old norm kept compact for the changed vertices (the role the
// cached per-edge attention plays in Algorithm 3).  Deleted and inserted in-edges contribute their terms on the old
// caches, folded into one compact row per destination before the graph changes, exactly as for the other models.
//
// Cached per layer: h^{l-1} (the layer input), the inverse norm of each of its rows (0 for a zero row, whose cosine
// is taken as 0), and the aggregate a_v.  Destinations with long in-lists are served through their items (partial
// rows of the sum or of the exchange), added up by the combine kernel below.
#include "common.h"

namespace {

constexpr int AG_WAVES = 4;        // waves per workgroup
constexpr int AG_BLOCKS = 4096;    // fixed grid: sizes are read on the device
constexpr int AG_TERMS = 4;        // row slots loaded together by a wave
constexpr int AG_LIST = 2 * AG_TERMS;     // terms handed over at a time (two per slot for rows of up to 128 floats)
constexpr float AG_GUARD_RATIO = 16.0f;   // an exchange larger than this many times what it leaves is redone in full

__device__ inline float wave_sum(float x) {
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) x += __shfl_xor(x, s, 64);
    return x;
}

__device__ inline bool in_set(const uint32_t* bm, int32_t v) { return (bm[(uint32_t)v >> 5] >> (v & 31)) & 1u; }

__device__ inline float sigmoidf(float x) { return 1.0f / (1.0f + expf(-x)); }

// A-GNN: acc += sum_t c[t] * (hv . row_t) * row_t for t < nt (uniform over the wave); the rows are loaded together.
// G-GCN (GATE): acc += sum_t c[t] * sigmoid(aux_t + hv) * row_t element by element (hv = the destination's W_2 h_v,
// aux_t = the source's W_1 h_u), c[t] = +-1.
// HALF (rows of up to 128 floats): a row takes 32 lanes, so the two halves of the wave take terms 2s and 2s+1 of row
// slot s; each half accumulates its own partial row, the caller adds the halves.  A slot beyond nt points at row 0
// with c = 0.
template <int NV, bool GATE, bool HALF>
__device__ inline void add_terms(const float* (&row)[AG_LIST], const float* (&aux)[AG_LIST], const float (&c)[AG_LIST],
                                 int nt, const float4 (&hv)[NV], float4 (&acc)[NV], const bool (&live)[NV], int lane,
                                 int col0) {
    const bool hi = HALF && lane >= 32;
    const float* r[AG_TERMS];
    const float* g1[AG_TERMS];
    float cc[AG_TERMS];
    bool on[AG_TERMS];
#pragma unroll
    for (int t = 0; t < AG_TERMS; ++t) {
        if (HALF) {
            r[t] = hi ? row[2 * t + 1] : row[2 * t];
            g1[t] = hi ? aux[2 * t + 1] : aux[2 * t];
            cc[t] = hi ? c[2 * t + 1] : c[2 * t];
            on[t] = 2 * t < nt;
        } else {
            r[t] = row[t]; g1[t] = aux[t]; cc[t] = c[t];
            on[t] = t < nt;
        }
    }
    float4 x[AG_TERMS][NV];
    if (GATE) {
        float4 g[AG_TERMS][NV];
#pragma unroll
        for (int t = 0; t < AG_TERMS; ++t)
#pragma unroll
            for (int q = 0; q < NV; ++q) {
                x[t][q] = make_float4(0.f, 0.f, 0.f, 0.f);
                g[t][q] = x[t][q];
                if (on[t] && live[q]) {
                    x[t][q] = *reinterpret_cast<const float4*>(r[t] + col0 + q * 256);
                    g[t][q] = *reinterpret_cast<const float4*>(g1[t] + col0 + q * 256);
                }
            }
#pragma unroll
        for (int t = 0; t < AG_TERMS; ++t)
#pragma unroll
            for (int q = 0; q < NV; ++q) {
                acc[q].x += cc[t] * sigmoidf(g[t][q].x + hv[q].x) * x[t][q].x;
                acc[q].y += cc[t] * sigmoidf(g[t][q].y + hv[q].y) * x[t][q].y;
                acc[q].z += cc[t] * sigmoidf(g[t][q].z + hv[q].z) * x[t][q].z;
                acc[q].w += cc[t] * sigmoidf(g[t][q].w + hv[q].w) * x[t][q].w;
            }
        return;
    }
    float d[AG_TERMS];
#pragma unroll
    for (int t = 0; t < AG_TERMS; ++t) {
        d[t] = 0.f;
#pragma unroll
        for (int q = 0; q < NV; ++q) {
            x[t][q] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (on[t] && live[q]) x[t][q] = *reinterpret_cast<const float4*>(r[t] + col0 + q * 256);
        }
    }
#pragma unroll
    for (int t = 0; t < AG_TERMS; ++t)
#pragma unroll
        for (int q = 0; q < NV; ++q)
            d[t] += hv[q].x * x[t][q].x + hv[q].y * x[t][q].y + hv[q].z * x[t][q].z + hv[q].w * x[t][q].w;
#pragma unroll
    for (int s = HALF ? 16 : 32; s >= 1; s >>= 1)         // HALF: the sums stay inside each half of the wave
#pragma unroll
        for (int t = 0; t < AG_TERMS; ++t) d[t] += __shfl_xor(d[t], s, 64);
#pragma unroll
    for (int t = 0; t < AG_TERMS; ++t) {
        const float k = cc[t] * d[t];                        // zero rows and c = 0 beyond nt: nothing is added
#pragma unroll
        for (int q = 0; q < NV; ++q) {
            acc[q].x += k * x[t][q].x; acc[q].y += k * x[t][q].y;
            acc[q].z += k * x[t][q].z; acc[q].w += k * x[t][q].w;
        }
    }
}

// acc += the terms of in-list entries [base, base + cnt) for destination row hv (cv = w / |h_v|): every entry when
// `full`, else the exchange new - old of the entries whose source changed.  Returns the number of rows' sources used.
template <int NV, bool GATE, bool HALF>
__device__ inline int sum_terms(const AgnnArgs& a, int64_t base, int32_t cnt, bool full, const float4 (&hv)[NV], float cv,
                                float4 (&acc)[NV], const bool (&live)[NV], int lane, int col0) {
    constexpr int NT = HALF ? AG_LIST : AG_TERMS;          // terms per hand-over
    const int D = a.D;
    int pairs = 0;
    for (int32_t j0 = 0; j0 < cnt; j0 += 64) {
        const int32_t j = j0 + lane;
        const int32_t u = j < cnt ? a.in.idx[base + j] : -1;
        bool take = u >= 0;
        int32_t slot = 0;
        if (!full) {
            take = take && in_set(a.src_bitmap, u);
            if (take) slot = a.src_slot[u];
        }
        const float ru = GATE ? 1.0f : (take ? a.R[u] : 0.f);
        const float ro = GATE ? 1.0f : ((take && !full) ? a.old_r[slot] : 0.f);
        unsigned long long m = __ballot(take);
        pairs += __popcll(m);
        // in in-list order, a few rows at a time: the sum does not depend on the schedule
        while (m) {
            const float* row[AG_LIST];
            const float* aux[AG_LIST];
            float c[AG_LIST];
#pragma unroll
            for (int t = 0; t < AG_LIST; ++t) { row[t] = a.H; aux[t] = a.H; c[t] = 0.f; }
            int nt = 0;
            if (full) {
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    if (m) {
                        const int b = __ffsll((long long)m) - 1;
                        m &= m - 1;
                        const int64_t uu = __shfl(u, b, 64);
                        row[t] = a.H + uu * D;
                        if (GATE) aux[t] = a.P1 + uu * D;
                        c[t] = cv * __shfl(ru, b, 64);
                        nt = t + 1;
                    }
                }
            } else if (HALF) {
                // two changed in-neighbours per pair of row slots, one per half of the wave: slot 2p holds their new
                // terms, slot 2p + 1 their old ones, so that each half adds a neighbour's new term and takes its old
                // one away back to back (the running sum stays as small as the exchange itself)
#pragma unroll
                for (int p = 0; p < AG_LIST / 4; ++p) {
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        if (m) {
                            const int b = __ffsll((long long)m) - 1;
                            m &= m - 1;
                            const int64_t uu = __shfl(u, b, 64), ss = __shfl(slot, b, 64);
                            row[4 * p + h] = a.H + uu * D;
                            c[4 * p + h] = cv * __shfl(ru, b, 64);
                            row[4 * p + 2 + h] = a.old_rows + ss * D;
                            c[4 * p + 2 + h] = -cv * __shfl(ro, b, 64);
                            if (GATE) { aux[4 * p + h] = a.P1 + uu * D; aux[4 * p + 2 + h] = a.old_p1 + ss * D; }
                            nt = 4 * p + 4;
                        }
                    }
                }
            } else {                                      // the new term of a changed in-neighbour minus its old one
#pragma unroll
                for (int t = 0; t < NT; t += 2) {
                    if (m) {
                        const int b = __ffsll((long long)m) - 1;
                        m &= m - 1;
                        const int64_t uu = __shfl(u, b, 64), ss = __shfl(slot, b, 64);
                        row[t] = a.H + uu * D;
                        c[t] = cv * __shfl(ru, b, 64);
                        row[t + 1] = a.old_rows + ss * D;
                        c[t + 1] = -cv * __shfl(ro, b, 64);
                        if (GATE) { aux[t] = a.P1 + uu * D; aux[t + 1] = a.old_p1 + ss * D; }
                        nt = t + 2;
                    }
                }
            }
            add_terms<NV, GATE, HALF>(row, aux, c, nt, hv, acc, live, lane, col0);
        }
    }
    return pairs;
}

// R[v] = 1 / |h_v| for the listed rows (list null: rows 0 .. n_all); r_old[m] keeps the value it replaces
__global__ void agnn_norms_kernel(const int32_t* list, const uint64_t* count_dev, int64_t bound, const float* H, int D,
                                  float* R, float* r_old) {
    const int lane = threadIdx.x & 63;
    int64_t count = list ? (int64_t)*count_dev : bound;
    if (count > bound) count = bound;
    const int64_t waves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    for (int64_t m = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6; m < count; m += waves) {
        const int64_t v = list ? (int64_t)list[m] : m;
        const float* row = H + v * D;
        float s = 0.f;
        for (int k = lane * 4; k < D; k += 256) {
            const float4 x = *reinterpret_cast<const float4*>(row + k);
            s += x.x * x.x + x.y * x.y + x.z * x.z + x.w * x.w;
        }
        s = wave_sum(s);
        if (lane == 0) {
            if (r_old) r_old[m] = R[v];
            R[v] = s > 0.f ? 1.0f / sqrtf(s) : 0.f;
        }
    }
}

// One wave per unit (a destination with a short in-list, or one item of a long one).  NV: 16-byte pieces of a row
// per lane (rows of up to 256 * NV floats).
template <int NV, bool GATE, bool HALF>
__global__ void __launch_bounds__(AG_WAVES * 64) agnn_gather_kernel(AgnnArgs a) {
    const int lane = threadIdx.x & 63;
    const int col0 = HALF ? (lane & 31) * 4 : lane * 4;    // HALF: both halves of the wave cover the same columns
    const bool writer = !HALF || lane < 32;
    const int D = a.D;
    const int64_t n_dst = (int64_t)a.lc->count;
    int64_t n_items = (int64_t)a.lc->n_items;
    if (n_items > a.hubs.item_cap) n_items = a.hubs.item_cap;
    const int64_t total = n_dst + n_items;
    const int64_t waves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    bool live[NV];
#pragma unroll
    for (int q = 0; q < NV; ++q) live[q] = col0 + q * 256 < D;
    long long pairs = 0;

    for (int64_t unit = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6; unit < total; unit += waves) {
        DstRec rec;
        int32_t cnt;
        int64_t base;
        bool part;
        int32_t chunk = 0;
        if (unit >= n_items) {
            rec = a.recs[unit - n_items];
            if (rec.deg > NRT_CHUNK) continue;               // served through its items
            cnt = rec.deg; base = rec.off; part = false;
        } else {
            chunk = a.hubs.item_chunk[unit];
            rec = a.recs[a.hubs.hub_slot[a.hubs.item_hub[unit]]];
            cnt = min(NRT_CHUNK, rec.deg - chunk * NRT_CHUNK);
            base = rec.off + (int64_t)chunk * NRT_CHUNK;
            part = true;
        }
        const int32_t v = rec.v;
        bool full = !a.incremental || in_set(a.src_bitmap, v);   // uniform over the wave
        float4 hv[NV], acc[NV];
#pragma unroll
        for (int q = 0; q < NV; ++q) {
            hv[q] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (live[q]) hv[q] = *reinterpret_cast<const float4*>((GATE ? a.P2 : a.H) + (int64_t)v * D + col0 + q * 256);
        }
        const float cv = GATE ? 1.0f : a.beta * a.R[v];

      // at most two passes: an exchange that cancels most of the row is redone as a full sum (see below)
      for (;;) {
#pragma unroll
        for (int q = 0; q < NV; ++q) acc[q] = make_float4(0.f, 0.f, 0.f, 0.f);
        pairs += sum_terms<NV, GATE, HALF>(a, base, cnt, full, hv, cv, acc, live, lane, col0);
        if (HALF) {                                           // the two halves summed different terms
#pragma unroll
            for (int q = 0; q < NV; ++q) {
                acc[q].x += __shfl_xor(acc[q].x, 32, 64); acc[q].y += __shfl_xor(acc[q].y, 32, 64);
                acc[q].z += __shfl_xor(acc[q].z, 32, 64); acc[q].w += __shfl_xor(acc[q].w, 32, 64);
            }
        }

        if (part) {
            // an item holds its share of the whole sum, or of the exchange (the first item also takes the structural
            // terms); the combine kernel adds the items up and, for an exchange, applies the guard
            const bool dd0 = !full && chunk == 0 && a.sd && in_set(a.dd_bitmap, v);
            const float* sd0 = dd0 ? a.sd + (int64_t)a.dd_slot[v] * D : nullptr;
#pragma unroll
            for (int q = 0; q < NV; ++q) {
                if (!live[q] || !writer) continue;
                float4 d = acc[q];
                if (dd0) {
                    const float4 e = *reinterpret_cast<const float4*>(sd0 + col0 + q * 256);
                    d.x += e.x; d.y += e.y; d.z += e.z; d.w += e.w;
                }
                *reinterpret_cast<float4*>(a.hubs.partial + unit * D + col0 + q * 256) = d;
            }
            break;
        }
        float* out = a.S + (int64_t)v * D;
        if (full) {
#pragma unroll
            for (int q = 0; q < NV; ++q)
                if (live[q] && writer) *reinterpret_cast<float4*>(out + col0 + q * 256) = acc[q];
            break;
        }
        const bool dd = a.sd && in_set(a.dd_bitmap, v);
        const float* sdrow = dd ? a.sd + (int64_t)a.dd_slot[v] * D : nullptr;
        float4 y[NV];
        float big = 0.f, left = 0.f;
#pragma unroll
        for (int q = 0; q < NV; ++q) {
            y[q] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (!live[q]) continue;
            float4 d = acc[q];
            if (dd) {
                const float4 e = *reinterpret_cast<const float4*>(sdrow + col0 + q * 256);
                d.x += e.x; d.y += e.y; d.z += e.z; d.w += e.w;
            }
            const float4 o = *reinterpret_cast<const float4*>(out + col0 + q * 256);
            y[q] = make_float4(o.x + d.x, o.y + d.y, o.z + d.z, o.w + d.w);
            big = fmaxf(big, fmaxf(fmaxf(fabsf(d.x), fabsf(d.y)), fmaxf(fabsf(d.z), fabsf(d.w))));
            left = fmaxf(left, fmaxf(fmaxf(fabsf(y[q].x), fabsf(y[q].y)), fmaxf(fabsf(y[q].z), fabsf(y[q].w))));
        }
#pragma unroll
        for (int sft = 32; sft >= 1; sft >>= 1) {
            big = fmaxf(big, __shfl_xor(big, sft, 64));
            left = fmaxf(left, __shfl_xor(left, sft, 64));
        }
        // Cancellation guard.  What an exchange leaves of a row that it mostly removes is rounding residue of the
        // removed terms; the next layer normalises this row (cosine), which would turn a residue of 1e-11 into a
        // direction.  Such a row is summed again over the whole in-list (an exact zero stays an exact zero).
        if (big > AG_GUARD_RATIO * left) { full = true; continue; }
#pragma unroll
        for (int q = 0; q < NV; ++q)
            if (live[q] && writer) *reinterpret_cast<float4*>(out + col0 + q * 256) = y[q];
        break;
      }
    }
    if (a.pair_ctr && lane == 0 && pairs) atomicAdd(&a.pair_ctr[blockIdx.x & 1023], (unsigned long long)pairs);
}

// One wave per destination with a long in-list: its items' rows are added up in item order.  They are the whole sum when
// the destination's own row changed (or nothing is incremental), else an exchange that is added to the cached
// aggregate under the same guard as above; a guarded destination is summed again over its whole in-list by this wave.
template <int NV, bool GATE>
__global__ void __launch_bounds__(AG_WAVES * 64) agnn_combine_kernel(AgnnArgs a) {
    const int lane = threadIdx.x & 63;
    const int D = a.D;
    int64_t nh = (int64_t)a.lc->n_hubs;
    if (nh > a.hubs.hub_cap) nh = a.hubs.hub_cap;
    const int64_t waves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    bool live[NV];
#pragma unroll
    for (int q = 0; q < NV; ++q) live[q] = lane * 4 + q * 256 < D;
    for (int64_t h = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6; h < nh; h += waves) {
        const DstRec rec = a.recs[a.hubs.hub_slot[h]];
        const int32_t nch = (rec.deg + NRT_CHUNK - 1) / NRT_CHUNK;
        const int64_t first = (int64_t)a.hubs.hub_first[h];
        const int32_t v = rec.v;
        const bool full = !a.incremental || in_set(a.src_bitmap, v);
        float4 tot[NV];
#pragma unroll
        for (int q = 0; q < NV; ++q) tot[q] = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int32_t c = 0; c < nch; ++c) {
#pragma unroll
            for (int q = 0; q < NV; ++q) {
                if (!live[q]) continue;
                const float4 x = *reinterpret_cast<const float4*>(a.hubs.partial + (first + c) * D + lane * 4 + q * 256);
                tot[q].x += x.x; tot[q].y += x.y; tot[q].z += x.z; tot[q].w += x.w;
            }
        }
        float* out = a.S + (int64_t)v * D;
        bool redo = false;
        if (!full) {
            float big = 0.f, left = 0.f;
#pragma unroll
            for (int q = 0; q < NV; ++q) {
                if (!live[q]) continue;
                const float4 o = *reinterpret_cast<const float4*>(out + lane * 4 + q * 256);
                const float4 d = tot[q];
                tot[q] = make_float4(o.x + d.x, o.y + d.y, o.z + d.z, o.w + d.w);
                big = fmaxf(big, fmaxf(fmaxf(fabsf(d.x), fabsf(d.y)), fmaxf(fabsf(d.z), fabsf(d.w))));
                left = fmaxf(left, fmaxf(fmaxf(fabsf(tot[q].x), fabsf(tot[q].y)), fmaxf(fabsf(tot[q].z), fabsf(tot[q].w))));
            }
#pragma unroll
            for (int sft = 32; sft >= 1; sft >>= 1) {
                big = fmaxf(big, __shfl_xor(big, sft, 64));
                left = fmaxf(left, __shfl_xor(left, sft, 64));
            }
            redo = big > AG_GUARD_RATIO * left;
        }
        if (redo) {
            float4 hv[NV];
#pragma unroll
            for (int q = 0; q < NV; ++q) {
                hv[q] = make_float4(0.f, 0.f, 0.f, 0.f);
                tot[q] = hv[q];
                if (live[q]) hv[q] = *reinterpret_cast<const float4*>((GATE ? a.P2 : a.H) + (int64_t)v * D + lane * 4 + q * 256);
            }
            sum_terms<NV, GATE, false>(a, rec.off, rec.deg, true, hv, GATE ? 1.0f : a.beta * a.R[v], tot, live, lane, lane * 4);
        }
#pragma unroll
        for (int q = 0; q < NV; ++q)
            if (live[q]) *reinterpret_cast<float4*>(out + lane * 4 + q * 256) = tot[q];
    }
}

// one wave per (destination of an updated edge, layer): SD^l[slot] = sum over the destination's updates, in the order of
// the batch plan, of sign * w * cos(h_dst, h_src) * h_src on the old caches (G-GCN: sign * gate * h_src); the wave owns
// the row, so nothing is accumulated with atomics
__global__ void agnn_structural_fold_kernel(AgnnFoldArgs a) {
    const int lane = threadIdx.x & 63;
    const int l = blockIdx.y;
    const int64_t nd = (int64_t)*a.n_slots;
    const int64_t waves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    const int D = a.D[l];
    for (int64_t s = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6; s < nd; s += waves) {
        const int32_t b = a.off[s], e = a.off[s + 1];
        const int32_t v = a.list[s];
        const float* hv = a.H[l] + (int64_t)v * D;
        float* dst = a.SD[l] + s * D;
        for (int k = lane; k < D; k += 64) dst[k] = 0.f;           // the row is this wave's alone
        for (int32_t j = b; j < e; ++j) {
            const int32_t op = a.ord[j];
            const bool is_del = op >= a.n_ins;
            const int32_t u = is_del ? a.del_src[op - a.n_ins] : a.ins_src[op];
            const float* hu = a.H[l] + (int64_t)u * D;
            const float sign = is_del ? -1.0f : 1.0f;
            if (a.gate) {               // G-GCN: sign * sigmoid(W_1 h_src + W_2 h_dst) * h_src, element by element
                const float* p1 = a.P1[l] + (int64_t)u * D;
                const float* p2 = a.P2[l] + (int64_t)v * D;
                for (int k = lane; k < D; k += 64) dst[k] += sign * sigmoidf(p1[k] + p2[k]) * hu[k];
                continue;
            }
            float d = 0.f;
            for (int k = lane; k < D; k += 64) d += hu[k] * hv[k];
            d = wave_sum(d);
            const float c = sign * a.beta[l] * a.R[l][u] * a.R[l][v] * d;
            for (int k = lane; k < D; k += 64) dst[k] += c * hu[k];
        }
    }
}

}  // namespace

nrt_status k_agnn_norms(const int32_t* list, const uint64_t* count_dev, int64_t bound, const float* H, int D, float* R,
                        float* r_old, hipStream_t s) {
    if (bound <= 0) return NRT_OK;
    int64_t g = cdiv(bound, 4);
    if (g > 4096) g = 4096;
    agnn_norms_kernel<<<(int)g, 256, 0, s>>>(list, count_dev, bound, H, D, R, r_old);
    LAUNCH_CHECK();
    return NRT_OK;
}

nrt_status k_agnn_gather(const AgnnArgs& a, hipStream_t s) {
    if (a.D % 4 || a.D > 1024) { nrt_set_error("agnn: row width must be a multiple of 4, at most 1024"); return NRT_ERR_UNSUPPORTED; }
    if (a.gate) {
        if (a.D <= 128) agnn_gather_kernel<1, true, true><<<AG_BLOCKS, AG_WAVES * 64, 0, s>>>(a);
        else if (a.D <= 256) agnn_gather_kernel<1, true, false><<<AG_BLOCKS, AG_WAVES * 64, 0, s>>>(a);
        else if (a.D <= 512) agnn_gather_kernel<2, true, false><<<AG_BLOCKS, AG_WAVES * 64, 0, s>>>(a);
        else agnn_gather_kernel<4, true, false><<<AG_BLOCKS, AG_WAVES * 64, 0, s>>>(a);
    } else {
        if (a.D <= 128) agnn_gather_kernel<1, false, true><<<AG_BLOCKS, AG_WAVES * 64, 0, s>>>(a);
        else if (a.D <= 256) agnn_gather_kernel<1, false, false><<<AG_BLOCKS, AG_WAVES * 64, 0, s>>>(a);
        else if (a.D <= 512) agnn_gather_kernel<2, false, false><<<AG_BLOCKS, AG_WAVES * 64, 0, s>>>(a);
        else agnn_gather_kernel<4, false, false><<<AG_BLOCKS, AG_WAVES * 64, 0, s>>>(a);
    }
    LAUNCH_CHECK();
    return NRT_OK;
}

nrt_status k_agnn_combine(const AgnnArgs& a, hipStream_t s) {
    if (a.gate) {
        if (a.D <= 256) agnn_combine_kernel<1, true><<<1024, AG_WAVES * 64, 0, s>>>(a);
        else if (a.D <= 512) agnn_combine_kernel<2, true><<<1024, AG_WAVES * 64, 0, s>>>(a);
        else agnn_combine_kernel<4, true><<<1024, AG_WAVES * 64, 0, s>>>(a);
    } else {
        if (a.D <= 256) agnn_combine_kernel<1, false><<<1024, AG_WAVES * 64, 0, s>>>(a);
        else if (a.D <= 512) agnn_combine_kernel<2, false><<<1024, AG_WAVES * 64, 0, s>>>(a);
        else agnn_combine_kernel<4, false><<<1024, AG_WAVES * 64, 0, s>>>(a);
    }
    LAUNCH_CHECK();
    return NRT_OK;
}

nrt_status k_agnn_structural_fold(const AgnnFoldArgs& a, hipStream_t s) {
    const int64_t nops = a.n_ins + a.n_del;
    if (nops <= 0 || a.n_layers <= 0) return NRT_OK;
    int64_t g = cdiv(nops, 4);
    if (g > 2048) g = 2048;
    agnn_structural_fold_kernel<<<dim3((unsigned)g, (unsigned)a.n_layers, 1), 256, 0, s>>>(a);
    LAUNCH_CHECK();
    return NRT_OK;
}
