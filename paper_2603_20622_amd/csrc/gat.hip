// GAT on the incremental path (Eq. 3-4; Algorithms 2 and 3).
//
// Cached per layer and vertex: z = x W, the two attention scalars per head as = a_src . z, ad = a_dst . z (they
// replace the per-edge cached attention that Algorithm 3 keeps: an old logit is recomputed from old scalars), a
// running bound m of the largest logit, the attention sum den = sum exp(e - m) (Algorithm 3's at_sum, shifted by
// m so that exp cannot overflow) and the context-free aggregate S = sum exp(e - m) z_u (Algorithm 3's a-hat).
//
// For an affected destination v:
//   * if its own z changed (its layer input changed), every logit of v has changed: v is recomputed over its full
//     new in-neighbourhood plus itself (Algorithm 2; the constrained-model rule of Section III-D, the
//     destination-affected case of Algorithm 4);
//   * otherwise Algorithm 3 touches only what changed:
//       den += sum (at_new - at_old),  S += sum (at_new z_new - at_old z_old)
//     over the in-neighbours whose z changed, plus the edge updates of the batch: a deleted in-edge contributes
//     (-at_old, -at_old z_old), folded on the old caches into a compact row per destination before the graph
//     changes (gat_structural_fold_kernel); an inserted in-edge contributes (+at_new, +at_new z_new) and is found
//     at the end of the in-list, where the graph appends.  m is raised first if a new logit exceeds it (den and S
//     are rescaled by exp(m_old - m_new)).  When the update removes most of the old attention mass (den shrinks
//     below 1/64 of its old value) the subtraction has cancelled the leading digits, and v is recomputed in full.
//   A destination with more than NRT_CHUNK in-edges is cut into items whenever some z changed in the layer: each item
//   holds its share of the full sums (own z changed) or of Algorithm 3's exchange relative to a bound of its own,
//   and the combine kernel merges them; when no z changed (edge updates only) such a destination takes the same
//   O(#updates) path as the others.
// One wave per destination; lane = 4 consecutive columns of the row, a head = head_dim/4 neighbouring lanes.
//
// RGAT (Table II row RGAT; template argument REL): the heads are the relations.  Every edge carries a relation id
// (its weight) and enters only the softmax group of that relation, so a lane skips the entries whose relation is not
// its head's; the self-loop belongs to every group; the layer output is the sum of the groups' results instead of
// their concatenation (width head_dim), formed through a row of LDS per wave.
#include "common.h"

namespace {

__device__ inline float leaky(float x, float slope) { return x > 0.f ? x : slope * x; }

// ------------------------------------------------------------------ attention scalars of the listed rows
__global__ void gat_scalars_kernel(GatArgs a) {
    const int64_t m = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int lane = threadIdx.x & 63;
    const int64_t count = a.rows ? (int64_t)*a.n_rows_dev : a.n;
    if (m >= count) return;
    const int64_t v = a.rows ? (int64_t)a.rows[m] : m;
    const int D = a.heads * a.head_dim;
    for (int k = 0; k < a.heads; ++k) {
        float ps = 0.f, pd = 0.f;
        for (int c = lane; c < a.head_dim; c += 64) {
            const float z = a.Z[v * D + k * a.head_dim + c];
            ps += a.att_src[k * a.head_dim + c] * z;
            pd += a.att_dst[k * a.head_dim + c] * z;
        }
#pragma unroll
        for (int s = 32; s >= 1; s >>= 1) { ps += __shfl_xor(ps, s, 64); pd += __shfl_xor(pd, s, 64); }
        if (lane == 0) {
            if (a.AS_old) a.AS_old[m * a.heads + k] = a.AS[v * a.heads + k];
            a.AS[v * a.heads + k] = ps;
            a.AD[v * a.heads + k] = pd;
        }
    }
}

// ------------------------------------------------------------------ structural terms (Algorithm 3 on edge updates)
// One wave per (destination of an updated edge, layer), before the graph and the caches change: the destination's
// deleted in-edges u->v, in the order of the batch plan, each contribute minus their old attention term relative to
// v's cached bound m, summed in registers into the compact row of v (no atomics: the wave owns the row).  Its
// inserted in-edges are only counted (by the plan): the gather finds them at the end of the in-list.
__global__ void gat_structural_fold_kernel(GatFoldArgs a) {
    const int lane = threadIdx.x & 63;
    const int l = blockIdx.y;
    const int64_t nd = (int64_t)*a.n_slots;
    const int64_t waves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    const int H = a.heads, hd = a.head_dim, D = H * hd;
    for (int64_t s = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6; s < nd; s += waves) {
        const int32_t b = a.off[s], e = a.off[s + 1];
        const int32_t v = a.list[s];
        for (int col = lane * 4; col < D; col += 256) {
            const int k = col / hd;
            const float adv = a.AD[l][(int64_t)v * H + k], mv = a.M[l][(int64_t)v * H + k];
            float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
            float den = 0.f;
            for (int32_t j = b; j < e; ++j) {
                const int32_t op = a.ord[j];
                if (op < a.n_ins) continue;                            // inserts come first in the run
                if (a.del_w && nrt_rel_of(a.del_w[op - a.n_ins], H) != k) continue;   // typed edge: its relation's group only
                const int32_t u = a.del_src[op - a.n_ins];
                const float w = __expf(leaky(adv + a.AS[l][(int64_t)u * H + k], a.slope) - mv);   // at most 1: m bounds every cached logit of v
                const float4 z = *reinterpret_cast<const float4*>(a.Z[l] + (int64_t)u * D + col);
                acc.x -= w * z.x; acc.y -= w * z.y; acc.z -= w * z.z; acc.w -= w * z.w;
                den -= w;
            }
            *reinterpret_cast<float4*>(a.SDS[l] + s * D + col) = acc;
            if (col % hd == 0) a.SDDEN[l][s * H + k] = den;
        }
    }
}

// ------------------------------------------------------------------ gather
// Softmax aggregate over `cnt` in-list entries starting at pool position `base`, optionally with the self-loop
// of v, all with current values (Algorithm 2).  Two passes: largest logit, then the shifted sums.
template <int NV, bool REL>
__device__ inline void gat_full_pass(const GatArgs& a, int32_t v, int64_t base, int32_t cnt, bool with_self, int lane,
                                     const int (&col)[NV], const int (&head)[NV], const bool (&live)[NV],
                                     const float (&adv)[NV], float (&mcur)[NV], float (&den)[NV], float4 (&acc)[NV]) {
    const int H = a.heads, D = a.heads * a.head_dim;
    const float slope = a.slope;
#pragma unroll
    for (int q = 0; q < NV; ++q)
        mcur[q] = (live[q] && with_self) ? leaky(adv[q] + a.AS[(int64_t)v * H + head[q]], slope) : -3.0e38f;
    for (int32_t j0 = 0; j0 < cnt; j0 += 64) {
        const int32_t jj = j0 + lane;
        const int32_t u = jj < cnt ? a.in.idx[base + jj] : -1;
        const int32_t rl = (REL && jj < cnt) ? nrt_rel_of(a.in.wts[base + jj], H) : -1;
        unsigned long long mask = __ballot(u >= 0);
        while (mask) {
            const int bit = __ffsll((long long)mask) - 1;
            mask &= mask - 1;
            const int32_t uu = __builtin_amdgcn_readlane(u, bit);
            const int32_t rr = REL ? __builtin_amdgcn_readlane(rl, bit) : -1;
#pragma unroll
            for (int q = 0; q < NV; ++q)
                if (live[q] && (!REL || head[q] == rr)) mcur[q] = fmaxf(mcur[q], leaky(adv[q] + a.AS[(int64_t)uu * H + head[q]], slope));
        }
    }
#pragma unroll
    for (int q = 0; q < NV; ++q) {
        den[q] = 0.f;
        acc[q] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (live[q] && with_self) {
            const float c = __expf(leaky(adv[q] + a.AS[(int64_t)v * H + head[q]], slope) - mcur[q]);
            const float4 z = *reinterpret_cast<const float4*>(a.Z + (int64_t)v * D + col[q]);
            den[q] = c;
            acc[q] = make_float4(c * z.x, c * z.y, c * z.z, c * z.w);
        }
    }
    for (int32_t j0 = 0; j0 < cnt; j0 += 64) {
        const int32_t jj = j0 + lane;
        const int32_t u = jj < cnt ? a.in.idx[base + jj] : -1;
        const int32_t rl = (REL && jj < cnt) ? nrt_rel_of(a.in.wts[base + jj], H) : -1;
        unsigned long long mask = __ballot(u >= 0);
        while (mask) {
            const int b0 = __ffsll((long long)mask) - 1;
            mask &= mask - 1;
            const int32_t u0 = __builtin_amdgcn_readlane(u, b0);
            const int32_t r0 = REL ? __builtin_amdgcn_readlane(rl, b0) : -1;
            int32_t u1 = -1, r1 = -1;
            if (mask) {
                const int b1 = __ffsll((long long)mask) - 1;
                mask &= mask - 1;
                u1 = __builtin_amdgcn_readlane(u, b1);
                if (REL) r1 = __builtin_amdgcn_readlane(rl, b1);
            }
#pragma unroll
            for (int q = 0; q < NV; ++q) {
                if (!live[q]) continue;
                float c0 = 0.f, c1 = 0.f;
                float4 z0 = make_float4(0.f, 0.f, 0.f, 0.f), z1 = z0;
                if (!REL || head[q] == r0) {
                    c0 = __expf(leaky(adv[q] + a.AS[(int64_t)u0 * H + head[q]], slope) - mcur[q]);
                    z0 = *reinterpret_cast<const float4*>(a.Z + (int64_t)u0 * D + col[q]);
                }
                if (u1 >= 0 && (!REL || head[q] == r1)) {
                    c1 = __expf(leaky(adv[q] + a.AS[(int64_t)u1 * H + head[q]], slope) - mcur[q]);
                    z1 = *reinterpret_cast<const float4*>(a.Z + (int64_t)u1 * D + col[q]);
                }
                den[q] += c0 + c1;
                acc[q].x += c0 * z0.x + c1 * z1.x; acc[q].y += c0 * z0.y + c1 * z1.y;
                acc[q].z += c0 * z0.z + c1 * z1.z; acc[q].w += c0 * z0.w + c1 * z1.w;
            }
        }
    }
}

// store context, aggregate and layer output h = act(S / den + b) of vertex v (list position s).  REL: the output is the
// sum over the heads (relations) of S / den, formed in `red`, a row of heads * head_dim floats of LDS owned by the wave.
template <int NV, bool REL>
__device__ inline void gat_store(const GatArgs& a, int32_t v, int64_t s, const int (&col)[NV], const int (&head)[NV],
                                 const bool (&live)[NV], const float (&mcur)[NV], const float (&den)[NV],
                                 const float4 (&acc)[NV], float* red, int lane) {
    const int H = a.heads, hd = a.head_dim, D = H * hd;
    if (REL) {
#pragma unroll
        for (int q = 0; q < NV; ++q) {
            if (!live[q]) continue;
            if ((col[q] % hd) == 0) {
                a.M[(int64_t)v * H + head[q]] = mcur[q];
                a.DEN[(int64_t)v * H + head[q]] = den[q];
            }
            *reinterpret_cast<float4*>(a.S + (int64_t)v * D + col[q]) = acc[q];
            const float inv = 1.0f / den[q];             // every group holds the self-loop: den > 0
            *reinterpret_cast<float4*>(red + col[q]) = make_float4(acc[q].x * inv, acc[q].y * inv, acc[q].z * inv, acc[q].w * inv);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        for (int c = lane * 4; c < hd; c += 256) {
            float4 y = make_float4(0.f, 0.f, 0.f, 0.f);
            for (int r = 0; r < H; ++r) {
                const float4 t = *reinterpret_cast<const float4*>(red + r * hd + c);
                y.x += t.x; y.y += t.y; y.z += t.z; y.w += t.w;
            }
            float yy[4] = {y.x, y.y, y.z, y.w};
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                if (a.bias) yy[t] += a.bias[c + t];
                if (a.act == 2) yy[t] = yy[t] > 0.f ? yy[t] : expm1f(yy[t]);
            }
            const float4 yo = make_float4(yy[0], yy[1], yy[2], yy[3]);
            if (a.Hout) *reinterpret_cast<float4*>(a.Hout + (int64_t)v * hd + c) = yo;
            if (a.out_rows && s < a.out_cap) *reinterpret_cast<float4*>(a.out_rows + s * hd + c) = yo;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();                 // the row is free for the wave's next destination
        return;
    }
#pragma unroll
    for (int q = 0; q < NV; ++q) {
        if (!live[q]) continue;
        if ((col[q] % hd) == 0) {
            a.M[(int64_t)v * H + head[q]] = mcur[q];
            a.DEN[(int64_t)v * H + head[q]] = den[q];
        }
        *reinterpret_cast<float4*>(a.S + (int64_t)v * D + col[q]) = acc[q];
        const float inv = 1.0f / den[q];
        float y[4] = {acc[q].x * inv, acc[q].y * inv, acc[q].z * inv, acc[q].w * inv};
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            if (a.bias) y[t] += a.bias[col[q] + t];
            if (a.act == 2) y[t] = y[t] > 0.f ? y[t] : expm1f(y[t]);
        }
        const float4 yo = make_float4(y[0], y[1], y[2], y[3]);
        if (a.Hout) *reinterpret_cast<float4*>(a.Hout + (int64_t)v * D + col[q]) = yo;
        if (a.out_rows && s < a.out_cap) *reinterpret_cast<float4*>(a.out_rows + s * D + col[q]) = yo;
    }
}

// Units [0, n_items): hub items (NRT_CHUNK in-list entries of a destination with a long in-list; they write partial
// (bound, sum, row) triples of the full sums or of the exchange).  Units
// [n_items, n_items + n_dst): the destinations themselves, hubs skipped.
template <int NV, bool REL>
__global__ void __launch_bounds__(256) gat_gather_kernel(GatArgs a) {
    __shared__ __attribute__((aligned(16))) float s_red[REL ? 4 * NV * 256 : 4];
    float* red = &s_red[REL ? (threadIdx.x >> 6) * NV * 256 : 0];
    const int lane = threadIdx.x & 63;
    const int64_t waves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    const int64_t n_dst = (int64_t)a.lc->count;
    int64_t n_items = (int64_t)a.lc->n_items;
    if (n_items > a.hubs.item_cap) n_items = a.hubs.item_cap;
    const int H = a.heads, hd = a.head_dim, D = H * hd;
    const float slope = a.slope;
    int col[NV], head[NV];
    bool live[NV];
#pragma unroll
    for (int q = 0; q < NV; ++q) {
        col[q] = lane * 4 + q * 256;
        live[q] = col[q] < D;
        head[q] = live[q] ? col[q] / hd : 0;
    }
    const bool any_src = !(a.src_bitmap && a.n_src_dev && *a.n_src_dev == 0);   // false: only edge updates in this layer
    long long rows_read = 0;
    for (int64_t unit = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6; unit < n_items + n_dst; unit += waves) {
        float adv[NV], mcur[NV], den[NV];
        float4 acc[NV];
        if (unit < n_items) {
            const int32_t chunk = a.hubs.item_chunk[unit];
            const DstRec rec = a.recs[a.hubs.hub_slot[a.hubs.item_hub[unit]]];
            const int32_t v = rec.v;
            const int32_t cnt = min(NRT_CHUNK, rec.deg - chunk * NRT_CHUNK);
            const int64_t base = rec.off + (int64_t)chunk * NRT_CHUNK;
#pragma unroll
            for (int q = 0; q < NV; ++q) adv[q] = live[q] ? a.AD[(int64_t)v * H + head[q]] : 0.f;
            const bool own = a.src_bitmap ? ((a.src_bitmap[v >> 5] >> (v & 31)) & 1u) != 0 : true;
            if (own) {                                        // every logit of v changed: its share of the full sums
                gat_full_pass<NV, REL>(a, v, base, cnt, false, lane, col, head, live, adv, mcur, den, acc);
                rows_read += cnt;
            } else {
                // Algorithm 3 on this part of the in-list, relative to a bound of its own (the cached bound of v raised
                // by the new logits met here); the combine kernel brings the parts to one bound
                const bool edge = (a.ddst_bitmap[v >> 5] >> (v & 31)) & 1u;
                const int32_t n_new = edge ? a.ins_cnt[a.dd_slot[v]] : 0;
                const int32_t first_new = rec.deg - n_new - chunk * NRT_CHUNK;   // entries from here on were inserted
#pragma unroll
                for (int q = 0; q < NV; ++q) mcur[q] = live[q] ? a.M[(int64_t)v * H + head[q]] : 0.f;
                for (int32_t j0 = 0; j0 < cnt; j0 += 64) {
                    const int32_t jj = j0 + lane;
                    const int32_t u = jj < cnt ? a.in.idx[base + jj] : -1;
                    const int32_t rl = (REL && jj < cnt) ? nrt_rel_of(a.in.wts[base + jj], H) : -1;
                    const bool ok = u >= 0 && (jj >= first_new || ((a.src_bitmap[(uint32_t)u >> 5] >> (u & 31)) & 1u));
                    unsigned long long mask = __ballot(ok);
                    while (mask) {
                        const int bit = __ffsll((long long)mask) - 1;
                        mask &= mask - 1;
                        const int32_t uu = __builtin_amdgcn_readlane(u, bit);
                        const int32_t rr = REL ? __builtin_amdgcn_readlane(rl, bit) : -1;
#pragma unroll
                        for (int q = 0; q < NV; ++q)
                            if (live[q] && (!REL || head[q] == rr)) mcur[q] = fmaxf(mcur[q], leaky(adv[q] + a.AS[(int64_t)uu * H + head[q]], slope));
                    }
                }
#pragma unroll
                for (int q = 0; q < NV; ++q) { den[q] = 0.f; acc[q] = make_float4(0.f, 0.f, 0.f, 0.f); }
                for (int32_t j0 = 0; j0 < cnt; j0 += 64) {
                    const int32_t jj = j0 + lane;
                    const int32_t u = jj < cnt ? a.in.idx[base + jj] : -1;
                    const int32_t rl = (REL && jj < cnt) ? nrt_rel_of(a.in.wts[base + jj], H) : -1;
                    const bool fresh = jj >= first_new;
                    const bool ok = u >= 0 && (fresh || ((a.src_bitmap[(uint32_t)u >> 5] >> (u & 31)) & 1u));
                    const int32_t sl = (ok && !fresh) ? a.src_slot[u] : -1;
                    unsigned long long mask = __ballot(ok);
                    while (mask) {
                        const int bit = __ffsll((long long)mask) - 1;
                        mask &= mask - 1;
                        const int32_t uu = __builtin_amdgcn_readlane(u, bit);
                        const int32_t ss = __builtin_amdgcn_readlane(sl, bit);     // -1: an inserted in-edge, new term only
                        const int32_t rr = REL ? __builtin_amdgcn_readlane(rl, bit) : -1;
                        rows_read += ss >= 0 ? 2 : 1;
#pragma unroll
                        for (int q = 0; q < NV; ++q) {
                            if (!live[q] || (REL && head[q] != rr)) continue;
                            const float cn = __expf(leaky(adv[q] + a.AS[(int64_t)uu * H + head[q]], slope) - mcur[q]);
                            const float4 zn = *reinterpret_cast<const float4*>(a.Z + (int64_t)uu * D + col[q]);
                            den[q] += cn;
                            acc[q].x += cn * zn.x; acc[q].y += cn * zn.y; acc[q].z += cn * zn.z; acc[q].w += cn * zn.w;
                            if (ss >= 0) {
                                const float co = __expf(leaky(adv[q] + a.AS_old[(int64_t)ss * H + head[q]], slope) - mcur[q]);
                                const float4 zo = *reinterpret_cast<const float4*>(a.Z_old + (int64_t)ss * D + col[q]);
                                den[q] -= co;
                                acc[q].x -= co * zo.x; acc[q].y -= co * zo.y; acc[q].z -= co * zo.z; acc[q].w -= co * zo.w;
                            }
                        }
                    }
                }
            }
#pragma unroll
            for (int q = 0; q < NV; ++q) {
                if (!live[q]) continue;
                if ((col[q] % hd) == 0) {
                    a.part_m[unit * H + head[q]] = mcur[q];
                    a.part_den[unit * H + head[q]] = den[q];
                }
                *reinterpret_cast<float4*>(a.hubs.partial + unit * D + col[q]) = acc[q];
            }
            continue;
        }
        const int64_t s = unit - n_items;
        const DstRec rec = a.recs[s];
        if (rec.deg > NRT_CHUNK && any_src) continue;         // served through its items
        const int32_t v = rec.v;
        const int64_t off = rec.off;
        const int32_t deg = rec.deg;
        bool full = true;
        int32_t n_new = 0;          // inserted in-edges of v: the last n_new entries of its in-list
        int64_t sd_row = -1;        // row of v's structural terms
        if (a.src_bitmap) {
            const bool own = (a.src_bitmap[v >> 5] >> (v & 31)) & 1u;
            const bool edge = (a.ddst_bitmap[v >> 5] >> (v & 31)) & 1u;
            full = own;
            if (edge && !own) { sd_row = a.dd_slot[v]; n_new = a.ins_cnt[sd_row]; }
        }
#pragma unroll
        for (int q = 0; q < NV; ++q) adv[q] = live[q] ? a.AD[(int64_t)v * H + head[q]] : 0.f;

        if (!full) {
            // ---- Algorithm 3: the in-neighbours whose z changed (entries before the inserted ones, skipped when no z
            // changed in this layer) and the inserted entries
            const int32_t n_kept = deg - n_new;
            const int32_t scan_end = any_src ? n_kept : 0;
            float mold[NV];
#pragma unroll
            for (int q = 0; q < NV; ++q) { mold[q] = live[q] ? a.M[(int64_t)v * H + head[q]] : 0.f; mcur[q] = mold[q]; }
            // pass 1: raise the bound to the largest new logit
            for (int32_t j0 = n_kept; j0 < deg; j0 += 64) {
                const int32_t jj = j0 + lane;
                const int32_t u = jj < deg ? a.in.idx[off + jj] : -1;
                const int32_t rl = (REL && jj < deg) ? nrt_rel_of(a.in.wts[off + jj], H) : -1;
                unsigned long long mask = __ballot(u >= 0);
                while (mask) {
                    const int bit = __ffsll((long long)mask) - 1;
                    mask &= mask - 1;
                    const int32_t uu = __builtin_amdgcn_readlane(u, bit);
                    const int32_t rr = REL ? __builtin_amdgcn_readlane(rl, bit) : -1;
#pragma unroll
                    for (int q = 0; q < NV; ++q)
                        if (live[q] && (!REL || head[q] == rr)) mcur[q] = fmaxf(mcur[q], leaky(adv[q] + a.AS[(int64_t)uu * H + head[q]], slope));
                }
            }
            for (int32_t j0 = 0; j0 < scan_end; j0 += 64) {
                const int32_t jj = j0 + lane;
                int32_t u = jj < scan_end ? a.in.idx[off + jj] : -1;
                bool ok = u >= 0 && ((a.src_bitmap[(uint32_t)u >> 5] >> (u & 31)) & 1u);
                const int32_t rl = (REL && ok) ? nrt_rel_of(a.in.wts[off + jj], H) : -1;
                unsigned long long mask = __ballot(ok);
                while (mask) {
                    const int bit = __ffsll((long long)mask) - 1;
                    mask &= mask - 1;
                    const int32_t uu = __builtin_amdgcn_readlane(u, bit);
                    const int32_t rr = REL ? __builtin_amdgcn_readlane(rl, bit) : -1;
#pragma unroll
                    for (int q = 0; q < NV; ++q)
                        if (live[q] && (!REL || head[q] == rr)) mcur[q] = fmaxf(mcur[q], leaky(adv[q] + a.AS[(int64_t)uu * H + head[q]], slope));
                }
            }
            bool redo = false;
            float den0[NV];
#pragma unroll
            for (int q = 0; q < NV; ++q) {
                const float f = __expf(mold[q] - mcur[q]);
                den[q] = live[q] ? a.DEN[(int64_t)v * H + head[q]] * f : 1.f;
                den0[q] = den[q];
                acc[q] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (live[q]) {
                    const float4 so = *reinterpret_cast<const float4*>(a.S + (int64_t)v * D + col[q]);
                    acc[q] = make_float4(so.x * f, so.y * f, so.z * f, so.w * f);
                    if (sd_row >= 0) {                            // deleted in-edges: terms relative to mold
                        const float4 sd = *reinterpret_cast<const float4*>(a.sd_s + sd_row * D + col[q]);
                        den[q] += a.sd_den[sd_row * H + head[q]] * f;
                        acc[q].x += sd.x * f; acc[q].y += sd.y * f; acc[q].z += sd.z * f; acc[q].w += sd.w * f;
                    }
                }
            }
            // pass 2: the inserted in-edges bring new terms ...
            for (int32_t j0 = n_kept; j0 < deg; j0 += 64) {
                const int32_t jj = j0 + lane;
                const int32_t u = jj < deg ? a.in.idx[off + jj] : -1;
                const int32_t rl = (REL && jj < deg) ? nrt_rel_of(a.in.wts[off + jj], H) : -1;
                unsigned long long mask = __ballot(u >= 0);
                rows_read += __popcll(mask);
                while (mask) {
                    const int bit = __ffsll((long long)mask) - 1;
                    mask &= mask - 1;
                    const int32_t uu = __builtin_amdgcn_readlane(u, bit);
                    const int32_t rr = REL ? __builtin_amdgcn_readlane(rl, bit) : -1;
#pragma unroll
                    for (int q = 0; q < NV; ++q) {
                        if (!live[q] || (REL && head[q] != rr)) continue;
                        const float cn = __expf(leaky(adv[q] + a.AS[(int64_t)uu * H + head[q]], slope) - mcur[q]);
                        const float4 zn = *reinterpret_cast<const float4*>(a.Z + (int64_t)uu * D + col[q]);
                        den[q] += cn;
                        acc[q].x += cn * zn.x; acc[q].y += cn * zn.y; acc[q].z += cn * zn.z; acc[q].w += cn * zn.w;
                    }
                }
            }
            // ... and the kept in-edges whose source changed exchange their old term for the new one
            for (int32_t j0 = 0; j0 < scan_end; j0 += 64) {
                const int32_t jj = j0 + lane;
                int32_t u = jj < scan_end ? a.in.idx[off + jj] : -1;
                bool ok = u >= 0 && ((a.src_bitmap[(uint32_t)u >> 5] >> (u & 31)) & 1u);
                int32_t sl = ok ? a.src_slot[u] : -1;
                const int32_t rl = (REL && ok) ? nrt_rel_of(a.in.wts[off + jj], H) : -1;
                unsigned long long mask = __ballot(ok);
                rows_read += 2 * __popcll(mask);
                while (mask) {
                    const int bit = __ffsll((long long)mask) - 1;
                    mask &= mask - 1;
                    const int32_t uu = __builtin_amdgcn_readlane(u, bit);
                    const int32_t ss = __builtin_amdgcn_readlane(sl, bit);
                    const int32_t rr = REL ? __builtin_amdgcn_readlane(rl, bit) : -1;
#pragma unroll
                    for (int q = 0; q < NV; ++q) {
                        if (!live[q] || (REL && head[q] != rr)) continue;
                        const float en = leaky(adv[q] + a.AS[(int64_t)uu * H + head[q]], slope);
                        const float eo = leaky(adv[q] + a.AS_old[(int64_t)ss * H + head[q]], slope);
                        const float cn = __expf(en - mcur[q]), co = __expf(eo - mcur[q]);
                        const float4 zn = *reinterpret_cast<const float4*>(a.Z + (int64_t)uu * D + col[q]);
                        const float4 zo = *reinterpret_cast<const float4*>(a.Z_old + (int64_t)ss * D + col[q]);
                        den[q] += cn - co;
                        acc[q].x += cn * zn.x - co * zo.x; acc[q].y += cn * zn.y - co * zo.y;
                        acc[q].z += cn * zn.z - co * zo.z; acc[q].w += cn * zn.w - co * zo.w;
                    }
                }
            }
#pragma unroll
            for (int q = 0; q < NV; ++q)
                if (live[q] && !(den[q] > den0[q] * (1.0f / 64.0f))) redo = true;
            full = __ballot(redo) != 0ULL;        // cancellation: recompute this destination over all its neighbours
        }
        if (full) {
            gat_full_pass<NV, REL>(a, v, off, deg, true, lane, col, head, live, adv, mcur, den, acc);
            rows_read += deg + 1;
        }
        gat_store<NV, REL>(a, v, s, col, head, live, mcur, den, acc, red, lane);
    }
    if (a.pair_ctr && lane == 0 && rows_read) atomicAdd(&a.pair_ctr[blockIdx.x & 1023], (unsigned long long)rows_read);
}

// one wave per hub: merge the partial triples of its items and its self-loop
template <int NV, bool REL>
__global__ void __launch_bounds__(256) gat_combine_kernel(GatArgs a) {
    __shared__ __attribute__((aligned(16))) float s_red[REL ? 4 * NV * 256 : 4];
    float* red = &s_red[REL ? (threadIdx.x >> 6) * NV * 256 : 0];
    const int lane = threadIdx.x & 63;
    const int64_t waves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    int64_t nh = (int64_t)a.lc->n_hubs;
    if (nh > a.hubs.hub_cap) nh = a.hubs.hub_cap;
    const int H = a.heads, hd = a.head_dim, D = H * hd;
    int col[NV], head[NV];
    bool live[NV];
#pragma unroll
    for (int q = 0; q < NV; ++q) {
        col[q] = lane * 4 + q * 256;
        live[q] = col[q] < D;
        head[q] = live[q] ? col[q] / hd : 0;
    }
    for (int64_t h = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6; h < nh; h += waves) {
        const int64_t s = a.hubs.hub_slot[h];
        const DstRec rec = a.recs[s];
        const int32_t nch = (rec.deg + NRT_CHUNK - 1) / NRT_CHUNK;
        const int64_t first = (int64_t)a.hubs.hub_first[h];
        float mcur[NV], den[NV], eself[NV];
        float4 acc[NV];
        const int32_t v = rec.v;
        const bool own = a.src_bitmap ? ((a.src_bitmap[v >> 5] >> (v & 31)) & 1u) != 0 : true;
        if (!own) {
            // the items hold Algorithm 3's exchanged terms, each relative to its own bound: bring the cached sums, the
            // structural terms and the items to the largest bound and add them up
            float mold[NV], den0[NV];
#pragma unroll
            for (int q = 0; q < NV; ++q) { mold[q] = live[q] ? a.M[(int64_t)v * H + head[q]] : 0.f; mcur[q] = mold[q]; }
            for (int32_t c = 0; c < nch; ++c)
#pragma unroll
                for (int q = 0; q < NV; ++q)
                    if (live[q]) mcur[q] = fmaxf(mcur[q], a.part_m[(first + c) * H + head[q]]);
            const bool edge = (a.ddst_bitmap[v >> 5] >> (v & 31)) & 1u;
            const int64_t sd_row = edge ? (int64_t)a.dd_slot[v] : -1;
#pragma unroll
            for (int q = 0; q < NV; ++q) {
                const float f = __expf(mold[q] - mcur[q]);
                den[q] = live[q] ? a.DEN[(int64_t)v * H + head[q]] * f : 1.f;
                den0[q] = den[q];
                acc[q] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (live[q]) {
                    const float4 so = *reinterpret_cast<const float4*>(a.S + (int64_t)v * D + col[q]);
                    acc[q] = make_float4(so.x * f, so.y * f, so.z * f, so.w * f);
                    if (sd_row >= 0) {
                        const float4 sd = *reinterpret_cast<const float4*>(a.sd_s + sd_row * D + col[q]);
                        den[q] += a.sd_den[sd_row * H + head[q]] * f;
                        acc[q].x += sd.x * f; acc[q].y += sd.y * f; acc[q].z += sd.z * f; acc[q].w += sd.w * f;
                    }
                }
            }
            for (int32_t c = 0; c < nch; ++c) {
#pragma unroll
                for (int q = 0; q < NV; ++q) {
                    if (!live[q]) continue;
                    const float f = __expf(a.part_m[(first + c) * H + head[q]] - mcur[q]);
                    const float4 p = *reinterpret_cast<const float4*>(a.hubs.partial + (first + c) * D + col[q]);
                    den[q] += f * a.part_den[(first + c) * H + head[q]];
                    acc[q].x += f * p.x; acc[q].y += f * p.y; acc[q].z += f * p.z; acc[q].w += f * p.w;
                }
            }
            bool redo = false;
#pragma unroll
            for (int q = 0; q < NV; ++q)
                if (live[q] && !(den[q] > den0[q] * (1.0f / 64.0f))) redo = true;
            if (__ballot(redo) != 0ULL) {     // cancellation: this wave recomputes the destination over all its neighbours
                float adv[NV];
#pragma unroll
                for (int q = 0; q < NV; ++q) adv[q] = live[q] ? a.AD[(int64_t)v * H + head[q]] : 0.f;
                gat_full_pass<NV, REL>(a, v, rec.off, rec.deg, true, lane, col, head, live, adv, mcur, den, acc);
            }
            gat_store<NV, REL>(a, v, s, col, head, live, mcur, den, acc, red, lane);
            continue;
        }
#pragma unroll
        for (int q = 0; q < NV; ++q) {
            eself[q] = live[q] ? leaky(a.AD[(int64_t)rec.v * H + head[q]] + a.AS[(int64_t)rec.v * H + head[q]], a.slope) : 0.f;
            mcur[q] = eself[q];
        }
        for (int32_t c = 0; c < nch; ++c)
#pragma unroll
            for (int q = 0; q < NV; ++q)
                if (live[q]) mcur[q] = fmaxf(mcur[q], a.part_m[(first + c) * H + head[q]]);
#pragma unroll
        for (int q = 0; q < NV; ++q) {
            den[q] = 0.f;
            acc[q] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (live[q]) {
                const float cs = __expf(eself[q] - mcur[q]);
                const float4 z = *reinterpret_cast<const float4*>(a.Z + (int64_t)rec.v * D + col[q]);
                den[q] = cs;
                acc[q] = make_float4(cs * z.x, cs * z.y, cs * z.z, cs * z.w);
            }
        }
        for (int32_t c = 0; c < nch; ++c) {
#pragma unroll
            for (int q = 0; q < NV; ++q) {
                if (!live[q]) continue;
                const float f = __expf(a.part_m[(first + c) * H + head[q]] - mcur[q]);
                const float4 p = *reinterpret_cast<const float4*>(a.hubs.partial + (first + c) * D + col[q]);
                den[q] += f * a.part_den[(first + c) * H + head[q]];
                acc[q].x += f * p.x; acc[q].y += f * p.y; acc[q].z += f * p.z; acc[q].w += f * p.w;
            }
        }
        gat_store<NV, REL>(a, rec.v, s, col, head, live, mcur, den, acc, red, lane);
    }
}

}  // namespace

nrt_status k_gat_scalars(const GatArgs& a, hipStream_t s) {
    const int64_t bound = a.rows ? a.rows_bound : a.n;
    if (bound <= 0) return NRT_OK;
    gat_scalars_kernel<<<(unsigned)cdiv(bound * 64, 256), 256, 0, s>>>(a);
    LAUNCH_CHECK();
    return NRT_OK;
}

nrt_status k_gat_structural_fold(const GatFoldArgs& a, hipStream_t s) {
    const int64_t nops = a.n_ins + a.n_del;
    if (nops <= 0 || a.n_layers <= 0) return NRT_OK;
    int64_t g = cdiv(nops, 4);
    if (g > 2048) g = 2048;
    gat_structural_fold_kernel<<<dim3((unsigned)g, (unsigned)a.n_layers, 1), 256, 0, s>>>(a);
    LAUNCH_CHECK();
    return NRT_OK;
}

nrt_status k_gat_gather(const GatArgs& a, hipStream_t s) {
    const int D = a.heads * a.head_dim;
    const int g = 8192;                     // fixed grid: sizes are read on the device
    if (a.rel) {
        if (!a.in.wts) { nrt_set_error("typed edges need a weighted graph"); return NRT_ERR_INVALID_ARG; }
        if (D <= 256) { gat_gather_kernel<1, true><<<g, 256, 0, s>>>(a); LAUNCH_CHECK(); gat_combine_kernel<1, true><<<2048, 256, 0, s>>>(a); }
        else if (D <= 512) { gat_gather_kernel<2, true><<<g, 256, 0, s>>>(a); LAUNCH_CHECK(); gat_combine_kernel<2, true><<<2048, 256, 0, s>>>(a); }
        else { gat_gather_kernel<4, true><<<g, 256, 0, s>>>(a); LAUNCH_CHECK(); gat_combine_kernel<4, true><<<2048, 256, 0, s>>>(a); }
        LAUNCH_CHECK();
        return NRT_OK;
    }
    if (D <= 256) { gat_gather_kernel<1, false><<<g, 256, 0, s>>>(a); LAUNCH_CHECK(); gat_combine_kernel<1, false><<<2048, 256, 0, s>>>(a); }
    else if (D <= 512) { gat_gather_kernel<2, false><<<g, 256, 0, s>>>(a); LAUNCH_CHECK(); gat_combine_kernel<2, false><<<2048, 256, 0, s>>>(a); }
    else { gat_gather_kernel<4, false><<<g, 256, 0, s>>>(a); LAUNCH_CHECK(); gat_combine_kernel<4, false><<<2048, 256, 0, s>>>(a); }
    LAUNCH_CHECK();
    return NRT_OK;
}
