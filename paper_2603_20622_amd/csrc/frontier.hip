// Affected-set expansion, one hop of Algorithm 4: the destinations of the out-edges of the previous
// hop's affected vertices join the affected set of this hop.
//
// The set under construction is one byte per vertex.  Setting a byte is an idempotent plain store, so the hop
// needs no atomics at all (a bitmap would need an atomic OR per new member; on this part device-scope atomics
// are far slower than stores).  The compaction that follows packs the bytes into a bitmap, ORs in the
// destinations of the updated edges and the previous set, and produces the sorted id list.
//
// The number of sources is only known on the device: the kernels stride over the source list with a fixed
// grid.  One wave walks an out-list of up to HUB_DEG entries; longer lists are queued (one atomic per workgroup)
// and then walked by many workgroups at once, so one celebrity vertex does not serialise the hop.
//
// When the previous hop already holds a large part of the graph, pushing along all its out-edges visits nearly
// every edge to find few new members.  The hop is then run in the pull direction: every vertex outside the
// source set looks for one in-neighbour inside it and stops at the first hit (a vertex that will join finds one
// within a few entries; the others mostly have short in-lists).  The caller allows this direction when the
// previous batch had a large source set at this hop; the device counter of the current batch decides, and the
// push kernels and the pull kernels read the same test, so exactly one direction does the work.
#include "common.h"

namespace {

constexpr int HUB_DEG = 512;
constexpr int HUB_GY = 16;      // workgroups that share one long out-list
constexpr int PULL_OWN = 32;    // in-list entries a lane checks by itself before the vertex is handed to a whole wave

__device__ inline bool hop_pulls(const PullArgs& p, const uint64_t* ns_dev) {
    return p.allowed && (int64_t)(*ns_dev) * 8 > p.n;
}

__global__ void __launch_bounds__(256) expand_kernel(Adj out, const int32_t* src_list, const uint64_t* ns_dev,
                                                     uint8_t* flags, unsigned long long* xhub_count,
                                                     int32_t* xhub_list, int64_t xhub_cap, PullArgs pull) {
    __shared__ int s_n;
    __shared__ unsigned long long s_base;
    __shared__ int32_t s_q[4];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    if (hop_pulls(pull, ns_dev)) return;        // the pull kernels serve this hop; nothing is queued for the hub kernel
    const int64_t ns = (int64_t)*ns_dev;
    const int64_t waves = (int64_t)gridDim.x * 4;
    for (int64_t s0 = (int64_t)blockIdx.x * 4; s0 < ns; s0 += waves) {     // workgroup-uniform trip count
        const int64_t s = s0 + w;
        int32_t hub = -1;
        if (s < ns) {
            const int32_t u = src_list[s];
            const int32_t d = out.deg[u];
            if (d > HUB_DEG) {
                hub = u;
            } else {
                const int64_t o = out.off[u];
                for (int32_t j = lane; j < d; j += 64) flags[out.idx[o + j]] = 1;
            }
        }
        // queue the long lists of this round with one atomic per workgroup
        if (threadIdx.x == 0) s_n = 0;
        __syncthreads();
        if (lane == 0 && hub >= 0) { const int my = atomicAdd(&s_n, 1); s_q[my] = hub; }
        __syncthreads();
        if (threadIdx.x == 0 && s_n > 0) s_base = atomicAdd(xhub_count, (unsigned long long)s_n);
        __syncthreads();
        if ((int)threadIdx.x < s_n && (int64_t)(s_base + threadIdx.x) < xhub_cap) xhub_list[s_base + threadIdx.x] = s_q[threadIdx.x];
        __syncthreads();
    }
}

__global__ void __launch_bounds__(256) expand_hubs_kernel(Adj out, uint8_t* flags, const unsigned long long* xhub_count,
                                                          const int32_t* xhub_list, int64_t xhub_cap) {
    int64_t nh = (int64_t)*xhub_count;
    if (nh > xhub_cap) nh = xhub_cap;
    for (int64_t h = blockIdx.x; h < nh; h += gridDim.x) {
        const int32_t u = xhub_list[h];
        const int32_t d = out.deg[u];
        const int64_t o = out.off[u];
        const int32_t stride = gridDim.y * blockDim.x;
        int32_t j = blockIdx.y * blockDim.x + threadIdx.x;
        for (; j + 3 * stride < d; j += 4 * stride) {
            const int32_t v0 = out.idx[o + j], v1 = out.idx[o + j + stride], v2 = out.idx[o + j + 2 * stride],
                          v3 = out.idx[o + j + 3 * stride];
            flags[v0] = 1; flags[v1] = 1; flags[v2] = 1; flags[v3] = 1;
        }
        for (; j < d; j += stride) flags[out.idx[o + j]] = 1;
    }
}

// Pull direction, first pass: one lane per vertex outside the source set checks up to PULL_OWN in-list entries;
// vertices with longer lists and no hit so far are queued (one atomic per wave) for the second pass.
__global__ void __launch_bounds__(256) expand_pull_kernel(Adj in, const uint64_t* ns_dev, uint8_t* flags, PullArgs p) {
    if (!hop_pulls(p, ns_dev)) return;
    const int lane = threadIdx.x & 63;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t n_round = (p.n + 63) & ~int64_t(63);               // whole waves stay together for the ballot
    for (int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; v < n_round; v += stride) {
        bool queue = false;
        if (v < p.n && !((p.src_bitmap[v >> 5] >> (v & 31)) & 1u)) {
            const int32_t d = in.deg[v];
            if (d > 0) {
                const int64_t o = in.off[v];
                const int32_t own = d < PULL_OWN ? d : PULL_OWN;
                bool hit = false;
                for (int32_t j = 0; j < own && !hit; ++j) {
                    const int32_t u = in.idx[o + j];
                    hit = (p.src_bitmap[(uint32_t)u >> 5] >> (u & 31)) & 1u;
                }
                if (hit) flags[v] = 1;
                else queue = d > PULL_OWN;
            }
        }
        const unsigned long long m = __ballot(queue);
        if (m) {
            unsigned long long base = 0;
            if (lane == 0) base = atomicAdd(p.long_count, (unsigned long long)__popcll(m));
            base = __shfl((long long)base, 0, 64);
            if (queue) {
                const int64_t at = (int64_t)base + __popcll(m & ((1ULL << lane) - 1ULL));
                if (at < p.long_cap) p.long_list[at] = (int32_t)v;
            }
        }
    }
}

// Pull direction, second pass: one wave per queued vertex, 64 entries per trip, stops at the first hit.
__global__ void __launch_bounds__(256) expand_pull_long_kernel(Adj in, const uint64_t* ns_dev, uint8_t* flags, PullArgs p) {
    if (!hop_pulls(p, ns_dev)) return;
    int64_t nl = (int64_t)*p.long_count;
    if (nl > p.long_cap) nl = p.long_cap;
    const int lane = threadIdx.x & 63;
    const int64_t waves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    for (int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6; i < nl; i += waves) {
        const int32_t v = p.long_list[i];
        const int32_t d = in.deg[v];
        const int64_t o = in.off[v];
        for (int32_t j0 = PULL_OWN; j0 < d; j0 += 64) {
            const int32_t j = j0 + lane;
            bool hit = false;
            if (j < d) {
                const int32_t u = in.idx[o + j];
                hit = (p.src_bitmap[(uint32_t)u >> 5] >> (u & 31)) & 1u;
            }
            if (__ballot(hit)) {
                if (lane == 0) flags[v] = 1;
                break;
            }
        }
    }
}

}  // namespace

nrt_status k_expand_frontier(const Adj& out, const int32_t* src_list, const uint64_t* ns_dev, int64_t ns_bound,
                             uint8_t* flags, LayerCtrs* lc, int32_t* xhub_list, int64_t xhub_cap, const Adj& in,
                             const PullArgs& pull, hipStream_t s) {
    if (ns_bound <= 0) return NRT_OK;
    unsigned long long* xc = (unsigned long long*)&lc->n_xhubs;
    int64_t g1 = cdiv(ns_bound, 4);
    if (g1 > 4096) g1 = 4096;
    expand_kernel<<<(int)g1, 256, 0, s>>>(out, src_list, ns_dev, flags, xc, xhub_list, xhub_cap, pull);
    LAUNCH_CHECK();
    int64_t gx = ns_bound < 512 ? ns_bound : 512;
    expand_hubs_kernel<<<dim3((unsigned)gx, HUB_GY, 1), 256, 0, s>>>(out, flags, xc, xhub_list, xhub_cap);
    LAUNCH_CHECK();
    if (pull.allowed) {
        int64_t g2 = cdiv(pull.n, 256);
        if (g2 > 8192) g2 = 8192;
        expand_pull_kernel<<<(int)g2, 256, 0, s>>>(in, ns_dev, flags, pull);
        LAUNCH_CHECK();
        expand_pull_long_kernel<<<2048, 256, 0, s>>>(in, ns_dev, flags, pull);
        LAUNCH_CHECK();
    }
    return NRT_OK;
}
