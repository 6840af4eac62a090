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
#include "common.h"

namespace {

constexpr int HUB_DEG = 512;
constexpr int HUB_GY = 16;      // workgroups that share one long out-list

__global__ void __launch_bounds__(256) expand_kernel(Adj out, const int32_t* src_list, const uint64_t* ns_dev,
                                                     uint8_t* flags, unsigned long long* xhub_count,
                                                     int32_t* xhub_list, int64_t xhub_cap) {
    __shared__ int s_n;
    __shared__ unsigned long long s_base;
    __shared__ int32_t s_q[4];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
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

}  // namespace

nrt_status k_expand_frontier(const Adj& out, const int32_t* src_list, const uint64_t* ns_dev, int64_t ns_bound,
                             uint8_t* flags, LayerCtrs* lc, int32_t* xhub_list, int64_t xhub_cap, hipStream_t s) {
    if (ns_bound <= 0) return NRT_OK;
    unsigned long long* xc = (unsigned long long*)&lc->n_xhubs;
    int64_t g1 = cdiv(ns_bound, 4);
    if (g1 > 4096) g1 = 4096;
    expand_kernel<<<(int)g1, 256, 0, s>>>(out, src_list, ns_dev, flags, xc, xhub_list, xhub_cap);
    LAUNCH_CHECK();
    int64_t gx = ns_bound < 512 ? ns_bound : 512;
    expand_hubs_kernel<<<dim3((unsigned)gx, HUB_GY, 1), 256, 0, s>>>(out, flags, xc, xhub_list, xhub_cap);
    LAUNCH_CHECK();
    return NRT_OK;
}
