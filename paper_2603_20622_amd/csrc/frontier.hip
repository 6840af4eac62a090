// Affected-set expansion, one hop of Algorithm 4: the destinations of the out-edges of the previous
// hop's affected vertices join the affected set of this hop.  The set is a bitmap over vertex ids; the
// caller has already OR-ed in the destinations of the updated edges and the previous set itself, and
// afterwards compacts the bitmap into a sorted id list.
//
// Work split: one wave per source walks an out-list of up to HUB_DEG entries; longer lists are queued and
// then walked by many workgroups at once, HUB_SPAN entries per workgroup step, so one celebrity vertex
// does not serialise the hop.
#include "common.h"

namespace {

constexpr int HUB_DEG = 2048;
constexpr int HUB_SPAN = 4096;
constexpr int HUB_GX = 64, HUB_GY = 32;

__device__ inline void mark(uint32_t* bitmap, int32_t v) {
    const uint32_t bit = 1u << (v & 31);
    uint32_t* w = &bitmap[v >> 5];
    if (!(*w & bit)) atomicOr(w, bit);   // test first (a stale 0 only costs a redundant atomic): most bits are already set on dense hops
}

__global__ void expand_kernel(Adj out, const int32_t* src_list, int64_t ns, uint32_t* bitmap,
                              unsigned long long* hub_count, int32_t* hub_list, int64_t hub_cap) {
    const int64_t s = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int lane = threadIdx.x & 63;
    if (s >= ns) return;
    const int32_t u = src_list[s];
    const int32_t d = out.deg[u];
    if (d > HUB_DEG) {
        if (lane == 0) {
            unsigned long long p = atomicAdd(hub_count, 1ULL);
            if ((int64_t)p < hub_cap) hub_list[p] = u;
        }
        return;
    }
    const int64_t o = out.off[u];
    for (int32_t j = lane; j < d; j += 64) mark(bitmap, out.idx[o + j]);
}

// few sources: a workgroup column per source, gridDim.y workgroups share a long out-list
__global__ void expand_block_kernel(Adj out, const int32_t* src_list, uint32_t* bitmap) {
    const int32_t u = src_list[blockIdx.x];
    const int32_t d = out.deg[u];
    const int64_t o = out.off[u];
    const int32_t stride = gridDim.y * blockDim.x;
    int32_t j = blockIdx.y * blockDim.x + threadIdx.x;
    for (; j + 3 * stride < d; j += 4 * stride) {
        const int32_t v0 = out.idx[o + j], v1 = out.idx[o + j + stride], v2 = out.idx[o + j + 2 * stride],
                      v3 = out.idx[o + j + 3 * stride];
        mark(bitmap, v0); mark(bitmap, v1); mark(bitmap, v2); mark(bitmap, v3);
    }
    for (; j < d; j += stride) mark(bitmap, out.idx[o + j]);
}

__global__ void expand_hubs_kernel(Adj out, uint32_t* bitmap, const unsigned long long* hub_count,
                                   const int32_t* hub_list, int64_t hub_cap) {
    int64_t nh = (int64_t)*hub_count;
    if (nh > hub_cap) nh = hub_cap;
    for (int64_t h = blockIdx.x; h < nh; h += gridDim.x) {
        const int32_t u = hub_list[h];
        const int32_t d = out.deg[u];
        const int64_t o = out.off[u];
        for (int32_t start = blockIdx.y * HUB_SPAN; start < d; start += gridDim.y * HUB_SPAN) {
            const int32_t end = min(d, start + HUB_SPAN);
            for (int32_t j = start + threadIdx.x; j < end; j += blockDim.x) mark(bitmap, out.idx[o + j]);
        }
    }
}

}  // namespace

nrt_status k_expand_frontier(const Adj& out, const int32_t* src_list, int64_t ns, uint32_t* bitmap,
                             int64_t* hub_scratch, int64_t hub_cap, hipStream_t s) {
    if (ns <= 0) return NRT_OK;
    if (ns <= 16384) {
        expand_block_kernel<<<dim3((unsigned)ns, 16, 1), 256, 0, s>>>(out, src_list, bitmap);
        LAUNCH_CHECK();
        return NRT_OK;
    }
    unsigned long long* hub_count = (unsigned long long*)hub_scratch;
    int32_t* hub_list = (int32_t*)(hub_scratch + 1);
    NRT_TRY(k_fill_u64((uint64_t*)hub_count, 1, 0, s));
    expand_kernel<<<(int)cdiv(ns * 64, 256), 256, 0, s>>>(out, src_list, ns, bitmap, hub_count, hub_list, hub_cap);
    LAUNCH_CHECK();
    expand_hubs_kernel<<<dim3(HUB_GX, HUB_GY, 1), 256, 0, s>>>(out, bitmap, hub_count, hub_list, hub_cap);
    LAUNCH_CHECK();
    return NRT_OK;
}
