// Small device primitives: fills, word-wise OR, exclusive scan, bitmap -> sorted id list compaction.
#include "common.h"

namespace {

constexpr int TPB = 256;     // threads per block of the scan kernels
constexpr int EPT = 4;       // elements per thread
constexpr int EPB = TPB * EPT;

__device__ inline uint64_t wave_incl_scan(uint64_t v) {
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        uint64_t o = __shfl_up((unsigned long long)v, d, 64);
        if (lane >= d) v += o;
    }
    return v;
}

// exclusive scan of one value per thread over the block; returns exclusive prefix, *block_total = sum
__device__ inline uint64_t block_excl_scan(uint64_t v, uint64_t* block_total) {
    __shared__ uint64_t wsum[TPB / 64];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    uint64_t inc = wave_incl_scan(v);
    if (lane == 63) wsum[w] = inc;
    __syncthreads();
    uint64_t base = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < TPB / 64; ++i) {
        uint64_t t = wsum[i];
        if (i < w) base += t;
        tot += t;
    }
    __syncthreads();
    *block_total = tot;
    return base + inc - v;
}

__global__ void fill_u32_kernel(uint32_t* p, int64_t n, uint32_t v) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = v;
}
__global__ void fill_u64_kernel(uint64_t* p, int64_t n, uint64_t v) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = v;
}
__global__ void multi_fill_kernel(FillJobs f) {
    const FillJob j = f.j[blockIdx.y];
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < j.n; i += stride) j.p[i] = j.v;
}
// dst[i][:] = src[list[i]][:] for i < min(*count, cap); one wave per row, 16 bytes per lane and trip
__global__ void gather_rows_kernel(float* dst, const float* src, const int32_t* list, const uint64_t* count, int64_t cap, int D) {
    int64_t n = (int64_t)*count;
    if (n > cap) n = cap;
    const int lane = threadIdx.x & 63;
    const int64_t waves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    for (int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6; i < n; i += waves) {
        const float* p = src + (int64_t)list[i] * D;
        for (int k = lane * 4; k < D; k += 256)
            *reinterpret_cast<float4*>(dst + i * D + k) = *reinterpret_cast<const float4*>(p + k);
    }
}
// dst[i][:] = src[ids[i]][:] for i < n_ids; an id outside [0, n) reads row 0 (the caller reports it as an error)
__global__ void gather_rows_checked_kernel(float* dst, const float* src, const int32_t* ids, int64_t n_ids, int64_t n, int D) {
    const int lane = threadIdx.x & 63;
    const int64_t waves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    for (int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6; i < n_ids; i += waves) {
        int32_t v = ids[i];
        if (v < 0 || v >= n) v = 0;
        const float* p = src + (int64_t)v * D;
        for (int k = lane * 4; k < D; k += 256)
            *reinterpret_cast<float4*>(dst + i * D + k) = *reinterpret_cast<const float4*>(p + k);
    }
}
__global__ void or_words_kernel(uint32_t* dst, const uint32_t* a, const uint32_t* b, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) dst[i] = a[i] | (b ? b[i] : 0u);
}
__global__ void concat_ids_kernel(int32_t* dst, const int32_t* a, int64_t na, const int32_t* b, int64_t nb, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < na + nb; i += stride) {
        const int32_t v = i < na ? a[i] : b[i - na];
        dst[i] = (v >= 0 && v < n) ? v : 0;
    }
}
__global__ void copy_u32_kernel(uint32_t* dst, const uint32_t* src, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) dst[i] = src[i];
}

// ---- scan ----
__global__ void scan_reduce_kernel(const uint64_t* data, int64_t n, uint64_t* tmp) {
    const int64_t base = (int64_t)blockIdx.x * EPB + (int64_t)threadIdx.x * EPT;
    uint64_t s = 0;
#pragma unroll
    for (int j = 0; j < EPT; ++j)
        if (base + j < n) s += data[base + j];
    uint64_t tot;
    block_excl_scan(s, &tot);
    if (threadIdx.x == 0) tmp[blockIdx.x] = tot;
}
// one block: exclusive scan of tmp[0..nb) in place, total out
__global__ void scan_top_kernel(uint64_t* tmp, int64_t nb, uint64_t* total) {
    uint64_t carry = 0;
    for (int64_t start = 0; start < nb; start += TPB) {
        int64_t i = start + threadIdx.x;
        uint64_t v = i < nb ? tmp[i] : 0;
        uint64_t tot;
        uint64_t ex = block_excl_scan(v, &tot);
        if (i < nb) tmp[i] = carry + ex;
        carry += tot;
    }
    if (threadIdx.x == 0) *total = carry;
}
__global__ void scan_apply_kernel(uint64_t* data, int64_t n, const uint64_t* tmp) {
    const int64_t base = (int64_t)blockIdx.x * EPB + (int64_t)threadIdx.x * EPT;
    uint64_t v[EPT];
    uint64_t s = 0;
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
        v[j] = base + j < n ? data[base + j] : 0;
        s += v[j];
    }
    uint64_t tot;
    uint64_t ex = block_excl_scan(s, &tot) + tmp[blockIdx.x];
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
        if (base + j < n) data[base + j] = ex;
        ex += v[j];
    }
}

// ---- set compaction ----
// word w of the set = (byte flags 32w .. 32w+31 packed) | or_a[w] | or_b[w]; the flags are cleared on the way
__device__ inline uint32_t pack_flags(uint8_t* flags, int64_t w, int64_t n) {
    uint32_t bits = 0;
    const int64_t v0 = w * 32;
    if (v0 + 32 <= n) {
        uint4* p = reinterpret_cast<uint4*>(flags + v0);
        const uint4 a = p[0], b = p[1];
        const uint32_t q[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
        uint32_t any = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            any |= q[i];
#pragma unroll
            for (int j = 0; j < 4; ++j) bits |= ((q[i] >> (8 * j)) & 0xffu ? 1u : 0u) << (4 * i + j);
        }
        if (any) { p[0] = make_uint4(0, 0, 0, 0); p[1] = make_uint4(0, 0, 0, 0); }
    } else {
        for (int64_t v = v0; v < n; ++v) {
            if (flags[v]) { bits |= 1u << (v - v0); flags[v] = 0; }
        }
    }
    return bits;
}
// bm |= ids (ids outside [0, n) raise *bad instead)
__global__ void mark_ids_kernel(uint32_t* bm, const int32_t* ids, int64_t n_ids, int64_t n, int32_t* bad) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_ids) return;
    const int32_t v = ids[i];
    if (v < 0 || v >= n) { *bad = 1; return; }
    atomicOr(&bm[v >> 5], 1u << (v & 31));
}
// bm &= ~(listed ids)
__global__ void clear_listed_bits_kernel(uint32_t* bm, const int32_t* list, const uint64_t* count) {
    const int64_t n = (int64_t)*count;
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) {
        const int32_t v = list[i];
        atomicAnd(&bm[v >> 5], ~(1u << (v & 31)));
    }
}
// Single-pass compaction.  A workgroup takes a ticket (so that every workgroup with a smaller ticket is already
// running), builds its 1024 words of the set and counts them, publishes the count, finds the number of set bits in
// front of it by looking back over its predecessors' published counts and running totals (one 64-bit cell per
// workgroup: status, call number, value; a cell of an earlier call reads as "not there yet", so nothing is cleared
// between calls), and emits its ids.  Layout of `state`: [0] ticket counter, [1] number of the last finished call,
// [2 + t] the cell of ticket t.  Every wait is on a workgroup that already runs and publishes before it waits itself;
// as a last resort a wait gives up after about a million polls and raises *err.
constexpr uint64_t CS_AGG = 1ULL << 62, CS_PREFIX = 2ULL << 62, CS_STATUS = 3ULL << 62, CS_VALUE = (1ULL << 40) - 1;
constexpr int CS_SPIN_LIMIT = 1 << 20;
struct CompactArgs {
    uint8_t* flags; const uint32_t *or_a, *or_b, *and_mask;
    uint32_t* out_bm; int64_t n, nw, nb;
    int32_t *list, *slot;
    unsigned long long* state; uint64_t* count;
    CompactExtra x;
};
// CEPT words per thread: 1 for sets over up to four million vertices (more, smaller workgroups: the ids of a word are
// emitted one after the other by its thread), 4 beyond
template <int CEPT>
__global__ void __launch_bounds__(TPB) compact_kernel(CompactArgs a) {
    constexpr int CEPB = TPB * CEPT;
    __shared__ uint64_t s_excl;
    __shared__ uint32_t s_words[CEPB];
    __shared__ int64_t s_ticket;
    __shared__ uint32_t s_call;
    const int tid = threadIdx.x, lane = tid & 63;
    if (tid == 0) {
        // acquire: the ticket below must not be taken before this value has arrived (the last ticket's workgroup rewrites it)
        s_call = ((uint32_t)__hip_atomic_load(&a.state[1], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT) + 1u) & 0x3fffffu;
        s_ticket = (int64_t)atomicAdd(&a.state[0], 1ULL);
    }
    __syncthreads();
    const int64_t t = s_ticket;
    const uint64_t call_tag = (uint64_t)s_call << 40;
    const int64_t base = t * CEPB + (int64_t)tid * CEPT;
    uint32_t w[CEPT];
    uint64_t cnt = 0;
#pragma unroll
    for (int j = 0; j < CEPT; ++j) {
        const int64_t wi = base + j;
        uint32_t bits = 0;
        if (wi < a.nw) {
            bits = a.flags ? pack_flags(a.flags, wi, a.n) : 0u;
            if (a.or_a) bits |= a.or_a[wi];
            if (a.or_b) bits |= a.or_b[wi];
            if (a.and_mask) bits &= a.x.and_invert ? ~a.and_mask[wi] : a.and_mask[wi];
            a.out_bm[wi] = bits;
        }
        w[j] = bits;
        s_words[tid * CEPT + j] = bits;
        cnt += __popc(bits);
    }
    uint64_t tot;
    const uint64_t ex = block_excl_scan(cnt, &tot);
    if (tid < 64) {
        unsigned long long* cell = &a.state[2 + t];
        uint64_t excl = 0;
        if (t == 0) {
            if (lane == 0) __hip_atomic_store(cell, CS_PREFIX | call_tag | tot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        } else {
            if (lane == 0) __hip_atomic_store(cell, CS_AGG | call_tag | tot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            int64_t look = t - 1;                       // lane i looks at ticket look - i
            bool failed = false;
            while (true) {
                const int64_t p = look - lane;
                uint64_t cellv = CS_PREFIX | call_tag;  // in front of ticket 0: a running total of 0
                int spins = 0;
                if (p >= 0) {
                    while (true) {
                        cellv = __hip_atomic_load(&a.state[2 + p], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        if ((cellv & CS_STATUS) != 0 && (cellv & ~(CS_STATUS | CS_VALUE)) == call_tag) break;
                        if (++spins > CS_SPIN_LIMIT) { failed = true; cellv = CS_PREFIX | call_tag; break; }
                        __builtin_amdgcn_s_sleep(2);
                    }
                }
                const unsigned long long has_prefix = __ballot((cellv & CS_STATUS) == CS_PREFIX);
                const int first = has_prefix ? __ffsll((long long)has_prefix) - 1 : 64;     // nearest predecessor with a running total
                uint64_t v = lane <= first ? (cellv & CS_VALUE) : 0;
#pragma unroll
                for (int sft = 32; sft >= 1; sft >>= 1) v += __shfl_xor((unsigned long long)v, sft, 64);
                excl += v;
                if (has_prefix) break;
                look -= 64;
            }
            if (__ballot(failed) && lane == 0 && a.x.err) *a.x.err = 1;
            if (lane == 0) __hip_atomic_store(cell, CS_PREFIX | call_tag | ((excl + tot) & CS_VALUE), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        if (lane == 0) {
            s_excl = excl;
            if (t == a.nb - 1) {        // every other workgroup has read the call number and taken its ticket by now
                *a.count = excl + tot;
                __hip_atomic_store(&a.state[1], (unsigned long long)s_call, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(&a.state[0], 0ULL, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }
    __syncthreads();
    uint64_t pos = s_excl + ex;
#pragma unroll
    for (int j = 0; j < CEPT; ++j) {
        uint32_t bits = w[j];
        while (bits) {
            const int b = __ffs(bits) - 1;
            bits &= bits - 1;
            const int32_t v = (int32_t)((base + j) * 32 + b);
            a.list[pos] = v;
            if (a.slot) a.slot[v] = (int32_t)pos;
            if (a.x.list2 && (int64_t)pos < a.x.cap2) a.x.list2[pos] = v;
            ++pos;
        }
    }
    // coarse copy of the set: bit i covers vertices [i << shift, (i + 1) << shift); the words of this workgroup cover
    // 32 * CEPB consecutive vertices, i.e. whole coarse words as long as a coarse word spans at most that many
    if (a.x.coarse) {
        const int sh = a.x.coarse_shift;                         // a coarse word spans at most this workgroup (checked by the host)
        const int per_block = CEPB >> sh;                        // coarse words of this workgroup
        for (int cw = tid; cw < per_block; cw += TPB) {
            uint32_t out = 0;
            for (int i = 0; i < 32; ++i) {
                const int v0 = (cw * 32 + i) << sh;              // first vertex of the bit's group, relative to the workgroup
                uint32_t any = 0;
                if (sh <= 5) {
                    const uint32_t word = s_words[v0 >> 5];
                    const uint32_t mask = sh == 5 ? 0xffffffffu : (((1u << (1 << sh)) - 1u) << (v0 & 31));
                    any = word & mask;
                } else {
                    const int w0 = v0 >> 5, nwg = 1 << (sh - 5);
                    for (int k = 0; k < nwg; ++k) any |= s_words[w0 + k];
                }
                if (any) out |= 1u << i;
            }
            const int64_t gcw = t * per_block + cw;
            if (gcw < a.x.coarse_words) a.x.coarse[gcw] = out;
        }
    }
}
__global__ void copy_counted_kernel(uint32_t* dst, const uint32_t* src, const uint64_t* count, int64_t cap) {
    int64_t n = (int64_t)*count;
    if (n > cap) n = cap;
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) dst[i] = src[i];
}

// ---- streaming kernels (bandwidth ceilings): a workgroup takes 8 * 256 consecutive 16-byte words per trip, eight
// independent loads per lane, marked non-temporal (streamed data is not worth a place in the caches; on this GPU the
// hint alone is worth more than a tenth of the read rate)
typedef float floatx4 __attribute__((ext_vector_type(4)));
constexpr int STREAM_U = 8;
__global__ void __launch_bounds__(256) stream_copy_kernel(floatx4* b, const floatx4* a, int64_t n4) {
    const int64_t chunk = (int64_t)STREAM_U * 256;
    const int64_t stride = (int64_t)gridDim.x * chunk;
    int64_t base = (int64_t)blockIdx.x * chunk + threadIdx.x;
    for (; base + (STREAM_U - 1) * 256 < n4; base += stride) {
        floatx4 x[STREAM_U];
#pragma unroll
        for (int u = 0; u < STREAM_U; ++u) x[u] = __builtin_nontemporal_load(a + base + u * 256);
#pragma unroll
        for (int u = 0; u < STREAM_U; ++u) __builtin_nontemporal_store(x[u], b + base + u * 256);
    }
    for (; base < n4; base += 256) b[base] = a[base];
}
__global__ void __launch_bounds__(256) stream_read_kernel(float* out, const floatx4* a, int64_t n4) {
    const int64_t chunk = (int64_t)STREAM_U * 256;
    const int64_t stride = (int64_t)gridDim.x * chunk;
    floatx4 s[STREAM_U];
#pragma unroll
    for (int u = 0; u < STREAM_U; ++u) s[u] = floatx4{0.f, 0.f, 0.f, 0.f};
    int64_t base = (int64_t)blockIdx.x * chunk + threadIdx.x;
    for (; base + (STREAM_U - 1) * 256 < n4; base += stride) {
        floatx4 x[STREAM_U];
#pragma unroll
        for (int u = 0; u < STREAM_U; ++u) x[u] = __builtin_nontemporal_load(a + base + u * 256);
#pragma unroll
        for (int u = 0; u < STREAM_U; ++u) s[u] += x[u];
    }
    for (; base < n4; base += 256) s[0] += a[base];
    float t = 0.f;
#pragma unroll
    for (int u = 0; u < STREAM_U; ++u) t += (s[u].x + s[u].y) + (s[u].z + s[u].w);
    if (t == -1.2345e30f) out[0] = t;        // keeps the loads alive; practically never taken
}

inline int grid_for(int64_t n, int tpb, int64_t cap = 65536) {
    int64_t g = cdiv(n, tpb);
    if (g < 1) g = 1;
    if (g > cap) g = cap;
    return (int)g;
}

}  // namespace

nrt_status k_fill_u32(uint32_t* p, int64_t n, uint32_t v, hipStream_t s) {
    if (n <= 0) return NRT_OK;
    fill_u32_kernel<<<grid_for(n, 256), 256, 0, s>>>(p, n, v);
    LAUNCH_CHECK();
    return NRT_OK;
}
nrt_status k_fill_u64(uint64_t* p, int64_t n, uint64_t v, hipStream_t s) {
    if (n <= 0) return NRT_OK;
    fill_u64_kernel<<<grid_for(n, 256), 256, 0, s>>>(p, n, v);
    LAUNCH_CHECK();
    return NRT_OK;
}
nrt_status k_multi_fill(const FillJobs& f, hipStream_t s) {
    if (f.count <= 0) return NRT_OK;
    int64_t longest = 0;
    for (int i = 0; i < f.count; ++i) longest = f.j[i].n > longest ? f.j[i].n : longest;
    if (longest <= 0) return NRT_OK;
    dim3 grid((unsigned)grid_for(longest, 256), (unsigned)f.count, 1);
    multi_fill_kernel<<<grid, 256, 0, s>>>(f);
    LAUNCH_CHECK();
    return NRT_OK;
}
nrt_status k_gather_rows(float* dst, const float* src, const int32_t* list, const uint64_t* count, int64_t cap, int64_t bound,
                         int D, hipStream_t s) {
    if (bound <= 0 || cap <= 0) return NRT_OK;
    int64_t g = cdiv(bound < cap ? bound : cap, 4);
    if (g > 4096) g = 4096;
    gather_rows_kernel<<<(int)g, 256, 0, s>>>(dst, src, list, count, cap, D);
    LAUNCH_CHECK();
    return NRT_OK;
}
nrt_status k_gather_rows_checked(float* dst, const float* src, const int32_t* ids, int64_t n_ids, int64_t n, int D,
                                 hipStream_t s) {
    if (n_ids <= 0) return NRT_OK;
    int64_t g = cdiv(n_ids, 4);
    if (g > 4096) g = 4096;
    gather_rows_checked_kernel<<<(int)g, 256, 0, s>>>(dst, src, ids, n_ids, n, D);
    LAUNCH_CHECK();
    return NRT_OK;
}
nrt_status k_or_words(uint32_t* dst, const uint32_t* a, const uint32_t* b, int64_t nwords, hipStream_t s) {
    if (nwords <= 0) return NRT_OK;
    or_words_kernel<<<grid_for(nwords, 256), 256, 0, s>>>(dst, a, b, nwords);
    LAUNCH_CHECK();
    return NRT_OK;
}
nrt_status k_concat_ids(int32_t* dst, const int32_t* a, int64_t na, const int32_t* b, int64_t nb, int64_t n, hipStream_t s) {
    if (na + nb <= 0) return NRT_OK;
    concat_ids_kernel<<<grid_for(na + nb, 256), 256, 0, s>>>(dst, a, na, b, nb, n);
    LAUNCH_CHECK();
    return NRT_OK;
}
nrt_status k_copy_i32(int32_t* dst, const int32_t* src, int64_t n, hipStream_t s) {
    if (n <= 0) return NRT_OK;
    copy_u32_kernel<<<grid_for(n, 256), 256, 0, s>>>((uint32_t*)dst, (const uint32_t*)src, n);
    LAUNCH_CHECK();
    return NRT_OK;
}
nrt_status k_copy_f32(float* dst, const float* src, int64_t n, hipStream_t s) {
    if (n <= 0) return NRT_OK;
    copy_u32_kernel<<<grid_for(n, 256), 256, 0, s>>>((uint32_t*)dst, (const uint32_t*)src, n);
    LAUNCH_CHECK();
    return NRT_OK;
}

nrt_status k_stream_copy(float* b, const float* a, int64_t n_floats, hipStream_t s) {
    if (n_floats < 4) return NRT_OK;
    const int64_t n4 = n_floats / 4;
    stream_copy_kernel<<<grid_for(n4 / STREAM_U, 256, 65536), 256, 0, s>>>((floatx4*)b, (const floatx4*)a, n4);
    LAUNCH_CHECK();
    return NRT_OK;
}
nrt_status k_stream_read(float* b, const float* a, int64_t n_floats, hipStream_t s) {
    if (n_floats < 4) return NRT_OK;
    const int64_t n4 = n_floats / 4;
    stream_read_kernel<<<grid_for(n4 / STREAM_U, 256, 65536), 256, 0, s>>>(b, (const floatx4*)a, n4);
    LAUNCH_CHECK();
    return NRT_OK;
}

nrt_status k_exclusive_scan_u64(uint64_t* data, int64_t n, uint64_t* tmp, int64_t tmp_len, uint64_t* total, hipStream_t s) {
    const int64_t nb = n > 0 ? cdiv(n, EPB) : 0;
    if (nb > tmp_len) { nrt_set_error("scan scratch too small"); return NRT_ERR_INVALID_ARG; }
    if (nb > 0) { scan_reduce_kernel<<<(int)nb, TPB, 0, s>>>(data, n, tmp); LAUNCH_CHECK(); }
    scan_top_kernel<<<1, TPB, 0, s>>>(tmp, nb, total);
    LAUNCH_CHECK();
    if (nb > 0) { scan_apply_kernel<<<(int)nb, TPB, 0, s>>>(data, n, tmp); LAUNCH_CHECK(); }
    return NRT_OK;
}

namespace {

// relation ids held as edge weights: integers in [0, R); anything else raises *bad
__device__ inline bool bad_relation(float w, int R) { return !(w >= 0.0f && w < (float)R && w == (float)(int)w); }

__global__ void check_relations_kernel(const float* w, int64_t count, int R, int32_t* bad) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count && bad_relation(w[i], R)) *bad = 1;
}

// the same over the live entries of every adjacency list: one wave per vertex, strided
__global__ void check_list_relations_kernel(Adj a, int64_t n, int R, int32_t* bad) {
    const int lane = threadIdx.x & 63;
    const int64_t waves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    for (int64_t v = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6; v < n; v += waves) {
        const int64_t off = a.off[v];
        const int32_t deg = a.deg[v];
        for (int32_t j = lane; j < deg; j += 64)
            if (bad_relation(a.wts[off + j], R)) *bad = 1;
    }
}

}  // namespace

nrt_status k_check_relations(const float* w, int64_t count, int R, int32_t* bad, hipStream_t s) {
    if (count <= 0) return NRT_OK;
    check_relations_kernel<<<(int)cdiv(count, 256), 256, 0, s>>>(w, count, R, bad);
    LAUNCH_CHECK();
    return NRT_OK;
}
nrt_status k_check_list_relations(const Adj& a, int64_t n, int R, int32_t* bad, hipStream_t s) {
    if (n <= 0) return NRT_OK;
    check_list_relations_kernel<<<grid_for(n * 64, 256, 4096), 256, 0, s>>>(a, n, R, bad);
    LAUNCH_CHECK();
    return NRT_OK;
}

nrt_status k_mark_ids(uint32_t* bm, const int32_t* ids, int64_t n_ids, int64_t n, int32_t* bad, hipStream_t s) {
    if (n_ids <= 0) return NRT_OK;
    mark_ids_kernel<<<(int)cdiv(n_ids, 256), 256, 0, s>>>(bm, ids, n_ids, n, bad);
    LAUNCH_CHECK();
    return NRT_OK;
}
nrt_status k_clear_listed_bits(uint32_t* bm, const int32_t* list, const uint64_t* count, int64_t bound, hipStream_t s) {
    if (bound <= 0) return NRT_OK;
    clear_listed_bits_kernel<<<grid_for(bound, 256, 2048), 256, 0, s>>>(bm, list, count);
    LAUNCH_CHECK();
    return NRT_OK;
}
nrt_status k_compact(uint8_t* flags, const uint32_t* or_a, const uint32_t* or_b, uint32_t* out_bm, int64_t n,
                     int32_t* list, int32_t* slot, uint64_t* state, int64_t state_len, uint64_t* count, hipStream_t s,
                     const uint32_t* and_mask, const CompactExtra* extra) {
    const int64_t nw = cdiv(n, 32);
    const int cept = nw <= 131072 ? 1 : 4;
    const int64_t nb = nw > 0 ? cdiv(nw, (int64_t)TPB * cept) : 0;
    if (nb + 2 > state_len) { nrt_set_error("compaction state too small"); return NRT_ERR_INVALID_ARG; }
    if (nb <= 0) return k_fill_u64(count, 1, 0, s);
    CompactArgs a;
    memset(&a, 0, sizeof(a));
    a.flags = flags; a.or_a = or_a; a.or_b = or_b; a.and_mask = and_mask;
    a.out_bm = out_bm; a.n = n; a.nw = nw; a.nb = nb;
    a.list = list; a.slot = slot;
    a.state = (unsigned long long*)state; a.count = count;
    if (extra) a.x = *extra;
    if (a.x.coarse && (1 << a.x.coarse_shift) > TPB * cept) {   // a coarse word would span several workgroups: built by its own kernel
        nrt_set_error("internal: coarse shift beyond the compaction's reach");
        return NRT_ERR_INVALID_ARG;
    }
    if (cept == 1) compact_kernel<1><<<(int)nb, TPB, 0, s>>>(a);
    else compact_kernel<4><<<(int)nb, TPB, 0, s>>>(a);
    LAUNCH_CHECK();
    return NRT_OK;
}

nrt_status k_copy_counted_i32(int32_t* dst, const int32_t* src, const uint64_t* count, int64_t cap, int64_t bound, hipStream_t s) {
    if (cap <= 0 || bound <= 0) return NRT_OK;
    copy_counted_kernel<<<grid_for(bound < cap ? bound : cap, 256, 2048), 256, 0, s>>>((uint32_t*)dst, (const uint32_t*)src, count, cap);
    LAUNCH_CHECK();
    return NRT_OK;
}
