// MoNet (Table II): the message of a vertex is the vector of its Gaussian kernel responses,
//   g_j(h) = exp(-1/2 sum_k prec[j][k] (h[k] - mu[j][k])^2),  j < J,
// which depends on the source row only, so the model folds deltas like the sum models: this file only provides the
// per-vertex transform h -> g(h) on the rows whose h changed (and their compact deltas new - old for the gather).
#include "common.h"

namespace {

constexpr int MN_WAVES = 4;

// One wave per listed row.  The row sits in LDS; lane j (and j + 64, ...) walks the row for kernel j with the
// transposed parameter tables, so that the 64 lanes read consecutive floats.
__global__ void __launch_bounds__(MN_WAVES * 64) monet_transform_kernel(MonetArgs a) {
    __shared__ float s_row[MN_WAVES][1024];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    int64_t count = a.rows ? (int64_t)*a.count_dev : a.bound;
    if (count > a.bound) count = a.bound;
    const int64_t waves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    const int d = a.d, J = a.J;
    for (int64_t m = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6; m < count; m += waves) {
        const int64_t v = a.rows ? (int64_t)a.rows[m] : m;
        const int64_t hr = a.h_is_compact ? m : v;        // compact input: row m belongs to vertex rows[m]
        for (int k = lane; k < d; k += 64) s_row[w][k] = a.H[hr * d + k];
        __builtin_amdgcn_wave_barrier();
        for (int j = lane; j < J; j += 64) {
            float q = 0.f;
            for (int k = 0; k < d; ++k) {
                const float t = s_row[w][k] - a.muT[(int64_t)k * J + j];
                q += a.precT[(int64_t)k * J + j] * t * t;
            }
            const float g = expf(-0.5f * q);
            if (a.DP) a.DP[m * J + j] = g - a.G[v * J + j];
            a.G[v * J + j] = g;
        }
        __builtin_amdgcn_wave_barrier();
    }
}

}  // namespace

nrt_status k_monet_transform(const MonetArgs& a, hipStream_t s) {
    if (a.bound <= 0) return NRT_OK;
    if (a.d > 1024) { nrt_set_error("monet: rows wider than 1024 floats"); return NRT_ERR_UNSUPPORTED; }
    int64_t g = cdiv(a.bound, MN_WAVES);
    if (g > 4096) g = 4096;
    monet_transform_kernel<<<(int)g, MN_WAVES * 64, 0, s>>>(a);
    LAUNCH_CHECK();
    return NRT_OK;
}
