// Affected-row dense update (Algorithm 1 line 7; "update" column of Table II) as an fp32 MFMA GEMM.
//
//   Y[m][:] = act( A[m][:] . W + bias ),  m over the affected rows only,
// where row m of A is formed on the fly from the cached rows of vertex rows[m]:
//   A_PLAIN        P0[v]
//   A_SCALE_GCN    P0[v] / sqrt(indeg(v)+1)                (msg_cbn of the GCN row applied to the cached sum)
//   A_CONCAT_MEAN  [ P0[v] || P1[v] / indeg(v) ]           (GraphSAGE: self row, mean = cached sum / count)
//   A_AXPY         c * P0[v] + P1[v]                       (GIN: (1+eps) x_v + cached weighted sum)
// The epilogue is the cache write-back: it stores the new row into h^l[v] and, for the next layer, the
// change of the source payload dp = y_new*cn - y_old*co (cn = co = 1 except for GCN, where the payload is
// y / sqrt(d_v) and the degree may have changed), so no separate pass re-reads the rows.
//
// Tiling: 256 threads = 4 waves; block tile 128 x BN; K is consumed in slices of 32 staged through LDS
// (rows padded to 36 floats so that the 16-byte operand reads of 8 neighbouring lanes cover all banks).
// Each wave owns (TM x TN) 32x32 accumulator tiles fed by v_mfma_f32_32x32x2_f32: lane = (i mod 32, half),
// the two halves supply two different k, so one 16-byte LDS read per operand feeds four MFMAs.
// Weights are kept transposed ([out][in]) so that both operands are read along k.
#include "common.h"

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BM = 128;
constexpr int KT = 32;
constexpr int LDS_STRIDE = KT + 4;

__device__ inline float gcn_scale(int32_t indeg) { return 1.0f / sqrtf((float)(indeg + 1)); }

__device__ inline float4 load_a(const GemmArgs& g, int64_t v, float sc, int k, bool ok) {
    float4 r = make_float4(0.f, 0.f, 0.f, 0.f);
    if (!ok || k >= g.K) return r;
    switch (g.a_mode) {
    case A_PLAIN:
        r = *reinterpret_cast<const float4*>(g.P0 + v * g.ldp + k);
        break;
    case A_SCALE_GCN: {
        r = *reinterpret_cast<const float4*>(g.P0 + v * g.ldp + k);
        r.x *= sc; r.y *= sc; r.z *= sc; r.w *= sc;
        break;
    }
    case A_CONCAT_MEAN:
        if (k < g.ldp) {
            r = *reinterpret_cast<const float4*>(g.P0 + v * g.ldp + k);
        } else {
            r = *reinterpret_cast<const float4*>(g.P1 + v * g.ldp + (k - g.ldp));
            r.x *= sc; r.y *= sc; r.z *= sc; r.w *= sc;
        }
        break;
    default: {
        const float4 p = *reinterpret_cast<const float4*>(g.P0 + v * g.ldp + k);
        const float4 q = *reinterpret_cast<const float4*>(g.P1 + v * g.ldp + k);
        r.x = fmaf(g.axpy_c, p.x, q.x); r.y = fmaf(g.axpy_c, p.y, q.y);
        r.z = fmaf(g.axpy_c, p.z, q.z); r.w = fmaf(g.axpy_c, p.w, q.w);
    }
    }
    return r;
}

template <int BN, int WM, int WN>
__global__ void __launch_bounds__(256) gemm_kernel(GemmArgs g) {
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    constexpr int A_LOADS = BM * KT / 4 / 256;   // float4 per thread per slice
    constexpr int B_LOADS = BN * KT / 4 / 256;
    __shared__ __attribute__((aligned(16))) float As[BM * LDS_STRIDE];
    __shared__ __attribute__((aligned(16))) float Bs[BN * LDS_STRIDE];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int64_t row_base = (int64_t)blockIdx.x * BM;
    const int col_base = blockIdx.y * BN;

    // rows this thread stages
    const int lr = tid >> 3, lk = (tid & 7) * 4;
    int64_t av[A_LOADS];
    float asc[A_LOADS];
    bool aok[A_LOADS];
#pragma unroll
    for (int p = 0; p < A_LOADS; ++p) {
        const int64_t m = row_base + lr + 32 * p;
        aok[p] = m < g.M;
        av[p] = aok[p] ? ((g.rows && !g.a_is_compact) ? (int64_t)g.rows[m] : m) : 0;
        asc[p] = 1.0f;
        if (aok[p] && g.a_mode == A_SCALE_GCN) asc[p] = gcn_scale(g.indeg[av[p]]);
        if (aok[p] && g.a_mode == A_CONCAT_MEAN) {
            const int32_t d = g.indeg[av[p]];
            asc[p] = d > 0 ? 1.0f / (float)d : 0.0f;
        }
    }

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    float4 ra[A_LOADS], rb[B_LOADS];
    auto fetch = [&](int k0) {
#pragma unroll
        for (int p = 0; p < A_LOADS; ++p) ra[p] = load_a(g, av[p], asc[p], k0 + lk, aok[p]);
#pragma unroll
        for (int p = 0; p < B_LOADS; ++p) {
            const int n = col_base + lr + 32 * p;
            const int k = k0 + lk;
            rb[p] = (n < g.N && k < g.K) ? *reinterpret_cast<const float4*>(g.Wt + (int64_t)n * g.K + k)
                                          : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    };

    fetch(0);
    const int half = lane >> 5, l32 = lane & 31;
    for (int k0 = 0; k0 < g.K; k0 += KT) {
#pragma unroll
        for (int p = 0; p < A_LOADS; ++p)
            *reinterpret_cast<float4*>(&As[(lr + 32 * p) * LDS_STRIDE + lk]) = ra[p];
#pragma unroll
        for (int p = 0; p < B_LOADS; ++p)
            *reinterpret_cast<float4*>(&Bs[(lr + 32 * p) * LDS_STRIDE + lk]) = rb[p];
        __syncthreads();
        if (k0 + KT < g.K) fetch(k0 + KT);
#pragma unroll
        for (int kk = 0; kk < KT; kk += 8) {
            float4 a[TM], b[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                a[i] = *reinterpret_cast<const float4*>(&As[((wm * TM + i) * 32 + l32) * LDS_STRIDE + kk + half * 4]);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                b[j] = *reinterpret_cast<const float4*>(&Bs[((wn * TN + j) * 32 + l32) * LDS_STRIDE + kk + half * 4]);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i].x, b[j].x, acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i].y, b[j].y, acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i].z, b[j].z, acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i].w, b[j].w, acc[i][j], 0, 0, 0);
                }
        }
        __syncthreads();
    }

    // epilogue = write-back
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int64_t m = row_base + (wm * TM + i) * 32 + 8 * (r / 4) + 4 * half + (r % 4);
            if (m >= g.M) continue;
            const int64_t v = g.rows ? (int64_t)g.rows[m] : m;
            float cn = 1.0f, co = 1.0f;
            if (g.DP && g.dp_scale_gcn) { cn = gcn_scale(g.indeg[v]); co = gcn_scale(g.indeg_old[v]); }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int n = col_base + (wn * TN + j) * 32 + l32;
                if (n >= g.N) continue;
                float y = acc[i][j][r];
                if (g.bias) y += g.bias[n];
                if (g.act == 1) y = fmaxf(y, 0.f);
                else if (g.act == 2) y = y > 0.f ? y : expm1f(y);
                if (g.out_compact) g.out_compact[m * g.N + n] = y;
                if (g.H) {
                    float* hp = g.H + v * g.N + n;
                    if (g.DP) g.DP[m * g.N + n] = y * cn - *hp * co;
                    *hp = y;
                }
            }
        }
    }
}

__global__ void transpose_kernel(const float* W, float* Wt, int K, int N) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < K * N) {
        const int k = i / N, n = i % N;
        Wt[(int64_t)n * K + k] = W[i];
    }
}

}  // namespace

nrt_status k_gemm(const GemmArgs& g, hipStream_t s) {
    if (g.M <= 0) return NRT_OK;
    if (g.K % 4 || g.ldp % 4) { nrt_set_error("gemm: widths must be multiples of 4"); return NRT_ERR_UNSUPPORTED; }
    const unsigned gx = (unsigned)cdiv(g.M, BM);
    if (g.N > 128) {
        gemm_kernel<256, 2, 2><<<dim3(gx, (unsigned)cdiv(g.N, 256)), 256, 0, s>>>(g);
    } else if (g.N > 64) {
        gemm_kernel<128, 2, 2><<<dim3(gx, 1), 256, 0, s>>>(g);
    } else if (g.N > 32) {
        gemm_kernel<64, 4, 1><<<dim3(gx, 1), 256, 0, s>>>(g);
    } else {
        gemm_kernel<32, 4, 1><<<dim3(gx, 1), 256, 0, s>>>(g);
    }
    LAUNCH_CHECK();
    return NRT_OK;
}

nrt_status k_transpose(const float* W, float* Wt, int K, int N, hipStream_t s) {
    transpose_kernel<<<(int)cdiv((int64_t)K * N, 256), 256, 0, s>>>(W, Wt, K, N);
    LAUNCH_CHECK();
    return NRT_OK;
}
