// Affected-row dense update (the update step of Algorithm 1; "update" column of Table II) as an fp32 MFMA GEMM.
//
//   Y[m][:] = act( A[m][:] . W + bias ),  m over the affected rows only,
// where row m of A is formed on the fly from the cached rows of vertex rows[m]:
//   A_PLAIN        P0[v]
//   A_SCALE_GCN    P0[v] / sqrt(indeg(v)+1)                (msg_cbn of the GCN row applied to the cached sum)
//   A_CONCAT_MEAN  [ P0[v] || P1[v] / indeg(v) ]           (GraphSAGE: self row, mean = cached sum / count;
//                                                           CommNet: indeg == nullptr, the cached sum itself)
//   A_AXPY         c * P0[v] + P1[v]                       (GIN: (1+eps) x_v + cached weighted sum)
//   A_PLAIN_ADD    P0[v], and add[v] / count(v) joins the product before the activation
//                                                          (RGCN: W_o h_v + mean of the relation messages)
//   A_AXPY_BIAS_RELU  ReLU(c * P0[v] + P1[v] + a_bias)     (GIN with its first product applied to the messages before
//                                                           the aggregation: P0 = x W_a by vertex, P1 = cached sum of those)
// The epilogue is the cache write-back: it stores the new row into h^l[v] and, for the next layer, the
// change of the source payload dp = y_new*cn - y_old*co (cn = co = 1 except for GCN, where the payload is
// y / sqrt(d_v) and the degree may have changed), so no separate pass re-reads the rows.
//
// Tiling: block tile 64 x {64, 128} with 4 waves, 64 x 256 with 8 waves (128 x 32 for the narrowest outputs).  Short
// tiles keep the register count low enough for several workgroups per compute unit, so one's row-index prologue
// and write-back epilogue overlap the others' MFMAs, and give small affected sets more tiles than compute units;
// K is consumed in slices of 32 staged through LDS
// (rows padded to 36 floats so that the 16-byte operand reads of 8 neighbouring lanes cover all banks).
// Each wave owns (TM x TN) 32x32 accumulator tiles fed by v_mfma_f32_32x32x2_f32: lane = (i mod 32, half),
// the two halves supply two different k, so one 16-byte LDS read per operand feeds four MFMAs.
// Weights are kept transposed ([out][in]) so that both operands are read along k.
#include "common.h"

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));


__device__ inline float gcn_scale(int32_t indeg) { return 1.0f / sqrtf((float)(indeg + 1)); }

// Branch-free on purpose: the address is clamped into the row, the raw value stays in registers and the mask /
// scale `mul` is applied only when the slice is written to LDS one iteration later, so that the loads of a slice
// are issued back to back and nothing waits for them before the MFMAs of the current slice have been issued.
constexpr bool two_sources(int amode) { return amode == A_AXPY || amode == A_AXPY_BIAS_RELU; }

template <int AMODE>
__device__ inline void load_a(const GemmArgs& g, int64_t v, float sc, int k, bool ok, float4& raw, float4& raw2, float& mul) {
    const bool live = ok && k < g.K;
    const int kc = k < g.K ? k : g.K - 4;
    float m = 1.0f;
    if (AMODE == A_PLAIN || AMODE == A_PLAIN_ADD) {
        raw = *reinterpret_cast<const float4*>(g.P0 + v * g.ldp + kc);
    } else if (AMODE == A_SCALE_GCN) {
        raw = *reinterpret_cast<const float4*>(g.P0 + v * g.ldp + kc);
        m = sc;
    } else if (AMODE == A_CONCAT_MEAN) {
        const bool self = kc < g.ldp;
        const float* p = (self ? g.P0 : g.P1) + v * g.ldp + (self ? kc : kc - g.ldp);
        raw = *reinterpret_cast<const float4*>(p);
        m = self ? 1.0f : sc;
    } else {
        raw = *reinterpret_cast<const float4*>(g.P0 + v * g.ldp + kc);
        raw2 = *reinterpret_cast<const float4*>(g.P1 + v * g.ldp + kc);
    }
    mul = live ? m : 0.0f;
}

template <int BM, int BN, int WM, int WN, int AMODE, int KT>
__global__ void __launch_bounds__(WM * WN * 64) gemm_kernel(GemmArgs g) {
    constexpr int NT = WM * WN * 64;       // threads of the workgroup
    constexpr int LDS_STRIDE = KT + 4;
    constexpr int TPR = KT / 4;            // threads that stage one row of a slice
    constexpr int RPP = NT / TPR;          // rows staged per pass
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    constexpr int A_LOADS = BM * KT / 4 / NT;    // float4 per thread per slice
    constexpr int B_LOADS = BN * KT / 4 / NT;
    __shared__ __attribute__((aligned(16))) float As[BM * LDS_STRIDE];
    __shared__ __attribute__((aligned(16))) float Bs[BN * LDS_STRIDE];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int col_base = blockIdx.y * BN;
    const int ldw = g.ldw ? g.ldw : g.K;
    const int64_t M = g.M_dev ? (int64_t)*g.M_dev : g.M;      // rows known only on the device: stride over the tiles
    // the next layer recomputes its aggregates from h when these rows are a large part of the graph: no payload deltas then
    float* const DPout = (g.dp_skip_large && 4 * M > g.n_vertices) ? nullptr : g.DP;
  for (int64_t row_base = (int64_t)blockIdx.x * BM; row_base < M; row_base += (int64_t)gridDim.x * BM) {

    // rows this thread stages
    const int lr = tid / TPR, lk = (tid % TPR) * 4;
    int64_t av[A_LOADS];
    float asc[A_LOADS];
    bool aok[A_LOADS];
#pragma unroll
    for (int p = 0; p < A_LOADS; ++p) {
        const int64_t m = row_base + lr + RPP * p;
        aok[p] = m < M;
        av[p] = aok[p] ? ((g.rows && !g.a_is_compact) ? (int64_t)g.rows[m] : m) : 0;
        asc[p] = 1.0f;
        if (aok[p] && AMODE == A_SCALE_GCN) asc[p] = gcn_scale(g.indeg[av[p]]);
        if (aok[p] && AMODE == A_CONCAT_MEAN && g.indeg) {          // no degree vector: the sum is used as it is
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

    float4 ra[A_LOADS], ra2[two_sources(AMODE) ? A_LOADS : 1], rb[B_LOADS];
    float am[A_LOADS], bmul[B_LOADS];
    auto fetch = [&](int k0) {
#pragma unroll
        for (int p = 0; p < A_LOADS; ++p) load_a<AMODE>(g, av[p], asc[p], k0 + lk, aok[p], ra[p], ra2[two_sources(AMODE) ? p : 0], am[p]);
#pragma unroll
        for (int p = 0; p < B_LOADS; ++p) {
            const int n = col_base + lr + RPP * p;
            const int k = k0 + lk;
            const int nc = n < g.N ? n : g.N - 1, kc = k < g.K ? k : g.K - 4;
            rb[p] = *reinterpret_cast<const float4*>(g.Wt + (int64_t)nc * ldw + kc);
            bmul[p] = (n < g.N && k < g.K) ? 1.0f : 0.0f;
        }
    };

    fetch(0);
    const int half = lane >> 5, l32 = lane & 31;
    for (int k0 = 0; k0 < g.K; k0 += KT) {
#pragma unroll
        for (int p = 0; p < A_LOADS; ++p) {
            float4 t = ra[p];
            if (two_sources(AMODE)) {
                const float4 q = ra2[p];
                t.x = fmaf(g.axpy_c, t.x, q.x); t.y = fmaf(g.axpy_c, t.y, q.y);
                t.z = fmaf(g.axpy_c, t.z, q.z); t.w = fmaf(g.axpy_c, t.w, q.w);
            }
            if (AMODE == A_AXPY_BIAS_RELU) {                 // the slice's k range is k0 + lk .. +3 (clamped like the loads)
                const int kb = k0 + lk < g.K ? k0 + lk : g.K - 4;
                const float4 ab = *reinterpret_cast<const float4*>(g.a_bias + kb);
                t.x = fmaxf(t.x + ab.x, 0.f); t.y = fmaxf(t.y + ab.y, 0.f);
                t.z = fmaxf(t.z + ab.z, 0.f); t.w = fmaxf(t.w + ab.w, 0.f);
            }
            t.x *= am[p]; t.y *= am[p]; t.z *= am[p]; t.w *= am[p];
            *reinterpret_cast<float4*>(&As[(lr + RPP * p) * LDS_STRIDE + lk]) = t;
        }
#pragma unroll
        for (int p = 0; p < B_LOADS; ++p) {
            float4 t = rb[p];
            t.x *= bmul[p]; t.y *= bmul[p]; t.z *= bmul[p]; t.w *= bmul[p];
            *reinterpret_cast<float4*>(&Bs[(lr + RPP * p) * LDS_STRIDE + lk]) = t;
        }
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

    // epilogue = write-back.  All old rows a lane needs are read before anything is stored, so the loads
    // are independent of the stores and stay in flight together.
    float bias[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int n = col_base + (wn * TN + j) * 32 + l32;
        bias[j] = (g.bias && n < g.N) ? g.bias[n] : 0.f;
    }
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int rb = 0; rb < 16; rb += 4) {
            int64_t mrow[4], vrow[4];
            float cn[4], co[4], oldv[4][TN], addv[4][AMODE == A_PLAIN_ADD ? TN : 1];
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                const int r = rb + rr;
                mrow[rr] = row_base + (wm * TM + i) * 32 + 8 * (r / 4) + 4 * half + (r % 4);
                const bool ok = mrow[rr] < M;
                vrow[rr] = ok ? (g.rows ? (int64_t)g.rows[mrow[rr]] : mrow[rr]) : 0;
                cn[rr] = 1.0f; co[rr] = 1.0f;
                if (ok && DPout && g.dp_scale_gcn) { cn[rr] = gcn_scale(g.indeg[vrow[rr]]); co[rr] = gcn_scale(g.indeg_old[vrow[rr]]); }
                float as = 0.f;                                   // scale of the row added before the activation
                if (AMODE == A_PLAIN_ADD && ok) {
                    as = 1.0f;
                    if (g.add_indeg) { const int32_t dg = g.add_indeg[vrow[rr]]; as = dg > 0 ? 1.0f / (float)dg : 0.0f; }
                }
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const int n = col_base + (wn * TN + j) * 32 + l32;
                    const int nc = n < g.N ? n : g.N - 1;
                    if (AMODE == A_PLAIN_ADD) addv[rr][j] = g.add[vrow[rr] * g.N + nc] * as;
                    if (g.H) oldv[rr][j] = DPout ? g.H[vrow[rr] * g.N + nc] : 0.f;   // vrow is 0 for rows past M: always in range
                    else oldv[rr][j] = (DPout && g.dp_no_h == 2) ? DPout[(ok ? mrow[rr] : 0) * g.N + nc] : 0.f;
                }
            }
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                if (mrow[rr] >= M) continue;
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const int n = col_base + (wn * TN + j) * 32 + l32;
                    if (n >= g.N) continue;
                    float y = acc[i][j][rb + rr] + bias[j];
                    if (AMODE == A_PLAIN_ADD) y += addv[rr][j];
                    if (g.act == 1) y = fmaxf(y, 0.f);
                    else if (g.act == 2) y = y > 0.f ? y : expm1f(y);
                    if (g.out_compact && mrow[rr] < g.out_cap) g.out_compact[mrow[rr] * g.N + n] = y;
                    if (g.H) {
                        if (DPout) DPout[mrow[rr] * g.N + n] = g.dp_store_old ? oldv[rr][j] : y * cn[rr] - oldv[rr][j] * co[rr];
                        g.H[vrow[rr] * g.N + n] = y;
                    } else if (DPout) {       // the layer's rows are not kept: the payload delta is built by two launches
                        if (g.dp_no_h == 1) DPout[mrow[rr] * g.N + n] = -y * co[rr];
                        else if (g.dp_no_h == 2) DPout[mrow[rr] * g.N + n] = oldv[rr][j] + y * cn[rr];
                    }
                }
            }
        }
    }
  }
}

// y = act(P0[v] * scale(v) + bias + add[v] / count(v)) with the same write-back as the GEMM's epilogue; scale is the GCN
// normalisation when a degree vector is given, else 1; the added row is optional; a thread owns four columns of a row
__global__ void rowwise_update_kernel(GemmArgs g) {
    const int64_t M = g.M_dev ? (int64_t)*g.M_dev : g.M;
    float* const DPout = (g.dp_skip_large && 4 * M > g.n_vertices) ? nullptr : g.DP;
    const int nq = g.N >> 2;
    const int64_t total = M * nq, stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
        const int64_t m = i / nq;
        const int n = (int)(i - m * nq) << 2;
        const int64_t v = g.rows ? (int64_t)g.rows[m] : m;
        const float sc = g.indeg ? gcn_scale(g.indeg[v]) : 1.0f;
        const float4 x = *reinterpret_cast<const float4*>(g.P0 + v * g.N + n);
        float y[4] = {x.x * sc, x.y * sc, x.z * sc, x.w * sc};
        float ad[4] = {0.f, 0.f, 0.f, 0.f};
        if (g.add) {                      // same order as the GEMM epilogue that this replaces: (product + bias) + added row
            float as = 1.0f;
            if (g.add_indeg) { const int32_t dg = g.add_indeg[v]; as = dg > 0 ? 1.0f / (float)dg : 0.0f; }
            const float4 q = *reinterpret_cast<const float4*>(g.add + v * g.N + n);
            ad[0] = q.x * as; ad[1] = q.y * as; ad[2] = q.z * as; ad[3] = q.w * as;
        }
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            if (g.bias) y[t] += g.bias[n + t];
            if (g.add) y[t] += ad[t];
            if (g.act == 1) y[t] = fmaxf(y[t], 0.f);
            else if (g.act == 2) y[t] = y[t] > 0.f ? y[t] : expm1f(y[t]);
        }
        const float4 yo = make_float4(y[0], y[1], y[2], y[3]);
        if (g.out_compact && m < g.out_cap) *reinterpret_cast<float4*>(g.out_compact + m * g.N + n) = yo;
        if (g.H) {
            if (DPout) {
                const float4 o = *reinterpret_cast<const float4*>(g.H + v * g.N + n);
                float cn = 1.0f, co = 1.0f;
                if (g.dp_scale_gcn) { cn = sc; co = gcn_scale(g.indeg_old[v]); }
                const float4 d = g.dp_store_old ? o : make_float4(yo.x * cn - o.x * co, yo.y * cn - o.y * co, yo.z * cn - o.z * co, yo.w * cn - o.w * co);
                *reinterpret_cast<float4*>(DPout + m * g.N + n) = d;
            }
            *reinterpret_cast<float4*>(g.H + v * g.N + n) = yo;
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

template <int AMODE>
static void launch_gemm(const GemmArgs& g, hipStream_t s) {
    const int BM = g.N > 32 ? 64 : 128;
    int64_t tiles = cdiv(g.M, BM);
    if (g.M_dev && tiles > 4096) tiles = 4096;               // device-sized problem: a fixed grid strides over the tiles
    const unsigned gx = (unsigned)tiles;
    if (g.N > 128) gemm_kernel<64, 256, 2, 4, AMODE, 32><<<dim3(gx, (unsigned)cdiv(g.N, 256)), 512, 0, s>>>(g);
    else if (g.N > 64) gemm_kernel<64, 128, 2, 2, AMODE, 32><<<dim3(gx, 1), 256, 0, s>>>(g);
    else if (g.N > 32) gemm_kernel<64, 64, 2, 2, AMODE, 32><<<dim3(gx, 1), 256, 0, s>>>(g);
    else gemm_kernel<128, 32, 4, 1, AMODE, 32><<<dim3(gx, 1), 256, 0, s>>>(g);
}

nrt_status k_gemm(const GemmArgs& g, hipStream_t s) {
    if (g.M <= 0) return NRT_OK;
    if (g.K % 4 || g.ldp % 4 || g.ldw % 4) { nrt_set_error("gemm: widths must be multiples of 4"); return NRT_ERR_UNSUPPORTED; }
    switch (g.a_mode) {
    case A_PLAIN: launch_gemm<A_PLAIN>(g, s); break;
    case A_SCALE_GCN: launch_gemm<A_SCALE_GCN>(g, s); break;
    case A_CONCAT_MEAN: launch_gemm<A_CONCAT_MEAN>(g, s); break;
    case A_PLAIN_ADD:
        if (!g.add) { nrt_set_error("gemm: the added rows are missing"); return NRT_ERR_INVALID_ARG; }
        launch_gemm<A_PLAIN_ADD>(g, s);
        break;
    case A_AXPY_BIAS_RELU:
        if (!g.a_bias) { nrt_set_error("gemm: the operand bias is missing"); return NRT_ERR_INVALID_ARG; }
        launch_gemm<A_AXPY_BIAS_RELU>(g, s);
        break;
    default: launch_gemm<A_AXPY>(g, s); break;
    }
    LAUNCH_CHECK();
    return NRT_OK;
}

nrt_status k_rowwise_update(const GemmArgs& g, hipStream_t s) {
    if (g.M <= 0) return NRT_OK;
    if (g.N % 4 || !g.P0 || (!g.indeg && !g.add)) { nrt_set_error("rowwise update: bad arguments"); return NRT_ERR_INVALID_ARG; }
    int64_t blocks = cdiv(g.M * (g.N / 4), 256);
    if (blocks > 8192) blocks = 8192;
    rowwise_update_kernel<<<(unsigned)blocks, 256, 0, s>>>(g);
    LAUNCH_CHECK();
    return NRT_OK;
}

nrt_status k_transpose(const float* W, float* Wt, int K, int N, hipStream_t s) {
    transpose_kernel<<<(int)cdiv((int64_t)K * N, 256), 256, 0, s>>>(W, Wt, K, N);
    LAUNCH_CHECK();
    return NRT_OK;
}
