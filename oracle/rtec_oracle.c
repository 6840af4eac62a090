/*
 * CPU oracle primitives, fp64.  TEST INFRASTRUCTURE ONLY: nothing on the product path
 * links or calls this file; it shares no code with the HIP kernels.
 *
 * Two per-destination neighbourhood reductions, written as the plain definitions:
 *
 *  orc_in_sum      a_v = sum over in-edges <u,v> of coef_uv * p_u
 *                  (the AGG step of the message-aggregate-update layer, Eq. 1, with a
 *                  sum aggregator; GCN Eq. 2, GraphSAGE and GIN all reduce to it once the
 *                  per-source payload p_u and per-edge coefficient are chosen by the caller)
 *
 *  orc_gat_attend  o_v = sum_u softmax_u(LeakyReLU(ad_v + as_u)) * z_u over u in N(v) U {v}
 *                  (GAT attention Eq. 3 and aggregation Eq. 4; Algorithm 2),
 *                  evaluated with the usual max-subtracted softmax, which is the same
 *                  function as the raw exp / sum form the paper prints.
 *
 * Edges come as an unordered list (src[e], dst[e]); each routine groups them by destination
 * with a counting sort of its own and then loops over destinations.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static int group_by_dst(int64_t n, int64_t e, const int32_t *dst, int64_t **start_out, int64_t **order_out)
{
    int64_t *start = (int64_t *)calloc((size_t)n + 1, sizeof(int64_t));
    int64_t *order = (int64_t *)malloc((size_t)(e > 0 ? e : 1) * sizeof(int64_t));
    int64_t *cursor = (int64_t *)malloc((size_t)(n > 0 ? n : 1) * sizeof(int64_t));
    if (!start || !order || !cursor) { free(start); free(order); free(cursor); return -1; }
    for (int64_t i = 0; i < e; ++i) start[dst[i] + 1] += 1;
    for (int64_t v = 0; v < n; ++v) start[v + 1] += start[v];
    memcpy(cursor, start, (size_t)n * sizeof(int64_t));
    for (int64_t i = 0; i < e; ++i) order[cursor[dst[i]]++] = i;
    free(cursor);
    *start_out = start;
    *order_out = order;
    return 0;
}

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* out[v][:] = sum_{e : dst[e] = v} (coef ? coef[e] : 1) * payload[src[e]][:] ; rows have d doubles. */
int orc_in_sum(int64_t n, int64_t e, const int32_t *src, const int32_t *dst, const double *coef,
               int64_t d, const double *payload, double *out)
{
    int64_t *start, *order;
    if (group_by_dst(n, e, dst, &start, &order)) return -1;
#pragma omp parallel for schedule(dynamic, 256)
    for (int64_t v = 0; v < n; ++v) {
        double *acc = out + v * d;
        for (int64_t k = 0; k < d; ++k) acc[k] = 0.0;
        for (int64_t j = start[v]; j < start[v + 1]; ++j) {
            int64_t ed = order[j];
            double c = coef ? coef[ed] : 1.0;
            const double *row = payload + (int64_t)src[ed] * d;
            for (int64_t k = 0; k < d; ++k) acc[k] += c * row[k];
        }
    }
    free(start);
    free(order);
    return 0;
}

/*
 * z: [n][heads*hd], as/ad: [n][heads], out: [n][heads*hd].
 * For every destination v and head k, over u in N(v) U {v}:
 *   e_uv = LeakyReLU_slope(ad[v][k] + as[u][k]);  alpha = softmax_u(e_uv);  out[v][k] = sum alpha * z[u][k].
 */
int orc_gat_attend(int64_t n, int64_t e, const int32_t *src, const int32_t *dst, int64_t heads, int64_t hd,
                   const double *z, const double *as, const double *ad, double slope, double *out)
{
    int64_t *start, *order;
    if (group_by_dst(n, e, dst, &start, &order)) return -1;
    const int64_t d = heads * hd;
#pragma omp parallel for schedule(dynamic, 256)
    for (int64_t v = 0; v < n; ++v) {
        for (int64_t k = 0; k < heads; ++k) {
            double self = ad[v * heads + k] + as[v * heads + k];
            self = self > 0 ? self : slope * self;
            double mx = self;
            for (int64_t j = start[v]; j < start[v + 1]; ++j) {
                int64_t u = src[order[j]];
                double lg = ad[v * heads + k] + as[u * heads + k];
                lg = lg > 0 ? lg : slope * lg;
                if (lg > mx) mx = lg;
            }
            double den = exp(self - mx);
            double *acc = out + v * d + k * hd;
            for (int64_t c = 0; c < hd; ++c) acc[c] = den * z[v * d + k * hd + c];
            for (int64_t j = start[v]; j < start[v + 1]; ++j) {
                int64_t u = src[order[j]];
                double lg = ad[v * heads + k] + as[u * heads + k];
                lg = lg > 0 ? lg : slope * lg;
                double wgt = exp(lg - mx);
                den += wgt;
                const double *row = z + u * d + k * hd;
                for (int64_t c = 0; c < hd; ++c) acc[c] += wgt * row[c];
            }
            for (int64_t c = 0; c < hd; ++c) acc[c] /= den;
        }
    }
    free(start);
    free(order);
    return 0;
}
