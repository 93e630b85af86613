/*
 * CollectiveKV prefill-stage oracle: TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, fp64 CPU statement of what the prefill stage of CollectiveKV caches
 * (paper section 4.2 "In the prefill stage": the linear projection to the user-specific
 * K/V, and section 4.3 "CollectiveKV Router": the routing map M = S W_r + b_r and the
 * index I[i] = argmax_j M[i][j]).  Only the inference form is written here; the sigmoid
 * weighting and the two router losses exist only in training.
 * Nothing in the product path may call this file, and it shares no code, header or table
 * with the HIP library.
 *
 * Data (T positions, users back to back; H heads; the embedding S is shared by the heads,
 * every head has its own projection, router and pool):
 *   S            [T][d_e]          history embedding
 *   w_rk, w_rv   [H][P][d_e]       router weights, one row per pool entry: row j of head h
 *                                  holds column j of that head's W_r (section 4.3)
 *   b_rk, b_rv   [H][P]   float    router bias b_r
 *   w_k, w_v     [H][d_u][d_e]     projection weights, row c holds column c of W_k (W_v)
 *   b_k, b_v     [H][d_u] float    projection bias
 *   idx_k, idx_v [T][H]   int32    out: I_k, I_v, 0-based; equal maxima give the lowest j
 *   user_k, user_v [T][H][d_u] double  out: K_u, V_u, unrounded
 * S and the weights are fp32 (dtype 0) or bfloat16 bit patterns (dtype 1); the biases are
 * always fp32.  Everything widens to fp64 exactly and is accumulated in fp64, with the
 * bias added last.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static double widen_p(const void *base, int64_t i, int dtype)
{
    if (dtype == 0)
        return (double)((const float *)base)[i];
    uint32_t bits = (uint32_t)((const uint16_t *)base)[i] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/* M[i][j] of one head: s . (row j of w_r) + b_r[j]   (section 4.3, first equation) */
static double route_score(const double *s, const void *w_r, const float *b_r, int h, int j,
                          int P, int d_e, int dtype)
{
    double m = 0.0;
    const int64_t row = ((int64_t)h * P + j) * d_e;
    for (int c = 0; c < d_e; ++c)
        m += s[c] * widen_p(w_r, row + c, dtype);
    return m + (double)b_r[(int64_t)h * P + j];
}

/* I[i] = argmax_j M[i][j]; the first (lowest) j among equal maxima */
static int32_t route(const double *s, const void *w_r, const float *b_r, int h, int P, int d_e, int dtype)
{
    int32_t best = 0;
    double best_m = route_score(s, w_r, b_r, h, 0, P, d_e, dtype);
    for (int j = 1; j < P; ++j) {
        const double m = route_score(s, w_r, b_r, h, j, P, d_e, dtype);
        if (m > best_m) { best_m = m; best = j; }
    }
    return best;
}

/* K_u[i][c] = s . (row c of w) + b[c]   (section 4.2, first equation) */
static void project(double *dst, const double *s, const void *w, const float *b, int h,
                    int d_u, int d_e, int dtype)
{
    for (int c = 0; c < d_u; ++c) {
        double a = 0.0;
        const int64_t row = ((int64_t)h * d_u + c) * d_e;
        for (int e = 0; e < d_e; ++e)
            a += s[e] * widen_p(w, row + e, dtype);
        dst[c] = a + (double)b[(int64_t)h * d_u + c];
    }
}

/* What the prefill stage caches for T positions.  The two sides have their own sizes (sharing only
 * keys or only values, ablation "sharing keys or values": the ordinary side has no router, P = 0,
 * and all its d_a columns come from the projection): P_k, P_v pool entries and d_uk, d_uv
 * projected columns.  P = 0: that side's indices are not written; d_u = 0: no user slice.
 * user_k is [T][H][d_uk], user_v [T][H][d_uv].  Returns 0, or -1 on a bad argument. */
int ckv_oracle_prefill(int H, int d_e, int d_uk, int d_uv, int P_k, int P_v, int dtype, int64_t T, const void *S,
                       const void *w_rk, const float *b_rk, const void *w_rv, const float *b_rv,
                       const void *w_k, const float *b_k, const void *w_v, const float *b_v,
                       int32_t *idx_k, int32_t *idx_v, double *user_k, double *user_v)
{
    if (H < 1 || d_e < 1 || d_uk < 0 || d_uv < 0 || P_k < 0 || P_v < 0 || T < 0 || (dtype != 0 && dtype != 1))
        return -1;
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t t = 0; t < T; ++t) {
        double *s = (double *)malloc(sizeof(double) * (size_t)d_e);
        for (int c = 0; c < d_e; ++c) s[c] = widen_p(S, t * d_e + c, dtype);
        for (int h = 0; h < H; ++h) {
            if (P_k > 0) idx_k[t * H + h] = route(s, w_rk, b_rk, h, P_k, d_e, dtype);
            if (P_v > 0) idx_v[t * H + h] = route(s, w_rv, b_rv, h, P_v, d_e, dtype);
            if (d_uk > 0) project(user_k + (t * H + h) * (int64_t)d_uk, s, w_k, b_k, h, d_uk, d_e, dtype);
            if (d_uv > 0) project(user_v + (t * H + h) * (int64_t)d_uv, s, w_v, b_v, h, d_uv, d_e, dtype);
        }
        free(s);
    }
    return 0;
}

/*
 * How far a candidate routing decision is from the maximum of its row of the routing map:
 *   gap[t][h] = max_j M[t][j] - M[t][cand[t][h]]   (>= 0, and 0 exactly when cand attains the maximum)
 *   mag[t][h] = sum_c |s_c * w_r[cand][c]| + |b_r[cand]|   (size of the terms behind M[t][cand])
 * An implementation that forms M in lower precision may pick a different entry than the fp64
 * argmax when two entries are closer than its rounding error; such a pick is still correct in
 * that precision, and the test that compares indices bounds gap by a multiple of mag instead.
 * Returns 0, or -1 on a bad argument (a candidate outside [0, P)).
 */
int ckv_oracle_router_gap(int H, int d_e, int P, int dtype, int64_t T, const void *S,
                          const void *w_r, const float *b_r, const int32_t *cand,
                          double *gap, double *mag)
{
    if (H < 1 || d_e < 1 || P < 1 || T < 0 || (dtype != 0 && dtype != 1))
        return -1;
    for (int64_t i = 0; i < T * H; ++i)
        if (cand[i] < 0 || cand[i] >= P) return -1;
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t t = 0; t < T; ++t) {
        double *s = (double *)malloc(sizeof(double) * (size_t)d_e);
        for (int c = 0; c < d_e; ++c) s[c] = widen_p(S, t * d_e + c, dtype);
        for (int h = 0; h < H; ++h) {
            const int32_t best = route(s, w_r, b_r, h, P, d_e, dtype);
            const int32_t c0 = cand[t * H + h];
            gap[t * H + h] = route_score(s, w_r, b_r, h, best, P, d_e, dtype) -
                             route_score(s, w_r, b_r, h, c0, P, d_e, dtype);
            double a = fabs((double)b_r[(int64_t)h * P + c0]);
            const int64_t row = ((int64_t)h * P + c0) * d_e;
            for (int c = 0; c < d_e; ++c) a += fabs(s[c] * widen_p(w_r, row + c, dtype));
            mag[t * H + h] = a;
        }
        free(s);
    }
    return 0;
}
