/*
 * CollectiveKV decode-stage oracle: TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, fp64 CPU statement of what the decode stage of CollectiveKV computes
 * (paper section 4.2 "In the decode stage", equations labelled "eq: Kc" and "eq: K",
 * and the appendix "Discussion of the sharing mechanism" for the column order).
 * It exists so that tests, the smoke check and the benchmark's cpu_baseline leg have
 * something independent to compare the GPU library with.  Nothing in the product
 * path may call it, and it shares no code, header or table with the HIP library.
 *
 * Data as the paper states the problem, one record per user, users back to back:
 *   lengths[B]                 n of each user (history length), n >= 0
 *   idx_k, idx_v  [T][H]       I_k, I_v: 0-based pool row of position t, head h;  T = sum(lengths)
 *   user_k, user_v [T][H][d_u] K_u, V_u: the user-specific slices ([T][H][d_a] for a side that is
 *                              not shared, see side_dims below)
 *   pool_k, pool_v [H][P][pool_ld]   P_k, P_v: one pool per head, d_g valid columns per row
 *   q   [B][H][Nq][d_a]        candidate queries, d_a = d_u + d_g
 *   out [B][H][Nq][d_a]        fp64
 * Stored values are fp32 (dtype 0) or bfloat16 bit patterns in uint16 (dtype 1).  Both
 * widen to fp64 exactly; no intermediate is ever rounded below fp64.
 *
 * The paper fixes gather and concat but not the attention form; the two forms below are
 * the ones the workloads name: softmax(scale * q.K^T) V and SiLU(scale * q.K^T) V / n,
 * non-causal over the user's whole history.  A user with n = 0 gets out = 0.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };
enum { ORACLE_SOFTMAX = 0, ORACLE_SILU_OVER_N = 1 };

static double widen(const void *base, int64_t i, int dtype)
{
    if (dtype == ORACLE_F32)
        return (double)((const float *)base)[i];
    /* bfloat16 is the upper half of an IEEE binary32 */
    uint32_t bits = (uint32_t)((const uint16_t *)base)[i] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

static size_t elem_size(int dtype) { return dtype == ORACLE_F32 ? 4u : 2u; }

/*
 * Sharing only one side (ablation "sharing keys or values": CollectiveK shares only the keys,
 * CollectiveV only the values).  share = 0: both sides are [user slice | pool row]; 1: only K is,
 * V is the ordinary cache; 2: only V is.  The ordinary (unshared) side keeps all d_a columns per
 * position in its user array and has no index and no pool: d_u' = d_a, d_g' = 0.
 * side: 0 = K, 1 = V.
 */
enum { ORACLE_SHARE_KV = 0, ORACLE_SHARE_K = 1, ORACLE_SHARE_V = 2 };
static void side_dims(int share, int side, int d_u, int d_g, int *du, int *dg)
{
    const int shared = share == ORACLE_SHARE_KV || (share == ORACLE_SHARE_K && side == 0) ||
                       (share == ORACLE_SHARE_V && side == 1);
    *du = shared ? d_u : d_u + d_g;
    *dg = shared ? d_g : 0;
}

/*
 * Final K row (or V row) of one position and head, widened to fp64:
 *   row[0 : d_u]     = user slice          (user-specific dimensions come first)
 *   row[d_u : d_a]   = pool[h][index]      (collective part, gathered by the stored index)
 * Section 4.2, eq. "eq: Kc" (gather) then eq. "eq: K" (concat).
 */
static void final_row(double *row, const void *user, const void *pool, const int32_t *idx,
                      int64_t t, int h, int H, int d_u, int d_g, int P, int64_t pool_ld, int dtype)
{
    for (int c = 0; c < d_u; ++c)
        row[c] = widen(user, (t * H + h) * (int64_t)d_u + c, dtype);
    if (d_g > 0) {
        int64_t r = idx[t * H + h];
        for (int c = 0; c < d_g; ++c)
            row[d_u + c] = widen(pool, ((int64_t)h * P + r) * pool_ld + c, dtype);
    }
}

/*
 * Attention outputs of the listed users.  users[] holds n_users user numbers (or NULL for
 * all B users in order); rows of out that belong to other users are not touched.
 * rss (same shape as out, or NULL) receives, for every output element c, the scale against which a
 * rounding error of the weights shows in that element: the positions are grouped by the value of
 * their weight (equal weights are rounded alike, so their errors add up coherently; different
 * weights err independently), and rss[c] = sqrt(sum over groups g of (sum_{i in g} w_i V_i[c])^2).
 * With all weights different this is the root-sum-square of the summands w_i V_i[c]; with all
 * weights equal it is |out[c]|.
 * sss (same shape, or NULL; needs rss) receives the scale against which a rounding error of the scores
 * shows: a score s_i = scale q . K_i summed in finite precision is off by some delta_i times
 * A_i = |scale| sum_k |q_k K_ik|, and to first order the output moves by
 *   softmax:   sum_i w_i (V_i[c] - out[c]) A_i delta_i      (d w_i = w_i (d s_i - sum_j w_j d s_j))
 *   SiLU / n:  sum_i f'(s_i) V_i[c] A_i delta_i / n,        f(s) = s sigma(s), f'(s) = sigma(s) (1 + s (1 - sigma(s)))
 * with the same grouping (equal rows have equal scores and equal errors, different rows err
 * independently): sss[c] = sqrt(sum over groups of (sum_{i in g} coefficient_i)^2).
 * acs (same shape, or NULL; needs rss) receives the scale against which the rounding of the additions of
 * out[c] = sum_i w_i V_i[c] shows when they are carried out in single precision in an order the oracle does
 * not know: sqrt(n) * (|out[c]| + sqrt(sum_i (w_i V_i[c])^2)), the positions taken one by one (a partial sum of
 * k of the n summands in an order unrelated to their values has mean (k/n) out[c] and a spread of at most the
 * root-sum-square of all summands, and there are n - 1 additions).
 * asum (same shape, or NULL) receives sum_i |w_i V_i[c]|: whatever the weights are rounded to, with a relative error of at
 * most u each, out[c] moves by at most u asum[c]; weights that are nearly equal (positions that share their key row up to a
 * narrow user slice) are rounded the same way, and then the errors add up like that and not like independent ones.
 * All four are extra outputs for the comparison rule of the tests; out does not depend on them.
 * Returns 0, or -1 on a bad argument (index outside [0,P), negative length, unknown mode).
 */
struct weighted { double w; int i; };
static int by_weight(const void *a, const void *b)
{
    const double x = ((const struct weighted *)a)->w, y = ((const struct weighted *)b)->w;
    return x < y ? -1 : (x > y ? 1 : 0);
}

static int attend_impl(int B, int H, int d_g, int d_u, int P, int Nq, int dtype, int mode, int share,
                       double scale, int64_t pool_ld,
                       const int32_t *lengths, const int32_t *idx_k, const int32_t *idx_v,
                       const void *user_k, const void *user_v,
                       const void *pool_k, const void *pool_v, const void *q,
                       double *out, double *rss, double *sss, double *acs, double *asum, const int32_t *users, int n_users)
{
    const int d_a = d_u + d_g;
    if (B < 0 || H < 1 || d_g < 0 || d_u < 0 || d_a < 1 || Nq < 1 || pool_ld < d_g)
        return -1;
    if (mode != ORACLE_SOFTMAX && mode != ORACLE_SILU_OVER_N)
        return -1;
    if (share < 0 || share > 2)
        return -1;
    int duk, dgk, duv, dgv;
    side_dims(share, 0, d_u, d_g, &duk, &dgk);
    side_dims(share, 1, d_u, d_g, &duv, &dgv);
    int64_t *offset = (int64_t *)malloc(sizeof(int64_t) * (size_t)(B + 1));
    offset[0] = 0;
    for (int b = 0; b < B; ++b) {
        if (lengths[b] < 0) { free(offset); return -1; }
        offset[b + 1] = offset[b] + lengths[b];
    }
    for (int64_t i = 0; i < offset[B] * H; ++i)
        if ((dgk > 0 && (idx_k[i] < 0 || idx_k[i] >= P)) || (dgv > 0 && (idx_v[i] < 0 || idx_v[i] >= P))) {
            free(offset);
            return -1;
        }
    if (!users) n_users = B;

    int bad = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int u = 0; u < n_users; ++u) {
        for (int h = 0; h < H; ++h) {
            const int b = users ? users[u] : u;
            if (b < 0 || b >= B) { bad = 1; continue; }
            const int n = lengths[b];
            const int64_t o = offset[b];
            double *K = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1) * d_a);
            double *V = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1) * d_a);
            double *w = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
            double *sc = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));  /* scores, and A_i (see above) */
            double *sa = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
            double *qv = (double *)malloc(sizeof(double) * (size_t)d_a);
            /* gather + concat: the user's final K and V, n x d_a */
            for (int i = 0; i < n; ++i) {
                final_row(K + (int64_t)i * d_a, user_k, pool_k, idx_k, o + i, h, H, duk, dgk, P, pool_ld, dtype);
                final_row(V + (int64_t)i * d_a, user_v, pool_v, idx_v, o + i, h, H, duv, dgv, P, pool_ld, dtype);
            }
            for (int j = 0; j < Nq; ++j) {
                const int64_t qo = (((int64_t)b * H + h) * Nq + j) * d_a;
                for (int c = 0; c < d_a; ++c) qv[c] = widen(q, qo + c, dtype);
                /* scores s_i = scale * q . K_i */
                for (int i = 0; i < n; ++i) {
                    double s = 0.0, m = 0.0;
                    for (int c = 0; c < d_a; ++c) {
                        s += qv[c] * K[(int64_t)i * d_a + c];
                        m += fabs(qv[c] * K[(int64_t)i * d_a + c]);
                    }
                    w[i] = sc[i] = scale * s;
                    sa[i] = fabs(scale) * m;
                }
                /* weights */
                if (mode == ORACLE_SOFTMAX) {
                    double m = -INFINITY, z = 0.0;
                    for (int i = 0; i < n; ++i) if (w[i] > m) m = w[i];
                    for (int i = 0; i < n; ++i) { w[i] = exp(w[i] - m); z += w[i]; }
                    for (int i = 0; i < n; ++i) w[i] /= z;
                } else {
                    for (int i = 0; i < n; ++i) w[i] = w[i] / (1.0 + exp(-w[i])) / (double)n;
                }
                /* out_j = sum_i w_i V_i */
                for (int c = 0; c < d_a; ++c) {
                    double a = 0.0;
                    for (int i = 0; i < n; ++i) a += w[i] * V[(int64_t)i * d_a + c];
                    out[qo + c] = a;
                }
                if (rss) {
                    /* positions in order of their weight, so that equal weights are neighbours */
                    struct weighted *ord = (struct weighted *)malloc(sizeof(struct weighted) * (size_t)(n > 0 ? n : 1));
                    for (int i = 0; i < n; ++i) { ord[i].w = w[i]; ord[i].i = i; }
                    qsort(ord, (size_t)n, sizeof ord[0], by_weight);
                    for (int c = 0; c < d_a; ++c) {
                        double a2 = 0.0, group = 0.0;
                        for (int k = 0; k < n; ++k) {
                            group += ord[k].w * V[(int64_t)ord[k].i * d_a + c];
                            if (k + 1 == n || ord[k + 1].w != ord[k].w) {  /* the group ends here */
                                a2 += group * group;
                                group = 0.0;
                            }
                        }
                        rss[qo + c] = sqrt(a2);
                    }
                    if (sss) {
                        /* coefficient of delta_i without V: w_i A_i (softmax), f'(s_i) A_i / n (SiLU) */
                        for (int i = 0; i < n; ++i) {
                            if (mode == ORACLE_SOFTMAX) {
                                sa[i] *= w[i];
                            } else {
                                const double sg = 1.0 / (1.0 + exp(-sc[i]));
                                sa[i] *= sg * (1.0 + sc[i] * (1.0 - sg)) / (double)n;
                            }
                        }
                        for (int c = 0; c < d_a; ++c) {
                            const double centre = mode == ORACLE_SOFTMAX ? out[qo + c] : 0.0;
                            double a2 = 0.0, group = 0.0;
                            for (int k = 0; k < n; ++k) {
                                group += sa[ord[k].i] * (V[(int64_t)ord[k].i * d_a + c] - centre);
                                if (k + 1 == n || ord[k + 1].w != ord[k].w) {
                                    a2 += group * group;
                                    group = 0.0;
                                }
                            }
                            sss[qo + c] = sqrt(a2);
                        }
                    }
                    free(ord);
                }
                if (acs) {
                    for (int c = 0; c < d_a; ++c) {
                        double a2 = 0.0;
                        for (int i = 0; i < n; ++i) {
                            const double t = w[i] * V[(int64_t)i * d_a + c];
                            a2 += t * t;
                        }
                        acs[qo + c] = sqrt((double)n) * (fabs(out[qo + c]) + sqrt(a2));
                    }
                }
                if (asum) {
                    for (int c = 0; c < d_a; ++c) {
                        double a1 = 0.0;
                        for (int i = 0; i < n; ++i) a1 += fabs(w[i] * V[(int64_t)i * d_a + c]);
                        asum[qo + c] = a1;
                    }
                }
            }
            free(K); free(V); free(w); free(sc); free(sa); free(qv);
        }
    }
    free(offset);
    return bad ? -1 : 0;
}

int ckv_oracle_attend(int B, int H, int d_g, int d_u, int P, int Nq, int dtype, int mode, int share,
                      double scale, int64_t pool_ld,
                      const int32_t *lengths, const int32_t *idx_k, const int32_t *idx_v,
                      const void *user_k, const void *user_v,
                      const void *pool_k, const void *pool_v, const void *q,
                      double *out, const int32_t *users, int n_users)
{
    return attend_impl(B, H, d_g, d_u, P, Nq, dtype, mode, share, scale, pool_ld, lengths, idx_k, idx_v, user_k, user_v,
                       pool_k, pool_v, q, out, NULL, NULL, NULL, NULL, users, n_users);
}

/* The same, and the root-sum-square of every element's summands in rss (see above). */
int ckv_oracle_attend_rss(int B, int H, int d_g, int d_u, int P, int Nq, int dtype, int mode, int share,
                          double scale, int64_t pool_ld,
                          const int32_t *lengths, const int32_t *idx_k, const int32_t *idx_v,
                          const void *user_k, const void *user_v,
                          const void *pool_k, const void *pool_v, const void *q,
                          double *out, double *rss, const int32_t *users, int n_users)
{
    return attend_impl(B, H, d_g, d_u, P, Nq, dtype, mode, share, scale, pool_ld, lengths, idx_k, idx_v, user_k, user_v,
                       pool_k, pool_v, q, out, rss, NULL, NULL, NULL, users, n_users);
}

/* The same, and the scale of the scores' rounding errors in sss, of the single-precision additions in acs and the sum of the
 * summands' magnitudes in asum (see above; acs and asum may be NULL). */
int ckv_oracle_attend_scales(int B, int H, int d_g, int d_u, int P, int Nq, int dtype, int mode, int share,
                             double scale, int64_t pool_ld,
                             const int32_t *lengths, const int32_t *idx_k, const int32_t *idx_v,
                             const void *user_k, const void *user_v,
                             const void *pool_k, const void *pool_v, const void *q,
                             double *out, double *rss, double *sss, double *acs, double *asum, const int32_t *users, int n_users)
{
    return attend_impl(B, H, d_g, d_u, P, Nq, dtype, mode, share, scale, pool_ld, lengths, idx_k, idx_v, user_k, user_v,
                       pool_k, pool_v, q, out, rss, sss, acs, asum, users, n_users);
}

/*
 * The final K and V rows themselves, in the storage dtype, [T][H][d_a]: a byte-for-byte
 * copy of the user slice followed by the gathered pool row (no arithmetic).
 */
int ckv_oracle_reconstruct(int H, int d_g, int d_u, int P, int dtype, int share, int64_t pool_ld, int64_t T,
                           const int32_t *idx_k, const int32_t *idx_v,
                           const void *user_k, const void *user_v,
                           const void *pool_k, const void *pool_v,
                           void *k_full, void *v_full)
{
    const size_t e = elem_size(dtype);
    const int d_a = d_u + d_g;
    if (share < 0 || share > 2)
        return -1;
    for (int side = 0; side < 2; ++side) {
        int du, dg;
        side_dims(share, side, d_u, d_g, &du, &dg);
        const int32_t *idx = side == 0 ? idx_k : idx_v;
        const char *user = (const char *)(side == 0 ? user_k : user_v);
        const char *pool = (const char *)(side == 0 ? pool_k : pool_v);
        char *full = (char *)(side == 0 ? k_full : v_full);
        for (int64_t t = 0; t < T; ++t)
            for (int h = 0; h < H; ++h) {
                const int64_t ph = t * H + h;
                char *dst = full + (size_t)ph * d_a * e;
                memcpy(dst, user + (size_t)ph * du * e, (size_t)du * e);
                if (dg > 0) {
                    if (idx[ph] < 0 || idx[ph] >= P)
                        return -1;
                    memcpy(dst + (size_t)du * e, pool + (((size_t)h * P + idx[ph]) * pool_ld) * e, (size_t)dg * e);
                }
            }
    }
    return 0;
}

/*
 * Cache-size accounting (section 5.1 "Metrics": the CollectiveKV cache is the global KV
 * indices plus the user-specific KV; section 4.4 counts one index as one element:
 * the load is s*d_u + s).  Counts are per K and V together, over T positions and H heads.
 *   stored_elems = T*H*2*(d_u + 1)       full_elems = T*H*2*d_a
 *   stored_bytes = T*H*2*(d_u*e + index_bytes)   full_bytes = T*H*2*d_a*e
 * With only one side shared the other side contributes its full d_a columns and no index.
 */
void ckv_oracle_cache_size(int64_t T, int H, int d_g, int d_u, int dtype, int index_bytes, int share,
                           int64_t *stored_elems, int64_t *full_elems,
                           int64_t *stored_bytes, int64_t *full_bytes)
{
    const int64_t e = (int64_t)elem_size(dtype);
    const int64_t ph = T * H;
    *stored_elems = 0;
    *stored_bytes = 0;
    for (int side = 0; side < 2; ++side) {
        int du, dg;
        side_dims(share, side, d_u, d_g, &du, &dg);
        /* a shared side stores its user slice and one index; an ordinary side stores d_a columns */
        *stored_elems += ph * ((int64_t)du + (dg > 0 ? 1 : 0));
        *stored_bytes += ph * ((int64_t)du * e + (dg > 0 ? index_bytes : 0));
    }
    *full_elems = ph * 2 * ((int64_t)d_u + d_g);
    *full_bytes = ph * 2 * ((int64_t)d_u + d_g) * e;
}

/* Number of threads the (user, head) loop may use from now on (n >= 1; without OpenMP nothing changes). */
void ckv_oracle_set_threads(int n)
{
#ifdef _OPENMP
    extern void omp_set_num_threads(int);
    if (n >= 1) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

int ckv_oracle_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
