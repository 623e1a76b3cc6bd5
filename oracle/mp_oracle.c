/*
 * mp_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, double-precision CPU statement of what the Multipole Attention decode path
 * computes, written from the paper's definitions (Sec. 3.1 Eq. 1, Sec. 3.2 Eq. 2, Sec. 3.3,
 * Sec. 3.4).  It shares nothing with the GPU library: no headers, no helpers, no tables.  Only
 * tests, the smoke check and the benchmark's cpu_baseline leg may call it.
 *
 * Everything is fp64, loops are written in the order of the definitions, and there is no
 * blocking, fusion or reordering.  Compile with -O2 -ffp-contract=off.
 *
 * Conventions
 *   - one "unit" = one (sequence, KV head); it owns n clustered tokens, Cf fine clusters and
 *     (two-level only) Cc coarse clusters; G query heads share the unit (grouped-query attention).
 *   - all matrices are row-major, d = head dimension.
 *   - `scale` multiplies every q.k and q.centroid product (the paper writes exp(q Kc^T) with the
 *     query taken as pre-scaled; here the 1/sqrt(d) factor is explicit).
 *   - clusters with N = 0 do not exist for ranking or for Eq. 2.
 *
 * Pins: see tests/test_oracle_*.py.  Readings of the paper that no passage fixes (budget rule at
 * cluster granularity, fine-level normaliser, rank key in the log domain) are "parity unpinned"
 * by the paper itself; they are pinned only through the invariants listed in those tests.
 */
#define _GNU_SOURCE
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double dot(const double *a, const double *b, int d)
{
    double s = 0.0;
    for (int i = 0; i < d; ++i) s += a[i] * b[i];
    return s;
}

/* ---------------------------------------------------------------------------------------------
 * Textbook softmax attention for G query rows over n keys (the quantity Eq. 1 / Eq. 2
 * approximate).  out[h] = sum_t softmax_t(scale * q_h.k_t) v_t ; lse[h] = log sum_t exp(...).
 * n == 0 gives out = 0 and lse = -inf.
 * ------------------------------------------------------------------------------------------- */
void mpo_full_attention(const double *q, const double *K, const double *V, int G, int n, int d,
                        double scale, double *out, double *lse)
{
    double *t = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
    for (int h = 0; h < G; ++h) {
        double m = -INFINITY;
        for (int i = 0; i < n; ++i) {
            t[i] = scale * dot(q + (size_t)h * d, K + (size_t)i * d, d);
            if (t[i] > m) m = t[i];
        }
        double den = 0.0;
        for (int j = 0; j < d; ++j) out[(size_t)h * d + j] = 0.0;
        for (int i = 0; i < n; ++i) {
            double w = exp(t[i] - m);
            den += w;
            for (int j = 0; j < d; ++j) out[(size_t)h * d + j] += w * V[(size_t)i * d + j];
        }
        if (n > 0)
            for (int j = 0; j < d; ++j) out[(size_t)h * d + j] /= den;
        if (lse) lse[h] = (n > 0) ? m + log(den) : -INFINITY;
    }
    free(t);
}

/* ---------------------------------------------------------------------------------------------
 * Ranking and budgeted selection (Sec. 3.1, paragraph after Eq. 1: clusters are ordered by their
 * centroid score and kept, best first, while the token budget allows).
 *
 * Order: higher rank key first, equal keys -> lower cluster index first.  Whole clusters only:
 * walk the order, add a cluster while the running token count stays <= budget, stop at the first
 * one that does not fit.
 * ------------------------------------------------------------------------------------------- */
typedef struct { double r; int32_t idx; } rank_item;

static int rank_cmp(const void *pa, const void *pb)
{
    const rank_item *a = (const rank_item *)pa, *b = (const rank_item *)pb;
    if (a->r > b->r) return -1;
    if (a->r < b->r) return 1;
    return (a->idx > b->idx) - (a->idx < b->idx);
}

/* ids[0..m): the clusters that take part; r[id], N[id] indexed by cluster id; mark[id] set to 1
 * for the retained ones (mark must be zeroed by the caller).  Returns retained token count. */
static int64_t budget_select(const int32_t *ids, int m, const double *r, const int32_t *N,
                             int64_t budget, uint8_t *mark)
{
    rank_item *it = (rank_item *)malloc(sizeof(rank_item) * (size_t)(m > 0 ? m : 1));
    for (int i = 0; i < m; ++i) { it[i].r = r[ids[i]]; it[i].idx = ids[i]; }
    qsort(it, (size_t)m, sizeof(rank_item), rank_cmp);
    int64_t used = 0;
    for (int i = 0; i < m; ++i) {
        int64_t nn = N[it[i].idx];
        if (used + nn > budget) break;
        used += nn;
        mark[it[i].idx] = 1;
    }
    free(it);
    return used;
}

/* log( sum_i w_i exp(x_i) ) over the listed terms, with max subtraction; -inf if no term. */
static double lse_weighted(const double *x, const double *w, int m)
{
    double mx = -INFINITY;
    for (int i = 0; i < m; ++i) if (x[i] > mx) mx = x[i];
    if (m == 0 || mx == -INFINITY) return -INFINITY;
    double s = 0.0;
    for (int i = 0; i < m; ++i) s += w[i] * exp(x[i] - mx);
    return mx + log(s);
}

/* ---------------------------------------------------------------------------------------------
 * One Multipole Attention decode step for one unit.
 *
 *   levels == 2 (Sec. 3.4):
 *     1. coarse logits l[h,c] = scale q_h.Kc_c ; per-head normaliser LSE_h = log sum_c N_c e^l
 *        (denominator of Eq. 1); rank key r_c = log mean_h exp(l[h,c] - LSE_h)  (Eq. 1, averaged
 *        over the query heads that share the KV head, Sec. 3.1 last paragraph; kept in the log
 *        domain so the order is that of the averaged score without underflow).
 *     2. promising coarse clusters P = budget_select(order by r_c, coarse_budget).
 *     3. fine candidates F = children of P.  l[h,f] likewise; the Eq. 1 denominator at this
 *        level is taken over everything that will enter the softmax through a centroid at this
 *        point: the candidates and the unpromising coarse clusters.
 *     4. selected fine clusters Sel = budget_select(order by r_f over F, key_budget).
 *   levels == 1 (Sec. 3.1-3.2): F = every fine cluster, no coarse terms.
 *     5. (Eq. 2 + exact part, one softmax)
 *        num_h = sum_{t in Sel keys or extra} e^{scale q_h.k_t} v_t
 *              + [mp_terms] ( sum_{f in F\Sel} N_f e^{l[h,f]} Vc_f + sum_{c not in P} N_c e^{l[h,c]} Vc_c )
 *        den_h = same with every value replaced by 1 ;  out_h = num_h / den_h.
 *
 *   mp_terms == 0 drops the Eq. 2 terms (sparse attention over the retrieved keys only, the
 *   comparison method of Sec. 5.1).
 *
 * Lookup query (Sec. 3.1, last paragraph, and Sec. 4): when the clusters were formed on keys
 * rotated to a fixed relative position, the centroid comparison uses a query rotated to the
 * matching fixed position.  ql takes the place of q in every centroid logit l[h,.] (steps 1, 3 and
 * the Eq. 2 terms of step 5, which reuse the logits of the lookup); the exact part of step 5 uses
 * q and the stored keys.  ql == q gives the plain method.
 *
 * Inputs (fp64, row-major):
 *   q, ql [G,d]; K,V [n,d] clustered tokens in sequence order; fine_of_token [n];
 *   Kc_f,Vc_f [Cf,d], N_f [Cf]; coarse_of_fine [Cf], Kc_c,Vc_c [Cc,d], N_c [Cc] (levels==2);
 *   Kx,Vx [nx,d] tokens that are always attended exactly (local buffer, sink tokens).
 * Outputs:
 *   out [G,d], lse [G] (= log den_h), promising [Cc], selected [Cf] (0/1),
 *   r_c [Cc], r_f [Cf] (NaN where the cluster did not take part), n_sel_keys (may be NULL).
 * Returns 0, or -1 if N_f / N_c disagree with fine_of_token / coarse_of_fine.
 * ------------------------------------------------------------------------------------------- */
int mpo_decode_unit(const double *q, const double *ql, int G, int d, double scale,
                    const double *K, const double *V, int n, const int32_t *fine_of_token,
                    int Cf, const double *Kc_f, const double *Vc_f, const int32_t *N_f,
                    int levels, int Cc, const int32_t *coarse_of_fine,
                    const double *Kc_c, const double *Vc_c, const int32_t *N_c,
                    const double *Kx, const double *Vx, int nx,
                    int64_t key_budget, int64_t coarse_budget, int mp_terms,
                    double *out, double *lse, uint8_t *promising, uint8_t *selected,
                    double *r_c, double *r_f, int64_t *n_sel_keys)
{
    /* consistency of the supplied clustering */
    {
        int32_t *cnt = (int32_t *)calloc((size_t)(Cf > 0 ? Cf : 1), sizeof(int32_t));
        int bad = 0;
        for (int t = 0; t < n; ++t) {
            int f = fine_of_token[t];
            if (f < 0 || f >= Cf) { bad = 1; break; }
            cnt[f]++;
        }
        for (int f = 0; f < Cf && !bad; ++f) if (cnt[f] != N_f[f]) bad = 1;
        if (!bad && levels == 2) {
            int64_t *cc = (int64_t *)calloc((size_t)(Cc > 0 ? Cc : 1), sizeof(int64_t));
            for (int f = 0; f < Cf; ++f) {
                int c = coarse_of_fine[f];
                if (c < 0 || c >= Cc) { bad = 1; break; }
                cc[c] += N_f[f];
            }
            for (int c = 0; c < Cc && !bad; ++c) if (cc[c] != N_c[c]) bad = 1;
            free(cc);
        }
        free(cnt);
        if (bad) return -1;
    }

    const size_t GCc = (size_t)G * (size_t)(Cc > 0 ? Cc : 1), GCf = (size_t)G * (size_t)(Cf > 0 ? Cf : 1);
    double *lc = (double *)malloc(sizeof(double) * GCc);   /* l[h,c] */
    double *lf = (double *)malloc(sizeof(double) * GCf);   /* l[h,f] */
    int32_t *ids = (int32_t *)malloc(sizeof(int32_t) * (size_t)((Cc > Cf ? Cc : Cf) + 1));
    /* scratch for one weighted log-sum-exp: over the entries of both levels, or over the G heads */
    const size_t nscr = (size_t)((Cc + Cf) + 1) > (size_t)G ? (size_t)((Cc + Cf) + 1) : (size_t)G;
    double *tx = (double *)malloc(sizeof(double) * nscr);
    double *tw = (double *)malloc(sizeof(double) * nscr);
    double *lseh = (double *)malloc(sizeof(double) * (size_t)G);

    if (promising) memset(promising, 0, (size_t)(Cc > 0 ? Cc : 0));
    memset(selected, 0, (size_t)Cf);
    uint8_t *prom = (uint8_t *)calloc((size_t)(Cc > 0 ? Cc : 1), 1);
    for (int c = 0; c < Cc; ++c) if (r_c) r_c[c] = NAN;
    for (int f = 0; f < Cf; ++f) if (r_f) r_f[f] = NAN;
    double *rc_loc = (double *)malloc(sizeof(double) * (size_t)(Cc > 0 ? Cc : 1));
    double *rf_loc = (double *)malloc(sizeof(double) * (size_t)(Cf > 0 ? Cf : 1));

    /* ---- steps 1-2: coarse level ---- */
    if (levels == 2) {
        int m = 0;
        for (int c = 0; c < Cc; ++c) if (N_c[c] > 0) ids[m++] = c;
        for (int h = 0; h < G; ++h) {
            for (int i = 0; i < m; ++i) {
                int c = ids[i];
                lc[(size_t)h * Cc + c] = scale * dot(ql + (size_t)h * d, Kc_c + (size_t)c * d, d);
                tx[i] = lc[(size_t)h * Cc + c];
                tw[i] = (double)N_c[c];
            }
            lseh[h] = lse_weighted(tx, tw, m);
        }
        for (int i = 0; i < m; ++i) {
            int c = ids[i];
            for (int h = 0; h < G; ++h) { tx[h] = lc[(size_t)h * Cc + c] - lseh[h]; tw[h] = 1.0; }
            rc_loc[c] = lse_weighted(tx, tw, G) - log((double)G);
            if (r_c) r_c[c] = rc_loc[c];
        }
        budget_select(ids, m, rc_loc, N_c, coarse_budget, prom);
        if (promising) memcpy(promising, prom, (size_t)Cc);
    }

    /* ---- steps 3-4: fine level ---- */
    int mF = 0;
    for (int f = 0; f < Cf; ++f) {
        if (N_f[f] <= 0) continue;
        if (levels == 2 && !prom[coarse_of_fine[f]]) continue;
        ids[mF++] = f;
    }
    for (int h = 0; h < G; ++h) {
        int m = 0;
        for (int i = 0; i < mF; ++i) {
            int f = ids[i];
            lf[(size_t)h * Cf + f] = scale * dot(ql + (size_t)h * d, Kc_f + (size_t)f * d, d);
            tx[m] = lf[(size_t)h * Cf + f];
            tw[m] = (double)N_f[f];
            ++m;
        }
        if (levels == 2)
            for (int c = 0; c < Cc; ++c)
                if (N_c[c] > 0 && !prom[c]) { tx[m] = lc[(size_t)h * Cc + c]; tw[m] = (double)N_c[c]; ++m; }
        lseh[h] = lse_weighted(tx, tw, m);
    }
    for (int i = 0; i < mF; ++i) {
        int f = ids[i];
        for (int h = 0; h < G; ++h) { tx[h] = lf[(size_t)h * Cf + f] - lseh[h]; tw[h] = 1.0; }
        rf_loc[f] = lse_weighted(tx, tw, G) - log((double)G);
        if (r_f) r_f[f] = rf_loc[f];
    }
    int64_t nsel = budget_select(ids, mF, rf_loc, N_f, key_budget, selected);
    if (n_sel_keys) *n_sel_keys = nsel;

    /* ---- step 5: one softmax over exact keys and centroid terms ---- */
    double *tl = (double *)malloc(sizeof(double) * (size_t)(n + nx + 1));
    for (int h = 0; h < G; ++h) {
        const double *qh = q + (size_t)h * d;
        double mx = -INFINITY;
        for (int t = 0; t < n; ++t) {
            if (!selected[fine_of_token[t]]) continue;
            tl[t] = scale * dot(qh, K + (size_t)t * d, d);
            if (tl[t] > mx) mx = tl[t];
        }
        for (int t = 0; t < nx; ++t) {
            tl[n + t] = scale * dot(qh, Kx + (size_t)t * d, d);
            if (tl[n + t] > mx) mx = tl[n + t];
        }
        if (mp_terms) {
            for (int i = 0; i < mF; ++i) {
                int f = ids[i];
                if (!selected[f] && lf[(size_t)h * Cf + f] > mx) mx = lf[(size_t)h * Cf + f];
            }
            if (levels == 2)
                for (int c = 0; c < Cc; ++c)
                    if (N_c[c] > 0 && !prom[c] && lc[(size_t)h * Cc + c] > mx) mx = lc[(size_t)h * Cc + c];
        }
        double den = 0.0;
        double *oh = out + (size_t)h * d;
        for (int j = 0; j < d; ++j) oh[j] = 0.0;
        for (int t = 0; t < n; ++t) {
            if (!selected[fine_of_token[t]]) continue;
            double w = exp(tl[t] - mx);
            den += w;
            for (int j = 0; j < d; ++j) oh[j] += w * V[(size_t)t * d + j];
        }
        for (int t = 0; t < nx; ++t) {
            double w = exp(tl[n + t] - mx);
            den += w;
            for (int j = 0; j < d; ++j) oh[j] += w * Vx[(size_t)t * d + j];
        }
        if (mp_terms) {
            for (int i = 0; i < mF; ++i) {
                int f = ids[i];
                if (selected[f]) continue;
                double w = (double)N_f[f] * exp(lf[(size_t)h * Cf + f] - mx);      /* Eq. 2 */
                den += w;
                for (int j = 0; j < d; ++j) oh[j] += w * Vc_f[(size_t)f * d + j];
            }
            if (levels == 2)
                for (int c = 0; c < Cc; ++c) {
                    if (N_c[c] <= 0 || prom[c]) continue;
                    double w = (double)N_c[c] * exp(lc[(size_t)h * Cc + c] - mx);  /* Eq. 2 */
                    den += w;
                    for (int j = 0; j < d; ++j) oh[j] += w * Vc_c[(size_t)c * d + j];
                }
        }
        if (den > 0.0) {
            for (int j = 0; j < d; ++j) oh[j] /= den;
            if (lse) lse[h] = mx + log(den);
        } else {
            if (lse) lse[h] = -INFINITY;
        }
    }
    free(tl); free(rf_loc); free(rc_loc); free(prom); free(lseh); free(tw); free(tx); free(ids);
    free(lf); free(lc);
    return 0;
}

/* Batch of U identical-shape units, one OpenMP thread per unit (arrays are the per-unit arrays of
 * mpo_decode_unit with a leading U axis; q is [U,G,d]).  Returns the number of failing units. */
int mpo_decode_batch(int U, const double *q, int G, int d, double scale,
                     const double *K, const double *V, int n, const int32_t *fine_of_token,
                     int Cf, const double *Kc_f, const double *Vc_f, const int32_t *N_f,
                     int levels, int Cc, const int32_t *coarse_of_fine,
                     const double *Kc_c, const double *Vc_c, const int32_t *N_c,
                     const double *Kx, const double *Vx, int nx,
                     int64_t key_budget, int64_t coarse_budget, int mp_terms,
                     double *out, double *lse, uint8_t *promising, uint8_t *selected)
{
    int fails = 0;
#pragma omp parallel for schedule(dynamic) reduction(+ : fails)
    for (int u = 0; u < U; ++u) {
        size_t cf = (size_t)Cf, cc = (size_t)(Cc > 0 ? Cc : 0), dd = (size_t)d;
        int rc = mpo_decode_unit(
            q + u * (size_t)G * dd, q + u * (size_t)G * dd, G, d, scale, K + u * (size_t)n * dd, V + u * (size_t)n * dd, n,
            fine_of_token + u * (size_t)n, Cf, Kc_f + u * cf * dd, Vc_f + u * cf * dd, N_f + u * cf,
            levels, Cc, levels == 2 ? coarse_of_fine + u * cf : NULL,
            levels == 2 ? Kc_c + u * cc * dd : NULL, levels == 2 ? Vc_c + u * cc * dd : NULL,
            levels == 2 ? N_c + u * cc : NULL,
            nx > 0 ? Kx + u * (size_t)nx * dd : NULL, nx > 0 ? Vx + u * (size_t)nx * dd : NULL, nx,
            key_budget, coarse_budget, mp_terms, out + u * (size_t)G * dd, lse + u * (size_t)G,
            levels == 2 ? promising + u * cc : NULL, selected + u * cf, NULL, NULL, NULL);
        if (rc != 0) fails += 1;
    }
    return fails;
}

void mpo_full_attention_batch(int U, const double *q, const double *K, const double *V, int G, int n,
                              int d, double scale, double *out, double *lse)
{
#pragma omp parallel for schedule(dynamic)
    for (int u = 0; u < U; ++u)
        mpo_full_attention(q + u * (size_t)G * d, K + u * (size_t)n * d, V + u * (size_t)n * d, G, n, d,
                           scale, out + u * (size_t)G * d, lse + u * (size_t)G);
}

/* ---------------------------------------------------------------------------------------------
 * k-means pieces (Sec. 3.1: k-means on the keys, centroid = mean of the members; Sec. 3.3).
 * ------------------------------------------------------------------------------------------- */

/* Round a double to the nearest bfloat16 value (8 significant bits, ties to even), returned as a
 * double.  The clustered index keeps its centroids in bf16, and every later step sees the rounded
 * values.  Magnitudes below 2^-126 (bf16 subnormals) go to signed zero. */
double mpo_round_bf16(double x)
{
    if (x == 0.0 || isnan(x) || isinf(x)) return x;
    int e;
    double m = frexp(fabs(x), &e);          /* |x| = m 2^e, m in [0.5,1) */
    if (e - 1 < -126) return copysign(0.0, x);
    double r = nearbyint(ldexp(m, 8));      /* 8 significant bits, default mode = ties to even */
    double y = ldexp(r, e - 8);
    if (e - 1 > 127 || y >= ldexp(1.0, 128)) y = INFINITY;
    return copysign(y, x);
}

void mpo_round_bf16_array(const double *x, double *y, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) y[i] = mpo_round_bf16(x[i]);
}

/* Assignment step: a[t] = argmin_j sum_i (x_t[i] - c_j[i])^2, equal distances -> lowest j. */
void mpo_assign(const double *X, int n, const double *C, int k, int d, int32_t *a)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < n; ++t) {
        double best = INFINITY;
        int bj = 0;
        for (int j = 0; j < k; ++j) {
            double s = 0.0;
            for (int i = 0; i < d; ++i) {
                double df = X[(size_t)t * d + i] - C[(size_t)j * d + i];
                s += df * df;
            }
            if (s < best) { best = s; bj = j; }
        }
        a[t] = bj;
    }
}

/* Member sums and counts: S[j] = sum of the points with a[t]==j (sequence order), cnt[j]. */
void mpo_member_sums(const double *X, int n, const int32_t *a, int k, int d, double *S, int32_t *cnt)
{
    for (size_t i = 0; i < (size_t)k * d; ++i) S[i] = 0.0;
    for (int j = 0; j < k; ++j) cnt[j] = 0;
    for (int t = 0; t < n; ++t) {
        int j = a[t];
        cnt[j]++;
        for (int i = 0; i < d; ++i) S[(size_t)j * d + i] += X[(size_t)t * d + i];
    }
}

/* Lloyd iterations from explicit seeds (Sec. 5.1: random initialisation, fixed iteration count).
 *   C <- X[init_idx]; repeat iters times: assign; every non-empty cluster's centroid <- bf16(mean
 *   of its members); an empty cluster keeps its centroid.
 * Outputs: C [k,d] (bf16-valued), a [n] (the last assignment), cnt [k] (its member counts). */
void mpo_lloyd(const double *X, int n, int d, const int32_t *init_idx, int k, int iters,
               double *C, int32_t *a, int32_t *cnt)
{
    double *S = (double *)malloc(sizeof(double) * (size_t)k * d);
    for (int j = 0; j < k; ++j)
        for (int i = 0; i < d; ++i) C[(size_t)j * d + i] = X[(size_t)init_idx[j] * d + i];
    for (int it = 0; it < iters; ++it) {
        mpo_assign(X, n, C, k, d, a);
        mpo_member_sums(X, n, a, k, d, S, cnt);
        for (int j = 0; j < k; ++j)
            if (cnt[j] > 0)
                for (int i = 0; i < d; ++i)
                    C[(size_t)j * d + i] = mpo_round_bf16(S[(size_t)j * d + i] / (double)cnt[j]);
    }
    free(S);
}

/* Lloyd iterations continuing from given centroids (used by the online refinement, Sec. 3.3). */
void mpo_lloyd_from(const double *X, int n, int d, int k, int iters, double *C, int32_t *a, int32_t *cnt)
{
    double *S = (double *)malloc(sizeof(double) * (size_t)k * d);
    for (int it = 0; it < iters; ++it) {
        mpo_assign(X, n, C, k, d, a);
        mpo_member_sums(X, n, a, k, d, S, cnt);
        for (int j = 0; j < k; ++j)
            if (cnt[j] > 0)
                for (int i = 0; i < d; ++i)
                    C[(size_t)j * d + i] = mpo_round_bf16(S[(size_t)j * d + i] / (double)cnt[j]);
    }
    free(S);
}

int mpo_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        n = omp_get_num_threads();
    }
#endif
    return n;
}
