/*
 * mage_oracle.c -- TEST INFRASTRUCTURE, not product code.
 *
 * Plain, slow, obviously-correct CPU implementation of what the MAGE hot path
 * computes (arxiv 2602.14209).  Only the test-suite, the smoke check and the
 * benchmark's cpu_baseline leg may call it; the HIP library shares no code,
 * header, table or helper with this file and never calls it.
 *
 * Arithmetic: every dot product, exponential, normaliser and weighted sum is
 * carried in fp64 from the exact input values (fp32 arrays; for bf16 workloads
 * the caller passes fp32 values that are exactly bf16-representable).  Results
 * are rounded once, at the end, to the output type.
 *
 * Readings of the paper taken here (each also listed in the design notes):
 *   - selection scores are post-softmax probabilities (Alg. 1 select stream,
 *     Eq. 5), normalised over the N prefix positions only (Sec. 4 Phase 1:
 *     A in R^{G x B x N});
 *   - group(h) = query heads hG .. hG+G-1 (contiguous GQA map);
 *   - Top-k ties go to the smaller index; a set is emitted ascending;
 *   - the ranking is taken on the fp32-rounded averaged probability (the
 *     precision the GPU path ranks in);
 *   - in-block keys are attended bidirectionally, unmasked, and are never
 *     subject to selection (Eq. 2: j indexes prefix positions; Alg. 1 Phase 2
 *     passes K_h,V_h and C[S] separately).
 *
 * Pins (tests/test_oracle_pins.py): scipy softmax + stable argsort on the
 * G=B=1 special case, torch scaled_dot_product_attention, brute-force sort
 * top-k, closed forms (Q=0, all-equal keys, one-hot values, planted spike),
 * sum-to-one invariants, shift/permutation invariances, k=L == exact.
 * The second workload at the end of this file (page estimator, set overlap) is pinned on numpy
 * block max/min, on page size 1 being the exact selection, on pages of identical rows (bound
 * exact), on a hand-computed sign-aware bound, and on python set intersection.
 * tests/test_oracle_mutations.py plants plausible mistakes in a copy of this file and requires every
 * one of them to fail a pin; tests/test_oracle_sanitizers.py runs every entry point under
 * AddressSanitizer and UndefinedBehaviorSanitizer; tests/golden/ holds a worked example small enough
 * to follow by hand.  No function of this file is unpinned.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int mage_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* logit of query row (q,g) against one key row: (sum_c Q[c]*K[c]) / sqrt(d)
 * -- Alg. 1 "softmax(Q K^T / sqrt(d))", Sec. 4 Phase 1. */
static double logit(const float *qrow, const float *krow, int d)
{
    double acc = 0.0;
    for (int c = 0; c < d; ++c)
        acc += (double)qrow[c] * (double)krow[c];
    return acc / sqrt((double)d);
}

/*
 * Block- and group-averaged prefix attention probabilities.
 *   A[g,q,j]   = softmax_j( Q1[q,g,:].K[j,kv(g),:] / sqrt(d) ),  j in [0,L)   (Alg. 1, select stream)
 *   pbar[g,j]  = (1/B) sum_q A[g,q,j]                                           (Eq. 2, block average)
 *   alpha[h,j] = (1/G) sum_{g in group(h)} pbar[g,j]                            (Eq. 5: 1/(GB) sum_g sum_q)
 * q1 [B,Hq,d], kc [L,Hkv,d]; pbar [Hq,L] (nullable), alpha [Hkv,L]; fp64 out.
 * Returns 0, or -1 on bad arguments / allocation failure.
 */
int mage_oracle_block_probs(int B, int Hq, int Hkv, int d, int64_t L,
                            const float *q1, const float *kc,
                            double *pbar, double *alpha)
{
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || d <= 0 || L <= 0 || Hq % Hkv != 0 || !q1 || !kc || !alpha)
        return -1;
    const int G = Hq / Hkv;
    double *pb = pbar ? pbar : (double *)malloc(sizeof(double) * (size_t)Hq * (size_t)L);
    if (!pb)
        return -1;
    int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int g = 0; g < Hq; ++g) {
        const int h = g / G;
        double *s = (double *)malloc(sizeof(double) * (size_t)L);
        double *row = pb + (size_t)g * (size_t)L;
        if (!s) {
#pragma omp atomic write
            fail = 1;
            continue;
        }
        for (int64_t j = 0; j < L; ++j)
            row[j] = 0.0;
        for (int q = 0; q < B; ++q) {
            const float *qrow = q1 + ((size_t)q * Hq + g) * d;
            double m = -INFINITY;
            for (int64_t j = 0; j < L; ++j) {
                s[j] = logit(qrow, kc + ((size_t)j * Hkv + h) * d, d);
                if (s[j] > m)
                    m = s[j];
            }
            double Z = 0.0;
            for (int64_t j = 0; j < L; ++j)
                Z += exp(s[j] - m);
            for (int64_t j = 0; j < L; ++j)
                row[j] += exp(s[j] - m) / Z;
        }
        for (int64_t j = 0; j < L; ++j)
            row[j] /= (double)B;
        free(s);
    }
    if (!fail) {
        for (int h = 0; h < Hkv; ++h)
            for (int64_t j = 0; j < L; ++j) {
                double acc = 0.0;
                for (int g = h * G; g < (h + 1) * G; ++g)
                    acc += pb[(size_t)g * (size_t)L + j];
                alpha[(size_t)h * (size_t)L + j] = acc / (double)G;
            }
    }
    if (!pbar)
        free(pb);
    return fail ? -1 : 0;
}

typedef struct {
    float v;
    int32_t j;
} scored;

/* larger score first; equal scores: smaller index first */
static int by_score_then_index(const void *a, const void *b)
{
    const scored *x = (const scored *)a, *y = (const scored *)b;
    if (x->v > y->v) return -1;
    if (x->v < y->v) return 1;
    return (x->j > y->j) - (x->j < y->j);
}

static int by_int(const void *a, const void *b)
{
    const int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/*
 * Top-k (Alg. 1 "S <- Top-k(alpha)", Eq. 5) by full sort: the k positions with
 * the largest score, ties to the smaller index, emitted in ascending index order.
 * score [L] fp32, idx_out [k].  Returns 0 or -1.
 */
int mage_oracle_topk(const float *score, int64_t L, int k, int32_t *idx_out)
{
    if (!score || !idx_out || L <= 0 || k <= 0 || (int64_t)k > L || L > INT32_MAX)
        return -1;
    scored *a = (scored *)malloc(sizeof(scored) * (size_t)L);
    if (!a)
        return -1;
    for (int64_t j = 0; j < L; ++j) {
        a[j].v = score[j];
        a[j].j = (int32_t)j;
    }
    qsort(a, (size_t)L, sizeof(scored), by_score_then_index);
    for (int i = 0; i < k; ++i)
        idx_out[i] = a[i].j;
    qsort(idx_out, (size_t)k, sizeof(int32_t), by_int);
    free(a);
    return 0;
}

/*
 * Step-1 selection (Alg. 1 select stream; Eq. 5): block_probs -> round alpha to
 * fp32 -> per-KV-head Top-k.  idx_out [Hkv,k]; alpha32_out [Hkv,L] (nullable);
 * pbar_out [Hq,L] fp64 (nullable); alpha_out [Hkv,L] fp64 (nullable).
 */
int mage_oracle_select(int B, int Hq, int Hkv, int d, int64_t L, int k,
                       const float *q1, const float *kc,
                       int32_t *idx_out, float *alpha32_out,
                       double *alpha_out, double *pbar_out)
{
    if (k <= 0 || (int64_t)k > L || !idx_out || Hkv <= 0 || L <= 0)
        return -1;
    double *alpha = alpha_out ? alpha_out : (double *)malloc(sizeof(double) * (size_t)Hkv * (size_t)L);
    float *a32 = alpha32_out ? alpha32_out : (float *)malloc(sizeof(float) * (size_t)Hkv * (size_t)L);
    int rc = (alpha && a32) ? mage_oracle_block_probs(B, Hq, Hkv, d, L, q1, kc, pbar_out, alpha) : -1;
    if (rc == 0) {
        for (size_t i = 0; i < (size_t)Hkv * (size_t)L; ++i)
            a32[i] = (float)alpha[i];
        for (int h = 0; h < Hkv && rc == 0; ++h)
            rc = mage_oracle_topk(a32 + (size_t)h * (size_t)L, L, k, idx_out + (size_t)h * k);
    }
    if (!alpha_out) free(alpha);
    if (!alpha32_out) free(a32);
    return rc;
}

/*
 * Attention of the B block queries over a set of cache positions plus the
 * block's own keys.
 *   idx == NULL : exact attention over all L cache positions (Alg. 1 main
 *                 stream "Attn(Q,K,V,C)"; the Exact baseline);
 *   idx != NULL : sparse attention -- the cache restricted to the k positions
 *                 idx[kv(g), :] (Alg. 1 Phase 2 "SparseAttn(Q_h,K_h,V_h,C[S])",
 *                 Sec. 4 Phase 2).
 * In both cases one softmax runs over the cache keys kept plus the nb in-block
 * keys (nb = 0 when k_blk == NULL), all logits scaled 1/sqrt(d), no mask.  nb equals B in
 * the method; it is a separate argument so that a test can evaluate a sample of the B
 * query rows against the full block.
 * q [B,Hq,d]; kc,vc [L,Hkv,d]; idx [Hkv,k]; k_blk,v_blk [nb,Hkv,d];
 * out [B,Hq,d] fp32; lse [B,Hq] fp32 (nullable; natural-log sum-exp of the logits).
 */
int mage_oracle_attn(int B, int Hq, int Hkv, int d, int64_t L,
                     const float *q, const float *kc, const float *vc,
                     const int32_t *idx, int k,
                     const float *k_blk, const float *v_blk, int nb_in,
                     float *out, float *lse)
{
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || d <= 0 || L <= 0 || Hq % Hkv != 0 || !q || !kc || !vc || !out)
        return -1;
    if (idx && (k <= 0 || (int64_t)k > L))
        return -1;
    if ((k_blk == NULL) != (v_blk == NULL))
        return -1;
    if (idx)
        for (size_t i = 0; i < (size_t)Hkv * (size_t)k; ++i)
            if (idx[i] < 0 || (int64_t)idx[i] >= L)
                return -1;
    const int G = Hq / Hkv;
    const int64_t nc = idx ? (int64_t)k : L;
    const int nb = k_blk ? nb_in : 0;
    if (nb < 0)
        return -1;
    const int64_t n = nc + nb;
    int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int r = 0; r < B * Hq; ++r) {
        const int qi = r / Hq, g = r % Hq, h = g / G;
        const float *qrow = q + ((size_t)qi * Hq + g) * d;
        double *s = (double *)malloc(sizeof(double) * (size_t)n);
        double *acc = (double *)malloc(sizeof(double) * (size_t)d);
        if (!s || !acc) {
#pragma omp atomic write
            fail = 1;
            free(s);
            free(acc);
            continue;
        }
        double m = -INFINITY;
        for (int64_t t = 0; t < n; ++t) {
            const float *krow;
            if (t < nc) {
                const int64_t j = idx ? (int64_t)idx[(size_t)h * k + t] : t;
                krow = kc + ((size_t)j * Hkv + h) * d;
            } else {
                krow = k_blk + ((size_t)(t - nc) * Hkv + h) * d;
            }
            s[t] = logit(qrow, krow, d);
            if (s[t] > m)
                m = s[t];
        }
        double Z = 0.0;
        for (int64_t t = 0; t < n; ++t)
            Z += exp(s[t] - m);
        for (int c = 0; c < d; ++c)
            acc[c] = 0.0;
        for (int64_t t = 0; t < n; ++t) {
            const float *vrow;
            if (t < nc) {
                const int64_t j = idx ? (int64_t)idx[(size_t)h * k + t] : t;
                vrow = vc + ((size_t)j * Hkv + h) * d;
            } else {
                vrow = v_blk + ((size_t)(t - nc) * Hkv + h) * d;
            }
            const double p = exp(s[t] - m) / Z;
            for (int c = 0; c < d; ++c)
                acc[c] += p * (double)vrow[c];
        }
        float *orow = out + ((size_t)qi * Hq + g) * d;
        for (int c = 0; c < d; ++c)
            orow[c] = (float)acc[c];
        if (lse)
            lse[(size_t)qi * Hq + g] = (float)(m + log(Z));
        free(s);
        free(acc);
    }
    return fail ? -1 : 0;
}

/*
 * Compacted selection (Sec. 4 Phase 2: the index set is fixed for steps 2..T, so the selected
 * rows may be copied once): dst[p,h,:] = src[idx[h,p],h,:] for p in [0,k).  src [L,Hkv,d],
 * idx [Hkv,k], dst [k,Hkv,d].  A copy: bit-exact by construction.
 */
int mage_oracle_compact(int Hkv, int d, int64_t L, int k, const float *src, const int32_t *idx, float *dst)
{
    if (Hkv <= 0 || d <= 0 || L <= 0 || k <= 0 || !src || !idx || !dst)
        return -1;
    for (int h = 0; h < Hkv; ++h)
        for (int p = 0; p < k; ++p) {
            const int32_t j = idx[(size_t)h * k + p];
            if (j < 0 || (int64_t)j >= L)
                return -1;
            memcpy(dst + ((size_t)p * Hkv + h) * d, src + ((size_t)j * Hkv + h) * d, sizeof(float) * (size_t)d);
        }
    return 0;
}

/* ------------------------------------------------------------------------------------------
 * Second workload: a Quest-style page estimator under per-block selection, and the two
 * set-overlap metrics the paper measures estimators with.
 *
 * Readings taken here (the paper describes Quest in one sentence and never says how its page
 * scores enter Eq. 2):
 *   - a page is a run of p consecutive cache positions of one KV head (the last page may be
 *     shorter); its summary is the per-channel maximum and minimum of its key rows
 *     (Sec. 2, "Methods for AR LLMs");
 *   - the page score of a query is the sign-aware upper bound on q.k over the page,
 *     sum_c max(q_c Kmax_c, q_c Kmin_c) (same passage);
 *   - the estimated score of position j is what the exact score becomes when every logit is
 *     replaced by the bound of its page: softmax over the L prefix positions of
 *     bound(page(j)) / sqrt(d).  Eq. 2 (per-block form) then averages these over the G heads and
 *     B tokens and takes Top-k exactly as for the exact scores, so with p = 1 the estimator IS
 *     the oracle;
 *   - ties (all positions of a page tie) go to the smaller index, as everywhere else.
 * ------------------------------------------------------------------------------------------ */

/*
 * Page summaries (Sec. 2, Quest): kmax[P,h,c] = max_j K[j,h,c], kmin likewise, j over page P =
 * [P*p, min((P+1)*p, L)).  kc [L,Hkv,d]; kmax, kmin [ceil(L/p),Hkv,d].
 */
int mage_oracle_page_summary(int Hkv, int d, int64_t L, int p, const float *kc, float *kmax, float *kmin)
{
    if (Hkv <= 0 || d <= 0 || L <= 0 || p <= 0 || !kc || !kmax || !kmin)
        return -1;
    const int64_t np = (L + p - 1) / p;
    for (int64_t P = 0; P < np; ++P)
        for (int h = 0; h < Hkv; ++h)
            for (int c = 0; c < d; ++c) {
                float mx = -INFINITY, mn = INFINITY;
                for (int64_t j = P * p; j < (P + 1) * p && j < L; ++j) {
                    const float v = kc[((size_t)j * Hkv + h) * d + c];
                    if (v > mx) mx = v;
                    if (v < mn) mn = v;
                }
                kmax[((size_t)P * Hkv + h) * d + c] = mx;
                kmin[((size_t)P * Hkv + h) * d + c] = mn;
            }
    return 0;
}

/* sign-aware upper bound of q.k over a page: sum_c max(q_c Kmax_c, q_c Kmin_c) (Sec. 2, Quest) */
static double page_bound(const float *qrow, const float *mx, const float *mn, int d)
{
    double acc = 0.0;
    for (int c = 0; c < d; ++c) {
        const double a = (double)qrow[c] * (double)mx[c], b = (double)qrow[c] * (double)mn[c];
        acc += a > b ? a : b;
    }
    return acc;
}

/*
 * Estimated per-block scores (Eq. 2, per-block form, with the exact score replaced by the
 * estimator's):  s[g,q,j] = softmax_j( bound[g,q,page(j)] / sqrt(d) ),  j in [0,L);
 * est[h,j] = 1/(GB) sum_{g in group(h)} sum_q s[g,q,j].
 * q [B,Hq,d]; kmax, kmin [ceil(L/p),Hkv,d]; est [Hkv,L] fp64.
 */
int mage_oracle_quest_probs(int B, int Hq, int Hkv, int d, int64_t L, int p,
                            const float *q, const float *kmax, const float *kmin, double *est)
{
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || d <= 0 || L <= 0 || p <= 0 || Hq % Hkv != 0 || !q || !kmax || !kmin || !est)
        return -1;
    const int G = Hq / Hkv;
    const int64_t np = (L + p - 1) / p;
    for (size_t i = 0; i < (size_t)Hkv * (size_t)L; ++i)
        est[i] = 0.0;
    int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int h = 0; h < Hkv; ++h) {
        double *s = (double *)malloc(sizeof(double) * (size_t)L);
        if (!s) {
#pragma omp atomic write
            fail = 1;
            continue;
        }
        double *row = est + (size_t)h * (size_t)L;
        for (int g = h * G; g < (h + 1) * G; ++g)
            for (int qi = 0; qi < B; ++qi) {
                const float *qrow = q + ((size_t)qi * Hq + g) * d;
                double m = -INFINITY;
                for (int64_t P = 0; P < np; ++P) {
                    const double b = page_bound(qrow, kmax + ((size_t)P * Hkv + h) * d, kmin + ((size_t)P * Hkv + h) * d, d) /
                                     sqrt((double)d);
                    for (int64_t j = P * p; j < (P + 1) * p && j < L; ++j)
                        s[j] = b;
                    if (b > m) m = b;
                }
                double Z = 0.0;
                for (int64_t j = 0; j < L; ++j)
                    Z += exp(s[j] - m);
                for (int64_t j = 0; j < L; ++j)
                    row[j] += exp(s[j] - m) / Z;
            }
        for (int64_t j = 0; j < L; ++j)
            row[j] /= (double)G * (double)B;
        free(s);
    }
    return fail ? -1 : 0;
}

/*
 * Estimated per-block KV subset (Eq. 2 with the estimator's scores): page summaries of kc ->
 * quest_probs -> round to fp32 -> per-KV-head Top-k over the L positions.
 * idx_out [Hkv,k]; est32_out [Hkv,L] (nullable).
 */
int mage_oracle_quest_select(int B, int Hq, int Hkv, int d, int64_t L, int p, int k,
                             const float *q, const float *kc, int32_t *idx_out, float *est32_out)
{
    if (k <= 0 || (int64_t)k > L || !idx_out || Hkv <= 0 || d <= 0 || L <= 0 || p <= 0)
        return -1;
    const int64_t np = (L + p - 1) / p;
    float *mx = (float *)malloc(sizeof(float) * (size_t)np * Hkv * d);
    float *mn = (float *)malloc(sizeof(float) * (size_t)np * Hkv * d);
    double *est = (double *)malloc(sizeof(double) * (size_t)Hkv * (size_t)L);
    float *e32 = est32_out ? est32_out : (float *)malloc(sizeof(float) * (size_t)Hkv * (size_t)L);
    int rc = (mx && mn && est && e32) ? mage_oracle_page_summary(Hkv, d, L, p, kc, mx, mn) : -1;
    if (rc == 0)
        rc = mage_oracle_quest_probs(B, Hq, Hkv, d, L, p, q, mx, mn, est);
    if (rc == 0) {
        for (size_t i = 0; i < (size_t)Hkv * (size_t)L; ++i)
            e32[i] = (float)est[i];
        for (int h = 0; h < Hkv && rc == 0; ++h)
            rc = mage_oracle_topk(e32 + (size_t)h * (size_t)L, L, k, idx_out + (size_t)h * k);
    }
    free(mx);
    free(mn);
    free(est);
    if (!est32_out) free(e32);
    return rc;
}

/*
 * |A intersect B| / k for two index sets of k distinct entries each, in any order: the ratio of
 * Eq. 1 (estimation accuracy: evaluated subset against an oracle subset) and of Eq. 3 (recall of the
 * step-1 oracle subset at a later noise level).  By direct comparison of every pair.
 */
double mage_oracle_overlap(int k, const int32_t *a, const int32_t *b)
{
    if (k <= 0 || !a || !b)
        return -1.0;
    int64_t common = 0;
    for (int i = 0; i < k; ++i)
        for (int j = 0; j < k; ++j)
            if (a[i] == b[j]) {
                ++common;
                break;
            }
    return (double)common / (double)k;
}

