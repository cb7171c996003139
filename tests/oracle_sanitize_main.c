/* Runs every entry point of the CPU oracle on small seeded inputs with exactly-sized heap buffers.
 * tests/test_oracle_sanitizers.py builds this file together with oracle/mage_oracle.c under
 * -fsanitize=address,undefined: any out-of-bounds access, use of uninitialised index or undefined
 * arithmetic in the oracle aborts the run.  The shapes include the ragged and degenerate cases
 * (one key, k = L, a short last page, one query row, no block keys). */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int mage_oracle_block_probs(int B, int Hq, int Hkv, int d, int64_t L, const float *q1, const float *kc, double *pbar, double *alpha);
int mage_oracle_topk(const float *score, int64_t L, int k, int32_t *idx_out);
int mage_oracle_select(int B, int Hq, int Hkv, int d, int64_t L, int k, const float *q1, const float *kc,
                       int32_t *idx_out, float *alpha32_out, double *alpha_out, double *pbar_out);
int mage_oracle_attn(int B, int Hq, int Hkv, int d, int64_t L, const float *q, const float *kc, const float *vc,
                     const int32_t *idx, int k, const float *k_blk, const float *v_blk, int nb_in, float *out, float *lse);
int mage_oracle_compact(int Hkv, int d, int64_t L, int k, const float *src, const int32_t *idx, float *dst);
int mage_oracle_page_summary(int Hkv, int d, int64_t L, int p, const float *kc, float *kmax, float *kmin);
int mage_oracle_quest_probs(int B, int Hq, int Hkv, int d, int64_t L, int p, const float *q, const float *kmax, const float *kmin, double *est);
int mage_oracle_quest_select(int B, int Hq, int Hkv, int d, int64_t L, int p, int k, const float *q, const float *kc,
                             int32_t *idx_out, float *est32_out);
double mage_oracle_overlap(int k, const int32_t *a, const int32_t *b);

static uint64_t state = 88172645463325252ull;
static float rnd(void)
{
    state ^= state << 13; state ^= state >> 7; state ^= state << 17;
    return (float)((double)(state >> 11) / 9007199254740992.0 * 4.0 - 2.0);
}
static float *fill(size_t n)
{
    float *p = malloc(n * sizeof(float));
    for (size_t i = 0; i < n; ++i) p[i] = rnd();
    return p;
}
#define REQUIRE(x) do { if (!(x)) { printf("FAILED: %s (line %d)\n", #x, __LINE__); return 1; } } while (0)

static int one_case(int B, int Hq, int Hkv, int d, int64_t L, int k, int p, int nb)
{
    float *q = fill((size_t)B * Hq * d), *kc = fill((size_t)L * Hkv * d), *vc = fill((size_t)L * Hkv * d);
    float *kb = nb ? fill((size_t)nb * Hkv * d) : NULL, *vb = nb ? fill((size_t)nb * Hkv * d) : NULL;
    double *pbar = malloc((size_t)Hq * L * sizeof(double)), *alpha = malloc((size_t)Hkv * L * sizeof(double));
    REQUIRE(mage_oracle_block_probs(B, Hq, Hkv, d, L, q, kc, pbar, alpha) == 0);
    int32_t *idx = malloc((size_t)Hkv * k * sizeof(int32_t));
    float *alpha32 = malloc((size_t)Hkv * L * sizeof(float));
    REQUIRE(mage_oracle_select(B, Hq, Hkv, d, L, k, q, kc, idx, alpha32, alpha, pbar) == 0);
    REQUIRE(mage_oracle_select(B, Hq, Hkv, d, L, k, q, kc, idx, NULL, NULL, NULL) == 0);
    for (int h = 0; h < Hkv; ++h) {
        int32_t *t = malloc((size_t)k * sizeof(int32_t));
        REQUIRE(mage_oracle_topk(alpha32 + (size_t)h * L, L, k, t) == 0);
        for (int i = 0; i < k; ++i) REQUIRE(t[i] == idx[(size_t)h * k + i]);
        free(t);
    }
    float *out = malloc((size_t)B * Hq * d * sizeof(float)), *lse = malloc((size_t)B * Hq * sizeof(float));
    REQUIRE(mage_oracle_attn(B, Hq, Hkv, d, L, q, kc, vc, NULL, 0, kb, vb, nb, out, lse) == 0);
    REQUIRE(mage_oracle_attn(B, Hq, Hkv, d, L, q, kc, vc, idx, k, kb, vb, nb, out, NULL) == 0);
    float *ks = malloc((size_t)k * Hkv * d * sizeof(float));
    REQUIRE(mage_oracle_compact(Hkv, d, L, k, kc, idx, ks) == 0);
    const int64_t np = (L + p - 1) / p;
    float *kmax = malloc((size_t)np * Hkv * d * sizeof(float)), *kmin = malloc((size_t)np * Hkv * d * sizeof(float));
    REQUIRE(mage_oracle_page_summary(Hkv, d, L, p, kc, kmax, kmin) == 0);
    double *est = malloc((size_t)Hkv * L * sizeof(double));
    REQUIRE(mage_oracle_quest_probs(B, Hq, Hkv, d, L, p, q, kmax, kmin, est) == 0);
    int32_t *qidx = malloc((size_t)Hkv * k * sizeof(int32_t));
    float *est32 = malloc((size_t)Hkv * L * sizeof(float));
    REQUIRE(mage_oracle_quest_select(B, Hq, Hkv, d, L, p, k, q, kc, qidx, est32) == 0);
    for (int h = 0; h < Hkv; ++h) {
        const double o = mage_oracle_overlap(k, idx + (size_t)h * k, qidx + (size_t)h * k);
        REQUIRE(o >= 0.0 && o <= 1.0);
    }
    free(q); free(kc); free(vc); free(kb); free(vb); free(pbar); free(alpha); free(idx); free(alpha32);
    free(out); free(lse); free(ks); free(kmax); free(kmin); free(est); free(qidx); free(est32);
    return 0;
}

int main(void)
{
    /* B, Hq, Hkv, d, L, k, p, nb */
    if (one_case(4, 4, 1, 64, 257, 33, 16, 4)) return 1;      /* ragged last page, ragged everything */
    if (one_case(1, 2, 2, 128, 1, 1, 16, 0)) return 1;        /* one key, one row per head, no block keys */
    if (one_case(3, 6, 2, 64, 40, 40, 8, 3)) return 1;        /* k = L, G = 3 */
    if (one_case(5, 7, 7, 32, 129, 7, 1, 5)) return 1;        /* G = 1, pages of one position */
    if (one_case(2, 8, 2, 16, 64, 16, 64, 2)) return 1;       /* one page */
    printf("OK\n");
    return 0;
}
