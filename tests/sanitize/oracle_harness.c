/*
 * Sanitizer harness for the CPU oracle (test infrastructure).
 *
 * Compiled together with oracle/rbe_oracle.c under -fsanitize=address,undefined
 * and run by tests/test_oracle_sanitized.py.  It calls every exported oracle
 * function on small, ragged shapes -- item counts that are not multiples of
 * anything, k larger than the corpus, empty ranges and id lists, queues longer
 * than a group -- with every array allocated at its exact size, so that an
 * out-of-range index, a misaligned access or an integer overflow anywhere in the
 * oracle aborts the run.  It prints one checksum line per case; the test
 * compares them with the same calls made through the ordinary build.
 */
#include <inttypes.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int32_t orc_binary_dot(const uint64_t *x, const uint64_t *y, uint32_t d);
void orc_popcounts(const uint64_t *planes, uint64_t N, uint32_t d, uint32_t P, const uint64_t *q_planes, uint32_t Pq, int32_t *out);
void orc_scores(const uint64_t *planes, const float *scales, uint64_t N, uint32_t d, uint32_t P, const uint64_t *q_planes,
                const float *q_scales, uint32_t Pq, uint64_t z0, uint64_t z1, double *out);
void orc_scores_at(const uint64_t *planes, const float *scales, uint64_t N, uint32_t d, uint32_t P, const uint64_t *q_planes,
                   const float *q_scales, uint32_t Pq, const int64_t *ids, uint64_t n_ids, double *out);
int64_t orc_topk(const uint64_t *planes, const float *scales, uint64_t N, uint32_t d, uint32_t P, const uint64_t *q_planes,
                 const float *q_scales, uint32_t Pq, uint64_t z0, uint64_t z1, uint64_t k, int64_t *ids_out, double *scores_out);
int64_t orc_topk_of_scores(const double *scores, const int64_t *ids, uint64_t n, uint64_t k, int64_t *ids_out, double *scores_out);
uint64_t orc_n_groups(uint64_t N, uint64_t Tb, uint64_t I);
int64_t orc_nearlossless(const uint64_t *planes, const float *scales, uint64_t N, uint32_t d, uint32_t P, const uint64_t *q_planes,
                         const float *q_scales, uint32_t Pq, uint64_t Tb, uint64_t I, uint64_t qlen, uint64_t k,
                         int64_t *ids_out, double *scores_out, int64_t *winners_ids, double *winners_scores);
void orc_encode(const float *x, uint64_t n, uint32_t d, uint32_t P, uint64_t *planes, float *scales);
void orc_recon_norms(const uint64_t *planes, const float *scales, uint64_t N, uint32_t d, uint32_t P, double *out);
void orc_scores_fq(const uint64_t *planes, const float *scales, uint64_t N, uint32_t d, uint32_t P, const float *q,
                   uint64_t z0, uint64_t z1, double *out);
void orc_scores_at_fq(const uint64_t *planes, const float *scales, uint64_t N, uint32_t d, uint32_t P, const float *q,
                      const int64_t *ids, uint64_t n_ids, double *out);
int64_t orc_topk_fq(const uint64_t *planes, const float *scales, uint64_t N, uint32_t d, uint32_t P, const float *q,
                    uint64_t z0, uint64_t z1, uint64_t k, int64_t *ids_out, double *scores_out);

/* splitmix64: the test regenerates the same inputs in Python */
static uint64_t g_state;
static uint64_t next_u64(void)
{
    uint64_t z = (g_state += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
static float next_unit(void) { return (float)((next_u64() >> 40) + 1) / 16777217.0f; }   /* (0, 1) */

static void *exact_alloc(size_t bytes) { void *p = malloc(bytes ? bytes : 1); if (!p) abort(); return p; }

static double fold(double acc, double v) { return acc * 1.000000119 + (isfinite(v) ? v : -12345.0); }

static void run_case(uint64_t N, uint32_t d, uint32_t P, uint32_t Pq, uint64_t k, uint64_t Tb, uint64_t I, uint64_t qlen, uint64_t seed)
{
    const uint32_t W = d / 64;
    g_state = seed;
    uint64_t *planes = exact_alloc(sizeof(uint64_t) * P * N * W);
    float *scales = exact_alloc(sizeof(float) * P * N);
    uint64_t *qp = exact_alloc(sizeof(uint64_t) * Pq * W);
    float *qs = exact_alloc(sizeof(float) * Pq);
    float *qf = exact_alloc(sizeof(float) * d);
    for (uint64_t i = 0; i < (uint64_t)P * N * W; ++i) planes[i] = next_u64();
    for (uint64_t i = 0; i < (uint64_t)P * N; ++i) scales[i] = next_unit();
    for (uint64_t i = 0; i < (uint64_t)Pq * W; ++i) qp[i] = next_u64();
    for (uint32_t i = 0; i < Pq; ++i) qs[i] = next_unit();
    for (uint32_t i = 0; i < d; ++i) qf[i] = next_unit() - 0.5f;

    double sum = 0.0;
    sum = fold(sum, (double)orc_binary_dot(qp, N ? planes : qp, d));

    int32_t *pc = exact_alloc(sizeof(int32_t) * N * P * Pq);
    orc_popcounts(planes, N, d, P, qp, Pq, pc);
    for (uint64_t i = 0; i < N * P * Pq; ++i) sum = fold(sum, pc[i]);

    const uint64_t z0 = N / 3, z1 = N - N / 5;
    double *sc = exact_alloc(sizeof(double) * (z1 - z0));
    orc_scores(planes, scales, N, d, P, qp, qs, Pq, z0, z1, sc);
    for (uint64_t i = 0; i < z1 - z0; ++i) sum = fold(sum, sc[i]);
    orc_scores(planes, scales, N, d, P, qp, qs, Pq, z1, z1, sc);            /* empty range */
    orc_scores_fq(planes, scales, N, d, P, qf, z0, z1, sc);
    for (uint64_t i = 0; i < z1 - z0; ++i) sum = fold(sum, sc[i]);

    const uint64_t n_ids = N ? 7 : 0;
    int64_t *ids = exact_alloc(sizeof(int64_t) * n_ids);
    double *at = exact_alloc(sizeof(double) * n_ids);
    for (uint64_t i = 0; i < n_ids; ++i) ids[i] = (int64_t)(i == 0 ? N - 1 : (i == 1 ? 0 : next_u64() % N));
    orc_scores_at(planes, scales, N, d, P, qp, qs, Pq, ids, n_ids, at);
    for (uint64_t i = 0; i < n_ids; ++i) sum = fold(sum, at[i]);
    orc_scores_at_fq(planes, scales, N, d, P, qf, ids, n_ids, at);
    for (uint64_t i = 0; i < n_ids; ++i) sum = fold(sum, at[i]);
    orc_scores_at(planes, scales, N, d, P, qp, qs, Pq, ids, 0, at);         /* empty list */

    int64_t *top_i = exact_alloc(sizeof(int64_t) * k);
    double *top_s = exact_alloc(sizeof(double) * k);
    sum = fold(sum, (double)orc_topk(planes, scales, N, d, P, qp, qs, Pq, 0, N, k, top_i, top_s));
    for (uint64_t i = 0; i < k; ++i) { sum = fold(sum, (double)top_i[i]); sum = fold(sum, top_s[i]); }
    sum = fold(sum, (double)orc_topk(planes, scales, N, d, P, qp, qs, Pq, z0, z1, k, top_i, top_s));
    for (uint64_t i = 0; i < k; ++i) sum = fold(sum, (double)top_i[i]);
    sum = fold(sum, (double)orc_topk_fq(planes, scales, N, d, P, qf, 0, N, k, top_i, top_s));
    for (uint64_t i = 0; i < k; ++i) { sum = fold(sum, (double)top_i[i]); sum = fold(sum, top_s[i]); }
    sum = fold(sum, (double)orc_topk(planes, scales, N, d, P, qp, qs, Pq, 0, N, 0, top_i, top_s));   /* k = 0 */

    orc_scores(planes, scales, N, d, P, qp, qs, Pq, z0, z1, sc);
    sum = fold(sum, (double)orc_topk_of_scores(sc, NULL, z1 - z0, k, top_i, top_s));
    for (uint64_t i = 0; i < k; ++i) sum = fold(sum, (double)top_i[i]);

    const uint64_t G = orc_n_groups(N, Tb, I);
    int64_t *w_i = exact_alloc(sizeof(int64_t) * G * qlen);
    double *w_s = exact_alloc(sizeof(double) * G * qlen);
    sum = fold(sum, (double)orc_nearlossless(planes, scales, N, d, P, qp, qs, Pq, Tb, I, qlen, k, top_i, top_s, w_i, w_s));
    for (uint64_t i = 0; i < k; ++i) { sum = fold(sum, (double)top_i[i]); sum = fold(sum, top_s[i]); }
    for (uint64_t i = 0; i < G * qlen; ++i) sum = fold(sum, (double)w_i[i]);
    sum = fold(sum, (double)orc_nearlossless(planes, scales, N, d, P, qp, qs, Pq, Tb, I, qlen, k, top_i, top_s, NULL, NULL));

    double *nrm = exact_alloc(sizeof(double) * N);
    orc_recon_norms(planes, scales, N, d, P, nrm);
    for (uint64_t i = 0; i < N; ++i) sum = fold(sum, nrm[i]);

    const uint64_t n_enc = N < 9 ? N : 9;
    float *x = exact_alloc(sizeof(float) * n_enc * d);
    uint64_t *ep = exact_alloc(sizeof(uint64_t) * P * n_enc * W);
    float *es = exact_alloc(sizeof(float) * P * n_enc);
    for (uint64_t i = 0; i < n_enc * d; ++i) x[i] = next_unit() - 0.5f;
    if (n_enc) x[3] = 0.0f;
    orc_encode(x, n_enc, d, P, ep, es);
    for (uint64_t i = 0; i < (uint64_t)P * n_enc * W; ++i) sum = fold(sum, (double)(ep[i] >> 11));
    for (uint64_t i = 0; i < (uint64_t)P * n_enc; ++i) sum = fold(sum, es[i]);

    printf("case N=%" PRIu64 " d=%u P=%u Pq=%u k=%" PRIu64 " Tb=%" PRIu64 " I=%" PRIu64 " qlen=%" PRIu64 " checksum=%.17g\n",
           N, d, P, Pq, k, Tb, I, qlen, sum);
    free(planes); free(scales); free(qp); free(qs); free(qf); free(pc); free(sc); free(ids); free(at);
    free(top_i); free(top_s); free(w_i); free(w_s); free(nrm); free(x); free(ep); free(es);
}

int main(void)
{
    run_case(1, 64, 1, 1, 3, 4, 3, 1, 11);
    run_case(37, 64, 3, 3, 10, 4, 3, 1, 12);
    run_case(37, 64, 3, 2, 50, 4, 3, 2, 13);          /* k > N */
    run_case(1000, 128, 4, 4, 100, 8, 16, 1, 14);
    run_case(1001, 128, 2, 3, 64, 256, 2, 3, 15);     /* queue longer than a group */
    run_case(613, 256, 2, 2, 613, 16, 5, 2, 16);      /* k == N */
    run_case(70001, 64, 2, 3, 1000, 256, 256, 1, 17); /* one block and a ragged tail */
    puts("done");
    return 0;
}
