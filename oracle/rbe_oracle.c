/*
 * CPU oracle for Recurrent Binary Embedding (RBE) retrieval.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, single-threaded
 * reference against which the GPU library is checked.  It shares no code,
 * header, table or helper with the GPU library, and the GPU library never
 * calls it.  Only the test-suite, the smoke check and the benchmark's
 * "cpu_baseline" leg may load it.
 *
 * Notation (paper Sec. 4-6): an item (the paper's "keyword") is stored as P
 * "ingredient vectors" (base vector + P-1 residual vectors, Eq. 8-11), each in
 * {-1,+1}^d and packed one bit per dimension: bit 1 <-> +1, bit 0 <-> -1,
 * dimension i <-> bit (i % 64) of 64-bit word (i / 64).  Ingredient vector j
 * of item z carries a non-negative fp32 scale a_j[z] (the paper's fixed
 * residual weight 2^-j and stored inverse norm are the special case
 * a_j[z] = 2^-j / ||b_z||, Sec. 4.3 and Sec. 5.1).  A query has Pq ingredient
 * vectors with scales c_i.
 *
 * Arrays: planes[P][N][W] (uint64, W = d/64), scales[P][N] (float),
 * q_planes[Pq][W], q_scales[Pq].
 *
 * Every floating-point combination below is done in double.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ */
/* Binary dot product (Sec. 5.1, the bit-wise identity following Eq. 14,
 * with the printed formula's sign and shift direction corrected):
 * for x, y in {-1,+1}^d,  x . y = d - 2 * popcount(bits(x) XOR bits(y)).   */
/* ------------------------------------------------------------------ */
static uint32_t popcount_xor(const uint64_t *x, const uint64_t *y, uint32_t W)
{
    uint32_t c = 0;
    for (uint32_t w = 0; w < W; ++w)
        c += (uint32_t)__builtin_popcountll(x[w] ^ y[w]);
    return c;
}

int32_t orc_binary_dot(const uint64_t *x, const uint64_t *y, uint32_t d)
{
    return (int32_t)d - 2 * (int32_t)popcount_xor(x, y, d / 64);
}

/* popcount(Q_i XOR K_j[z]) for every item, corpus plane j and query plane i.
 * out[z][j][i], int32.                                                      */
void orc_popcounts(const uint64_t *planes, uint64_t N, uint32_t d, uint32_t P,
                   const uint64_t *q_planes, uint32_t Pq, int32_t *out)
{
    const uint32_t W = d / 64;
    for (uint64_t z = 0; z < N; ++z)
        for (uint32_t j = 0; j < P; ++j)
            for (uint32_t i = 0; i < Pq; ++i)
                out[(z * P + j) * Pq + i] = (int32_t)popcount_xor(
                    q_planes + (uint64_t)i * W, planes + ((uint64_t)j * N + z) * W, W);
}

/* ------------------------------------------------------------------ */
/* Score of one (query, item) pair: the dot product of the two RBE
 * embeddings expanded into binary dot products (Eq. 14 with general
 * weights):  s = sum_j sum_i a_j[z] * c_i * (b_q^i . b_z^j).               */
/* ------------------------------------------------------------------ */
static double score_pair(const uint64_t *planes, const float *scales, uint64_t N,
                         uint32_t d, uint32_t P, uint64_t z,
                         const uint64_t *q_planes, const float *q_scales, uint32_t Pq)
{
    const uint32_t W = d / 64;
    double s = 0.0;
    for (uint32_t j = 0; j < P; ++j) {
        const double a = (double)scales[(uint64_t)j * N + z];
        const uint64_t *kj = planes + ((uint64_t)j * N + z) * W;
        for (uint32_t i = 0; i < Pq; ++i) {
            const int32_t dot = (int32_t)d - 2 * (int32_t)popcount_xor(q_planes + (uint64_t)i * W, kj, W);
            s += a * (double)q_scales[i] * (double)dot;
        }
    }
    return s;
}

/* Dense scores of one query against items [z0, z1).  out[z - z0], double.  */
void orc_scores(const uint64_t *planes, const float *scales, uint64_t N,
                uint32_t d, uint32_t P,
                const uint64_t *q_planes, const float *q_scales, uint32_t Pq,
                uint64_t z0, uint64_t z1, double *out)
{
    for (uint64_t z = z0; z < z1; ++z)
        out[z - z0] = score_pair(planes, scales, N, d, P, z, q_planes, q_scales, Pq);
}

/* Scores of one query against an explicit list of item ids.  out[r], double. */
void orc_scores_at(const uint64_t *planes, const float *scales, uint64_t N,
                   uint32_t d, uint32_t P,
                   const uint64_t *q_planes, const float *q_scales, uint32_t Pq,
                   const int64_t *ids, uint64_t n_ids, double *out)
{
    for (uint64_t r = 0; r < n_ids; ++r)
        out[r] = score_pair(planes, scales, N, d, P, (uint64_t)ids[r], q_planes, q_scales, Pq);
}

/* ------------------------------------------------------------------ */
/* Exact top-k under the total order (score descending, id ascending).
 * Definition: sort every (score, id) by that order and keep the first k.
 * For large N the sort is replaced by a bounded binary heap that keeps the
 * k best seen so far (worst at the root); the result is the same set and is
 * sorted at the end.                                                        */
/* ------------------------------------------------------------------ */
typedef struct { double s; int64_t id; } cand_t;

/* 1 if a ranks strictly before (is better than) b */
static int better(const cand_t *a, const cand_t *b)
{
    if (a->s != b->s) return a->s > b->s;
    return a->id < b->id;
}

static void heap_sift_down(cand_t *h, uint64_t n, uint64_t p)
{   /* root = worst element */
    for (;;) {
        uint64_t l = 2 * p + 1, r = l + 1, w = p;
        if (l < n && better(&h[w], &h[l])) w = l;
        if (r < n && better(&h[w], &h[r])) w = r;
        if (w == p) return;
        cand_t t = h[p]; h[p] = h[w]; h[w] = t;
        p = w;
    }
}

static void heap_sift_up(cand_t *h, uint64_t c)
{
    while (c > 0) {
        uint64_t p = (c - 1) / 2;
        if (!better(&h[p], &h[c])) return;   /* parent already worse-or-equal */
        cand_t t = h[p]; h[p] = h[c]; h[c] = t;
        c = p;
    }
}

typedef struct { cand_t *h; uint64_t n, k; } topk_t;

static void topk_offer(topk_t *t, double s, int64_t id)
{
    cand_t c = { s, id };
    if (t->k == 0) return;
    if (t->n < t->k) {
        t->h[t->n] = c;
        heap_sift_up(t->h, t->n);
        t->n++;
    } else if (better(&c, &t->h[0])) {
        t->h[0] = c;
        heap_sift_down(t->h, t->n, 0);
    }
}

static int cmp_rank(const void *pa, const void *pb)
{
    const cand_t *a = (const cand_t *)pa, *b = (const cand_t *)pb;
    if (better(a, b)) return -1;
    if (better(b, a)) return 1;
    return 0;
}

/* Writes min(k, count) results, best first; the tail up to k is filled with
 * id = -1, score = -inf.  Returns the number of valid results.             */
static uint64_t topk_finish(topk_t *t, int64_t *ids_out, double *scores_out)
{
    qsort(t->h, t->n, sizeof(cand_t), cmp_rank);
    for (uint64_t r = 0; r < t->k; ++r) {
        if (r < t->n) { ids_out[r] = t->h[r].id; scores_out[r] = t->h[r].s; }
        else          { ids_out[r] = -1;         scores_out[r] = -INFINITY; }
    }
    return t->n;
}

/* Exact top-k of one query over items [z0, z1) (ids are global item ids).  */
int64_t orc_topk(const uint64_t *planes, const float *scales, uint64_t N,
                 uint32_t d, uint32_t P,
                 const uint64_t *q_planes, const float *q_scales, uint32_t Pq,
                 uint64_t z0, uint64_t z1, uint64_t k,
                 int64_t *ids_out, double *scores_out)
{
    topk_t t = { (cand_t *)malloc((k ? k : 1) * sizeof(cand_t)), 0, k };
    if (!t.h) return -1;
    for (uint64_t z = z0; z < z1; ++z)
        topk_offer(&t, score_pair(planes, scales, N, d, P, z, q_planes, q_scales, Pq), (int64_t)z);
    uint64_t n = topk_finish(&t, ids_out, scores_out);
    free(t.h);
    return (int64_t)n;
}

/* Top-k of an explicit list of (score, id) pairs (same order).             */
int64_t orc_topk_of_scores(const double *scores, const int64_t *ids, uint64_t n,
                           uint64_t k, int64_t *ids_out, double *scores_out)
{
    topk_t t = { (cand_t *)malloc((k ? k : 1) * sizeof(cand_t)), 0, k };
    if (!t.h) return -1;
    for (uint64_t r = 0; r < n; ++r)
        topk_offer(&t, scores[r], ids ? ids[r] : (int64_t)r);
    uint64_t m = topk_finish(&t, ids_out, scores_out);
    free(t.h);
    return (int64_t)m;
}

/* ------------------------------------------------------------------ */
/* Near-lossless selection (Algorithm 1, Sec. 6.2; miss model in Appendix A).
 * The selector partitions the item ids into groups; every group forwards only
 * its best qlen items (the paper runs it with qlen = 1) and the answer is the
 * exact top-k of what was forwarded.  The partition follows from how the
 * algorithm hands ids to its Tb threads per block, each thread taking I ids at
 * a stride of Tb: consecutive spans of Tb*I ids form a block, and inside a
 * block the ids congruent modulo Tb share a group.  Group number
 *     g(z) = (z div (Tb*I)) * Tb + (z mod Tb),
 * and conversely group g holds the ids
 *     (g div Tb) * Tb*I + (g mod Tb) + m*Tb,   m = 0 .. I-1,   that are < N.
 * Order inside a group and in the answer: score descending, id ascending.
 * winners_ids / winners_scores (optional): [n_groups][qlen], best first,
 * id -1 / score -inf where a group has fewer than qlen items.                */
/* ------------------------------------------------------------------ */
uint64_t orc_n_groups(uint64_t N, uint64_t Tb, uint64_t I)
{
    const uint64_t span = Tb * I;
    return ((N + span - 1) / span) * Tb;
}

int64_t orc_nearlossless(const uint64_t *planes, const float *scales, uint64_t N,
                         uint32_t d, uint32_t P,
                         const uint64_t *q_planes, const float *q_scales, uint32_t Pq,
                         uint64_t Tb, uint64_t I, uint64_t qlen, uint64_t k,
                         int64_t *ids_out, double *scores_out,
                         int64_t *winners_ids, double *winners_scores)
{
    const uint64_t G = orc_n_groups(N, Tb, I);
    if (qlen == 0) return -1;
    cand_t *kept = (cand_t *)malloc(qlen * sizeof(cand_t));     /* one group's best, best first */
    topk_t t = { (cand_t *)malloc((k ? k : 1) * sizeof(cand_t)), 0, k };
    if (!kept || !t.h) { free(kept); free(t.h); return -1; }

    for (uint64_t g = 0; g < G; ++g) {
        const uint64_t first = (g / Tb) * Tb * I + (g % Tb);
        uint64_t n_kept = 0;
        for (uint64_t m = 0; m < I; ++m) {
            const uint64_t z = first + m * Tb;
            if (z >= N) break;
            const cand_t c = { score_pair(planes, scales, N, d, P, z, q_planes, q_scales, Pq), (int64_t)z };
            /* position of c among the kept entries; entries after it move down, the last may fall off */
            uint64_t pos = n_kept;
            while (pos > 0 && better(&c, &kept[pos - 1])) --pos;
            if (pos >= qlen) continue;
            if (n_kept < qlen) ++n_kept;
            for (uint64_t e = n_kept - 1; e > pos; --e) kept[e] = kept[e - 1];
            kept[pos] = c;
        }
        for (uint64_t e = 0; e < qlen; ++e) {
            const int live = e < n_kept;
            if (winners_ids)    winners_ids[g * qlen + e] = live ? kept[e].id : -1;
            if (winners_scores) winners_scores[g * qlen + e] = live ? kept[e].s : -INFINITY;
            if (live) topk_offer(&t, kept[e].s, kept[e].id);
        }
    }
    uint64_t n = topk_finish(&t, ids_out, scores_out);
    free(t.h);
    free(kept);
    return (int64_t)n;
}

/* ------------------------------------------------------------------ */
/* Stand-in encoder (the learned RBE layers of Eq. 8-11 need trained
 * matrices that are not available; this greedy residual binariser produces
 * vectors of the same form).  For t = 0..P-1, with r_0 = x:
 *     alpha_t = mean_i |r_t[i]|              (sum in double, stored as fp32)
 *     bit_t[i] = 1 if r_t[i] > 0 else 0      (rho of Eq. 12: rho(0) = -1)
 *     r_{t+1}[i] = fp32( r_t[i] - alpha_t * (2*bit_t[i] - 1) )
 * x: [n][d] fp32.  planes: [P][n][W], scales: [P][n].                       */
/* ------------------------------------------------------------------ */
void orc_encode(const float *x, uint64_t n, uint32_t d, uint32_t P,
                uint64_t *planes, float *scales)
{
    const uint32_t W = d / 64;
    float *r = (float *)malloc(sizeof(float) * d);
    for (uint64_t z = 0; z < n; ++z) {
        memcpy(r, x + z * d, sizeof(float) * d);
        for (uint32_t t = 0; t < P; ++t) {
            double sum = 0.0;
            for (uint32_t i = 0; i < d; ++i) sum += fabs((double)r[i]);
            const float alpha = (float)(sum / (double)d);
            uint64_t *out = planes + ((uint64_t)t * n + z) * W;
            for (uint32_t w = 0; w < W; ++w) out[w] = 0;
            for (uint32_t i = 0; i < d; ++i) {
                const int bit = r[i] > 0.0f;
                if (bit) out[i / 64] |= (uint64_t)1 << (i % 64);
                r[i] = (float)((double)r[i] - (double)alpha * (bit ? 1.0 : -1.0));
            }
            scales[(uint64_t)t * n + z] = alpha;
        }
    }
    free(r);
}

/* ------------------------------------------------------------------ */
/* Euclidean norm of each item's reconstructed embedding
 *     khat_z = sum_j a_j[z] * b_z^j,     b_z^j in {-1,+1}^d,
 * by unpacking the bits (no popcount shortcut).  This is the keyword-side
 * magnitude that the cosine of Eq. 14 divides by (Sec. 5.1).  out[z], double. */
/* ------------------------------------------------------------------ */
void orc_recon_norms(const uint64_t *planes, const float *scales, uint64_t N,
                     uint32_t d, uint32_t P, double *out)
{
    const uint32_t W = d / 64;
    for (uint64_t z = 0; z < N; ++z) {
        double n2 = 0.0;
        for (uint32_t i = 0; i < d; ++i) {
            double v = 0.0;
            for (uint32_t j = 0; j < P; ++j) {
                const uint64_t word = planes[((uint64_t)j * N + z) * W + i / 64];
                const double sgn = ((word >> (i % 64)) & 1) ? 1.0 : -1.0;
                v += (double)scales[(uint64_t)j * N + z] * sgn;
            }
            n2 += v * v;
        }
        out[z] = sqrt(n2);
    }
}


/* ------------------------------------------------------------------ */
/* Hybrid scoring: a full-precision query against RBE items (the paper's
 * "hybrid rbe" model m_5, Sec. 8.1: 32-bit query, binary keyword).  With
 * q in R^d and the item reconstructed as khat_z = sum_j a_j[z] b_z^j,
 *     s(q, z) = q . khat_z = sum_j a_j[z] * sum_i q[i] * b_z^j[i],
 * evaluated by unpacking every bit (no table, no popcount), in double.     */
/* ------------------------------------------------------------------ */
static double score_pair_fq(const uint64_t *planes, const float *scales, uint64_t N,
                            uint32_t d, uint32_t P, uint64_t z, const float *q)
{
    const uint32_t W = d / 64;
    double s = 0.0;
    for (uint32_t j = 0; j < P; ++j) {
        const uint64_t *kj = planes + ((uint64_t)j * N + z) * W;
        double t = 0.0;
        for (uint32_t i = 0; i < d; ++i)
            t += ((kj[i / 64] >> (i % 64)) & 1) ? (double)q[i] : -(double)q[i];
        s += (double)scales[(uint64_t)j * N + z] * t;
    }
    return s;
}

void orc_scores_fq(const uint64_t *planes, const float *scales, uint64_t N, uint32_t d, uint32_t P,
                   const float *q, uint64_t z0, uint64_t z1, double *out)
{
    for (uint64_t z = z0; z < z1; ++z) out[z - z0] = score_pair_fq(planes, scales, N, d, P, z, q);
}

void orc_scores_at_fq(const uint64_t *planes, const float *scales, uint64_t N, uint32_t d, uint32_t P,
                      const float *q, const int64_t *ids, uint64_t n_ids, double *out)
{
    for (uint64_t r = 0; r < n_ids; ++r)
        out[r] = score_pair_fq(planes, scales, N, d, P, (uint64_t)ids[r], q);
}

int64_t orc_topk_fq(const uint64_t *planes, const float *scales, uint64_t N, uint32_t d, uint32_t P,
                    const float *q, uint64_t z0, uint64_t z1, uint64_t k,
                    int64_t *ids_out, double *scores_out)
{
    topk_t t = { (cand_t *)malloc((k ? k : 1) * sizeof(cand_t)), 0, k };
    if (!t.h) return -1;
    for (uint64_t z = z0; z < z1; ++z)
        topk_offer(&t, score_pair_fq(planes, scales, N, d, P, z, q), (int64_t)z);
    uint64_t n = topk_finish(&t, ids_out, scores_out);
    free(t.h);
    return (int64_t)n;
}
