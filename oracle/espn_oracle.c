/*
 * CPU oracle for the late-interaction re-ranking path: candidate gather through
 * CSR offsets, MaxSim score (Eq. 1, Sec. 2.1), ranked top-k (Sec. 2.1: the
 * re-ranking stage sorts candidates by score).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is the slow, plain definition the GPU path
 * is checked against; only the tests, the smoke check and the benchmark's
 * cpu_baseline leg may call it.  It shares no code with the HIP library.
 *
 * Everything is evaluated in IEEE double on the 16-bit inputs widened exactly
 * (Sec. 3.1 fixes the stored vectors at 16 bits; nothing else is rounded).
 * Loops run in index order; there is no blocking or reordering, so each
 * function can be read against Eq. 1 by eye.  The only concurrency is an
 * OpenMP "parallel for" over (query, candidate) pairs, each of which is computed
 * by one thread on its own, so the thread count does not change any result.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Widen one IEEE-754 binary16 bit pattern to double, exactly.
 * sign(1) exponent(5, bias 15) fraction(10). */
double espn_oracle_half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int expo = (h >> 10) & 0x1f;
    int frac = h & 0x3ff;
    double v;
    if (expo == 0) {
        v = ldexp((double)frac, -24);              /* zero and subnormals: frac * 2^-10 * 2^-14 */
    } else if (expo == 31) {
        v = frac ? NAN : INFINITY;
    } else {
        v = ldexp((double)(1024 + frac), expo - 25); /* (1 + frac/1024) * 2^(expo-15) */
    }
    return sign ? -v : v;
}

/*
 * Eq. 1 for one (query, document) pair.
 *   q    : Q rows of d binary16 values (the query embedding matrix E_q)
 *   doc  : t rows of d binary16 values (the document embedding matrix E_d)
 * Returns sum over query rows i of max over document rows j of <q_i, doc_j>.
 * A document with no rows has an empty max, taken as -infinity.
 */
double espn_oracle_maxsim_pair(const uint16_t *q, int32_t Q,
                               const uint16_t *doc, int64_t t, int32_t d)
{
    /* widen both matrices once (exact), then evaluate Eq. 1 as written */
    double *qd = (double *)malloc(sizeof(double) * ((size_t)Q * d + 1));
    double *dd = (double *)malloc(sizeof(double) * ((size_t)t * d + 1));
    if (!qd || !dd) { free(qd); free(dd); return NAN; }
    for (int64_t x = 0; x < (int64_t)Q * d; ++x) qd[x] = espn_oracle_half_to_double(q[x]);
    for (int64_t x = 0; x < t * d; ++x) dd[x] = espn_oracle_half_to_double(doc[x]);

    double score = 0.0;
    for (int32_t i = 0; i < Q; ++i) {
        double best = -INFINITY;
        for (int64_t j = 0; j < t; ++j) {
            double dot = 0.0;
            for (int32_t c = 0; c < d; ++c) dot += qd[(int64_t)i * d + c] * dd[j * d + c];
            if (dot > best) best = dot;
        }
        score += best;
    }
    free(qd);
    free(dd);
    return score;
}

/*
 * Scores of every candidate of every query.
 *   emb     : packed table, [total_tokens, d] binary16, row-major
 *   offsets : [n_docs + 1] row offsets; document id owns rows offsets[id] .. offsets[id+1]-1
 *   q       : [B, Q, d] binary16
 *   cand    : [B, K] document ids
 *   scores  : [B, K] out
 * Returns 0, or -1 if a candidate id is outside [0, n_docs) (nothing is written for it).
 */
int espn_oracle_scores(const uint16_t *emb, const int64_t *offsets, int64_t n_docs, int32_t d,
                       const uint16_t *q, const int64_t *cand,
                       int32_t B, int32_t Q, int32_t K, double *scores, int32_t threads)
{
    int bad = 0;
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
#else
    (void)threads;
#endif
#pragma omp parallel for collapse(2) schedule(dynamic, 16) reduction(| : bad)
    for (int32_t b = 0; b < B; ++b) {
        for (int32_t kk = 0; kk < K; ++kk) {
            int64_t id = cand[(int64_t)b * K + kk];
            if (id < 0 || id >= n_docs) { bad |= 1; continue; }
            int64_t s = offsets[id], e = offsets[id + 1];
            scores[(int64_t)b * K + kk] =
                espn_oracle_maxsim_pair(q + (int64_t)b * Q * d, Q, emb + s * d, e - s, d);
        }
    }
    return bad ? -1 : 0;
}

typedef struct { double score; int64_t id; int32_t slot; } ranked_t;

/* Ranking order: higher score first; equal scores: lower document id first;
 * identical (score, id): lower candidate slot first (the two are indistinguishable
 * in the output, the slot only makes the order total). */
static int ranked_cmp(const void *pa, const void *pb)
{
    const ranked_t *a = (const ranked_t *)pa, *b = (const ranked_t *)pb;
    if (a->score > b->score) return -1;
    if (a->score < b->score) return 1;
    if (a->id < b->id) return -1;
    if (a->id > b->id) return 1;
    return (a->slot > b->slot) - (a->slot < b->slot);
}

/*
 * Ranked list: per query, sort all K candidates by the order above and emit the first k.
 *   scores [B,K], cand [B,K]  ->  out_ids [B,k], out_scores [B,k]
 * Scores must not be NaN.  Returns 0, or -1 if k is outside [0, K] or memory runs out.
 */
int espn_oracle_topk(const double *scores, const int64_t *cand, int32_t B, int32_t K, int32_t k,
                     int64_t *out_ids, double *out_scores)
{
    if (k < 0 || k > K) return -1;
    ranked_t *r = (ranked_t *)malloc(sizeof(ranked_t) * (size_t)(K > 0 ? K : 1));
    if (!r) return -1;
    for (int32_t b = 0; b < B; ++b) {
        for (int32_t kk = 0; kk < K; ++kk) {
            r[kk].score = scores[(int64_t)b * K + kk];
            r[kk].id = cand[(int64_t)b * K + kk];
            r[kk].slot = kk;
        }
        qsort(r, (size_t)K, sizeof(ranked_t), ranked_cmp);
        for (int32_t j = 0; j < k; ++j) {
            out_ids[(int64_t)b * k + j] = r[j].id;
            out_scores[(int64_t)b * k + j] = r[j].score;
        }
    }
    free(r);
    return 0;
}

/* The whole path: scores, then ranked top-k.  all_scores ([B,K]) may be NULL. */
int espn_oracle_rerank(const uint16_t *emb, const int64_t *offsets, int64_t n_docs, int32_t d,
                       const uint16_t *q, const int64_t *cand,
                       int32_t B, int32_t Q, int32_t K, int32_t k,
                       int64_t *out_ids, double *out_scores, double *all_scores, int32_t threads)
{
    double *tmp = all_scores;
    if (!tmp) {
        tmp = (double *)malloc(sizeof(double) * (size_t)B * (size_t)K + 8);
        if (!tmp) return -1;
    }
    int rc = espn_oracle_scores(emb, offsets, n_docs, d, q, cand, B, Q, K, tmp, threads);
    if (rc == 0) rc = espn_oracle_topk(tmp, cand, B, K, k, out_ids, out_scores);
    if (!all_scores) free(tmp);
    return rc;
}

/*
 * Score aggregation (Sec. 3.1): the MaxSim score of a candidate is combined with the score the
 * candidate generator gave it, through a scaling factor:  total = S + alpha * prior.
 *   prior : [B, K] binary32 first-stage scores (widened exactly), alpha a plain argument.
 */
int espn_oracle_scores_prior(const uint16_t *emb, const int64_t *offsets, int64_t n_docs, int32_t d,
                             const uint16_t *q, const int64_t *cand, const float *prior, double alpha,
                             int32_t B, int32_t Q, int32_t K, double *scores, int32_t threads)
{
    int rc = espn_oracle_scores(emb, offsets, n_docs, d, q, cand, B, Q, K, scores, threads);
    if (rc != 0) return rc;
    for (int64_t x = 0; x < (int64_t)B * K; ++x) scores[x] = scores[x] + alpha * (double)prior[x];
    return 0;
}

/*
 * Partial re-ranking (Sec. 4.4).  The candidate list of a query arrives in the first stage's order,
 * best first.  Only its first R entries are scored with MaxSim and sorted by that score; the other
 * K - R entries are appended behind them in the order they came.  The first k entries of the
 * resulting list are written out.  Entries that were not re-ranked carry no MaxSim score: NaN.
 *   cand [B,K]  ->  out_ids [B,k], out_scores [B,k];  0 <= R <= K, 0 <= k <= K.
 */
int espn_oracle_rerank_partial(const uint16_t *emb, const int64_t *offsets, int64_t n_docs, int32_t d,
                               const uint16_t *q, const int64_t *cand,
                               int32_t B, int32_t Q, int32_t K, int32_t R, int32_t k,
                               int64_t *out_ids, double *out_scores, int32_t threads)
{
    if (R < 0 || R > K || k < 0 || k > K) return -1;
    int64_t *head = (int64_t *)calloc((size_t)B * R + 1, sizeof(int64_t));
    int64_t *ids = (int64_t *)malloc(sizeof(int64_t) * ((size_t)B * R + 1));
    double *top = (double *)malloc(sizeof(double) * ((size_t)B * R + 1));
    if (!head || !ids || !top) { free(head); free(ids); free(top); return -1; }
    for (int32_t b = 0; b < B; ++b)
        for (int32_t j = 0; j < R; ++j) head[(int64_t)b * R + j] = cand[(int64_t)b * K + j];
    /* the first R candidates, fully ranked among themselves */
    int rc = espn_oracle_rerank(emb, offsets, n_docs, d, q, head, B, Q, R, R, ids, top, NULL, threads);
    if (rc == 0) {
        for (int32_t b = 0; b < B; ++b)
            for (int32_t j = 0; j < k; ++j) {
                if (j < R) {
                    out_ids[(int64_t)b * k + j] = ids[(int64_t)b * R + j];
                    out_scores[(int64_t)b * k + j] = top[(int64_t)b * R + j];
                } else {
                    out_ids[(int64_t)b * k + j] = cand[(int64_t)b * K + j];
                    out_scores[(int64_t)b * k + j] = NAN;
                }
            }
    }
    free(head); free(ids); free(top);
    return rc;
}

/*
 * Merging two scored lists of one query (Sec. 4.3: the documents re-ranked early by the
 * prefetcher and those re-ranked afterwards are combined by sorting on the score).
 *   a: ids_a/sc_a [B,ka], b: ids_b/sc_b [B,kb]  ->  the first k of their union in ranking order.
 */
int espn_oracle_merge(const int64_t *ids_a, const double *sc_a, int32_t ka,
                      const int64_t *ids_b, const double *sc_b, int32_t kb,
                      int32_t B, int32_t k, int64_t *out_ids, double *out_scores)
{
    const int32_t n = ka + kb;
    if (ka < 0 || kb < 0 || k < 0 || k > n) return -1;
    int64_t *ids = (int64_t *)malloc(sizeof(int64_t) * ((size_t)B * n + 1));
    double *sc = (double *)malloc(sizeof(double) * ((size_t)B * n + 1));
    if (!ids || !sc) { free(ids); free(sc); return -1; }
    for (int32_t b = 0; b < B; ++b) {
        for (int32_t j = 0; j < ka; ++j) {
            ids[(int64_t)b * n + j] = ids_a[(int64_t)b * ka + j];
            sc[(int64_t)b * n + j] = sc_a[(int64_t)b * ka + j];
        }
        for (int32_t j = 0; j < kb; ++j) {
            ids[(int64_t)b * n + ka + j] = ids_b[(int64_t)b * kb + j];
            sc[(int64_t)b * n + ka + j] = sc_b[(int64_t)b * kb + j];
        }
    }
    int rc = espn_oracle_topk(sc, ids, B, n, k, out_ids, out_scores);
    free(ids); free(sc);
    return rc;
}

/*
 * Eq. 4: the largest query batch whose embedding fetch still fits the time it may hide behind,
 *   threshold = bandwidth * budget / (data size per query).
 */
double espn_oracle_batch_threshold(double bandwidth_bytes_per_s, double budget_s, double bytes_per_query)
{
    return bandwidth_bytes_per_s * budget_s / bytes_per_query;
}

/*
 * Compressed table (Sec. 6: newer 8-bit formats shrink the re-ranking index, which lowers the data
 * size per query of Eq. 4).  A token vector is stored as d codes of the 8-bit floating-point format
 * E4M3 of the OCP 8-bit floating point specification (1 sign bit, 4 exponent bits with bias 7,
 * 3 fraction bits; no infinities; S.1111.111 is NaN), and every document carries one positive
 * scale: the stored vector is  scale[doc] * decode(code).
 */
double espn_oracle_e4m3_to_double(uint8_t c)
{
    int sign = (c >> 7) & 1;
    int expo = (c >> 3) & 0xf;
    int frac = c & 0x7;
    double v;
    if (expo == 15 && frac == 7) v = NAN;
    else if (expo == 0) v = ldexp((double)frac, -9);          /* subnormal: frac/8 * 2^-6 */
    else v = ldexp((double)(8 + frac), expo - 10);            /* (1 + frac/8) * 2^(expo-7) */
    return sign ? -v : v;
}

/* Eq. 1 on a compressed table: same loops as espn_oracle_maxsim_pair on the decoded rows; the
 * document's scale multiplies every one of its dot products. */
int espn_oracle_scores_e4m3(const uint8_t *codes, const float *doc_scale, const int64_t *offsets,
                            int64_t n_docs, int32_t d, const uint16_t *q, const int64_t *cand,
                            int32_t B, int32_t Q, int32_t K, double *scores, int32_t threads)
{
    int bad = 0;
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
#else
    (void)threads;
#endif
#pragma omp parallel for collapse(2) schedule(dynamic, 16) reduction(| : bad)
    for (int32_t b = 0; b < B; ++b) {
        for (int32_t kk = 0; kk < K; ++kk) {
            int64_t id = cand[(int64_t)b * K + kk];
            if (id < 0 || id >= n_docs) { bad |= 1; continue; }
            int64_t s = offsets[id], e = offsets[id + 1];
            double scale = (double)doc_scale[id];
            /* widen the query and the document once (exact decode, then the scale), then Eq. 1 as written */
            double *qd = (double *)malloc(sizeof(double) * ((size_t)Q * d + 1));
            double *dd = (double *)malloc(sizeof(double) * ((size_t)(e - s) * d + 1));
            double score = NAN;
            if (qd && dd) {
                for (int64_t x = 0; x < (int64_t)Q * d; ++x)
                    qd[x] = espn_oracle_half_to_double(q[(int64_t)b * Q * d + x]);
                for (int64_t x = 0; x < (e - s) * d; ++x)
                    dd[x] = scale * espn_oracle_e4m3_to_double(codes[s * d + x]);
                score = 0.0;
                for (int32_t i = 0; i < Q; ++i) {
                    double best = -INFINITY;
                    for (int64_t j = 0; j < e - s; ++j) {
                        double dot = 0.0;
                        for (int32_t c = 0; c < d; ++c) dot += qd[(int64_t)i * d + c] * dd[j * d + c];
                        if (dot > best) best = dot;
                    }
                    score += best;
                }
            }
            free(qd);
            free(dd);
            scores[(int64_t)b * K + kk] = score;
        }
    }
    return bad ? -1 : 0;
}

/* Number of threads the parallel loop over queries will use (for reporting). */
int32_t espn_oracle_max_threads(void)
{
#ifdef _OPENMP
    return (int32_t)omp_get_max_threads();
#else
    return 1;
#endif
}
