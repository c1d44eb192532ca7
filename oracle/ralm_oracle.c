/*
 * CPU oracle for the RaLMSpec retrieval hot path.  TEST INFRASTRUCTURE ONLY:
 * it exists so that tests, the smoke check and the benchmark's CPU-baseline leg
 * can say what the right answer is.  It shares no code with the HIP library
 * and the product never calls it.
 *
 * Everything here is the plain definition written out, slow and obvious:
 *
 *  - knowledge-base retrieval C.retrieve(q_1..q_s) of Alg. 1 (the batched
 *    verification step) with the exact dense retriever of Section 5.1
 *    ("Retrievers"): score every datastore row against every query by inner
 *    product, sort ALL rows by (score descending, row id ascending), return the
 *    first k.  Batched retrieval is by definition the same as retrieving for
 *    each query on its own (Section 1: the method preserves the outputs).
 *  - speculative retrieval Q.retrieve(q) of Alg. 1: the same ranking with the
 *    same metric, restricted to the entries of the request's local cache
 *    (Section 3, "Speculative retrieval", and the caption of Fig. 2), top-1.
 *  - the verification compare m = argmin_i (d^_i != d_i) of Alg. 1, per request.
 *  - the cache update Q.insert(C.retrieve(..)) of Alg. 1: the documents that a
 *    verification step retrieved go into the request's local cache (Section 3,
 *    "Batched verification": top-1 update, or top-k update = prefetching,
 *    Fig. 2; Section 5.3: for KNN-LM the next n entries after a retrieved one).
 *  - the stride scheduler OS^3 (Section 4, Appendix A.2): the objective as the
 *    expectation over the distribution of the first mismatch, divided by the
 *    expected latency; the accuracy estimate; the best stride by trying all.
 *  - the KNN-LM neighbour distribution (Section 5.3): weights over the k
 *    retrieved entries from their scores, summed per target token.
 *
 * Readings where the paper is silent:
 *  - metric: inner product (dense passage retrieval scores, raw inner product
 *    for KNN-LM keys);
 *  - ties: equal scores are ordered by the lower row id, everywhere;
 *  - precision: inputs are fp32 (or fp16/bf16 keys widened exactly); each
 *    product is formed in double, the d products are added left to right in
 *    double, and the sum is rounded once to fp32.  Comparisons are made on
 *    that fp32 value;
 *  - first mismatch is reported 0-based, and equals the request's stride when
 *    every speculated id matches;
 *  - the paper's cache has no stated capacity; here it has C slots, an id that
 *    is already cached is not inserted again, and when the slots are full the
 *    oldest inserted id is overwritten (first in, first out).  Results of the
 *    steps after the first mis-speculated one belong to a context that is
 *    rolled back, so they are not inserted when the caller passes the first
 *    mismatch.
 *
 * Threads (OpenMP, if compiled in) only split independent rows between cores;
 * no blocking, no reordering of any sum.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1, ORACLE_F16 = 2 };

typedef struct {
    float score;
    int32_t id;
} scored_t;

/* widen one stored element to fp32 exactly */
static float widen_f16(uint16_t h)
{
    uint32_t sign = (uint32_t)(h >> 15) << 31;
    int exp = (h >> 10) & 0x1F;
    uint32_t man = h & 0x3FF;
    float mag;
    if (exp == 0)
        mag = ldexpf((float)man, -24); /* subnormal or zero */
    else if (exp == 31)
        mag = man ? NAN : INFINITY;
    else
        mag = ldexpf((float)(man | 0x400), exp - 25);
    uint32_t bits;
    memcpy(&bits, &mag, 4);
    bits |= sign;
    memcpy(&mag, &bits, 4);
    return mag;
}

static float widen_bf16(uint16_t b)
{
    uint32_t bits = (uint32_t)b << 16;
    float f;
    memcpy(&f, &bits, 4);
    return f;
}

static float element(const void *X, int dtype, int64_t index)
{
    if (dtype == ORACLE_F32)
        return ((const float *)X)[index];
    if (dtype == ORACLE_F16)
        return widen_f16(((const uint16_t *)X)[index]);
    return widen_bf16(((const uint16_t *)X)[index]);
}

/* <q, x_row>: products and sum in double, one rounding to fp32 */
static float inner_product(const float *q, const void *X, int dtype, int64_t row, int64_t ld,
                           int32_t d)
{
    double sum = 0.0;
    for (int32_t c = 0; c < d; ++c)
        sum += (double)q[c] * (double)element(X, dtype, row * ld + c);
    return (float)sum;
}

/*
 * The squared-distance metric of KNN-LM datastores (Section 5.3: entries are
 * ranked by their distance to the context embedding): the score of a row is
 * minus its squared Euclidean distance to the query, so that "larger score =
 * better" holds for both metrics.  Differences of fp32 values are exact in
 * double; squares and sum in double, left to right, one rounding to fp32.
 */
static float neg_sq_distance(const float *q, const void *X, int dtype, int64_t row, int64_t ld,
                             int32_t d)
{
    double sum = 0.0;
    for (int32_t c = 0; c < d; ++c) {
        double diff = (double)q[c] - (double)element(X, dtype, row * ld + c);
        sum += diff * diff;
    }
    return (float)(-sum);
}

/*
 * The other plausible reading of "fp32 inner product" (the paper does not say how
 * its retriever accumulates): every product rounded to fp32, the d products
 * added left to right in fp32.  Not what the library computes; kept so that
 * tests can count how many answers depend on the reading (only near-ties do).
 */
static float inner_product_f32_sequential(const float *q, const void *X, int dtype, int64_t row,
                                          int64_t ld, int32_t d)
{
    volatile float sum = 0.0f;   /* volatile: every partial sum is rounded to fp32, never kept wider */
    for (int32_t c = 0; c < d; ++c) {
        volatile float prod = q[c] * element(X, dtype, row * ld + c);
        sum = sum + prod;
    }
    return sum;
}

enum { ORACLE_IP = 0, ORACLE_L2 = 1, ORACLE_IP_F32_SEQUENTIAL = 2 };

static float score_of(int metric, const float *q, const void *X, int dtype, int64_t row, int64_t ld,
                      int32_t d)
{
    return metric == ORACLE_L2 ? neg_sq_distance(q, X, dtype, row, ld, d)
                               : inner_product(q, X, dtype, row, ld, d);
}

/* (score descending, id ascending) */
static int by_score_then_id(const void *pa, const void *pb)
{
    const scored_t *a = (const scored_t *)pa, *b = (const scored_t *)pb;
    if (a->score > b->score) return -1;
    if (a->score < b->score) return 1;
    if (a->id < b->id) return -1;
    if (a->id > b->id) return 1;
    return 0;
}

int ralm_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* scores[j] = score of X[j] for j in [0, n): one query against a block of rows */
void ralm_oracle_scores_metric(const float *q, const void *X, int dtype, int64_t n, int32_t d,
                               int64_t ld, int metric, float *scores)
{
    if (metric == ORACLE_IP_F32_SEQUENTIAL) {
#pragma omp parallel for schedule(static)
        for (int64_t j = 0; j < n; ++j)
            scores[j] = inner_product_f32_sequential(q, X, dtype, j, ld, d);
        return;
    }
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < n; ++j)
        scores[j] = score_of(metric, q, X, dtype, j, ld, d);
}

void ralm_oracle_scores(const float *q, const void *X, int dtype, int64_t n, int32_t d,
                        int64_t ld, float *scores)
{
    ralm_oracle_scores_metric(q, X, dtype, n, d, ld, ORACLE_IP, scores);
}

/*
 * Exact dense retrieval: for each of Q queries, all N scores, a full sort,
 * the first k.  out_ids/out_scores are [Q, k] row-major.  Returns 0, or -1 on
 * bad arguments / allocation failure.
 */
int ralm_oracle_retrieve_topk_metric(const float *queries, int64_t Q, const void *X, int dtype,
                                     int64_t N, int32_t d, int64_t ld, int32_t k, int metric,
                                     int32_t *out_ids, float *out_scores)
{
    if (Q < 0 || N < 1 || d < 1 || k < 1 || k > N || ld < d) return -1;
    scored_t *all = (scored_t *)malloc((size_t)N * sizeof(scored_t));
    if (!all) return -1;
    for (int64_t i = 0; i < Q; ++i) {
        const float *q = queries + i * (int64_t)d;
        if (metric == ORACLE_IP_F32_SEQUENTIAL) {
#pragma omp parallel for schedule(static)
            for (int64_t j = 0; j < N; ++j) {
                all[j].score = inner_product_f32_sequential(q, X, dtype, j, ld, d);
                all[j].id = (int32_t)j;
            }
        } else {
#pragma omp parallel for schedule(static)
            for (int64_t j = 0; j < N; ++j) {
                all[j].score = score_of(metric, q, X, dtype, j, ld, d);
                all[j].id = (int32_t)j;
            }
        }
        qsort(all, (size_t)N, sizeof(scored_t), by_score_then_id);
        for (int32_t r = 0; r < k; ++r) {
            out_ids[i * k + r] = all[r].id;
            out_scores[i * k + r] = all[r].score;
        }
    }
    free(all);
    return 0;
}

int ralm_oracle_retrieve_topk(const float *queries, int64_t Q, const void *X, int dtype,
                              int64_t N, int32_t d, int64_t ld, int32_t k, int32_t *out_ids,
                              float *out_scores)
{
    return ralm_oracle_retrieve_topk_metric(queries, Q, X, dtype, N, d, ld, k, ORACLE_IP, out_ids, out_scores);
}

/*
 * Speculative retrieval from the per-request local cache.  Request r owns the
 * row ids cache_ids[r*C .. r*C + cache_len[r]) and the queries
 * q_offsets[r] .. q_offsets[r+1].  For each query: rank the cached rows with
 * the retriever's own metric and take the first.  An empty cache gives id -1
 * and score -inf.
 */
int ralm_oracle_cache_lookup_metric(const int32_t *cache_ids, const int32_t *cache_len, int32_t C,
                                    int64_t R, const float *queries, const int64_t *q_offsets,
                                    const void *X, int dtype, int64_t N, int32_t d, int64_t ld,
                                    int metric, int32_t *spec_ids, float *spec_scores)
{
    if (R < 0 || C < 0 || d < 1 || ld < d) return -1;
    scored_t *ranked = (scored_t *)malloc((size_t)(C > 0 ? C : 1) * sizeof(scored_t));
    if (!ranked) return -1;
    for (int64_t r = 0; r < R; ++r) {
        int32_t len = cache_len[r];
        if (len < 0 || len > C) { free(ranked); return -1; }
        for (int64_t i = q_offsets[r]; i < q_offsets[r + 1]; ++i) {
            const float *q = queries + i * (int64_t)d;
            for (int32_t e = 0; e < len; ++e) {
                int32_t id = cache_ids[r * (int64_t)C + e];
                if (id < 0 || id >= N) { free(ranked); return -1; }
                ranked[e].score = score_of(metric, q, X, dtype, id, ld, d);
                ranked[e].id = id;
            }
            qsort(ranked, (size_t)len, sizeof(scored_t), by_score_then_id);
            spec_ids[i] = len ? ranked[0].id : -1;
            spec_scores[i] = len ? ranked[0].score : -INFINITY;
        }
    }
    free(ranked);
    return 0;
}

int ralm_oracle_cache_lookup(const int32_t *cache_ids, const int32_t *cache_len, int32_t C,
                             int64_t R, const float *queries, const int64_t *q_offsets,
                             const void *X, int dtype, int64_t N, int32_t d, int64_t ld,
                             int32_t *spec_ids, float *spec_scores)
{
    return ralm_oracle_cache_lookup_metric(cache_ids, cache_len, C, R, queries, q_offsets, X, dtype, N, d, ld,
                                           ORACLE_IP, spec_ids, spec_scores);
}

/*
 * Verification compare.  Request r speculated ids spec[q_offsets[r] + i] for
 * its steps i = 0 .. s_r - 1; the knowledge base returned
 * truth[(q_offsets[r] + i) * true_stride] for the same steps.  first_mismatch[r]
 * is the smallest i where they differ, or s_r when none does.
 */
void ralm_oracle_verify(const int32_t *spec, const int32_t *truth, int64_t true_stride,
                        const int64_t *q_offsets, int64_t R, int32_t *first_mismatch)
{
    for (int64_t r = 0; r < R; ++r) {
        int64_t s = q_offsets[r + 1] - q_offsets[r];
        int64_t m = s;
        for (int64_t i = 0; i < s; ++i) {
            int64_t at = q_offsets[r] + i;
            if (spec[at] != truth[at * true_stride]) { m = i; break; }
        }
        first_mismatch[r] = (int32_t)m;
    }
}

/*
 * Cache update after a verification step (Alg. 1, Q.insert; Section 3, "Batched
 * verification": top-1 / top-k update; Section 5.3: next-n update for KNN-LM).
 *
 * Request r holds cache_len[r] ids in cache_ids[r*C ..]; cache_head[r] is the
 * slot that the next insertion into a FULL cache overwrites.  The knowledge
 * base returned truth[(q_offsets[r] + i) * true_stride + j] as the rank-j id of
 * the request's step i.  Steps i = 0 .. n_r - 1 are taken, in order, where
 * n_r = s_r, or min(first_mismatch[r] + 1, s_r) when first_mismatch is given
 * (the steps up to and including the first mis-speculated one: Appendix A.2
 * counts exactly these as verified).  Of each step the ranks j = 0 .. p-1 are
 * taken, in order.  A taken id t stands for the candidates
 *     t                       when n_next == 0   (the document itself)
 *     t+1, t+2, .., t+n_next  when n_next > 0    (its successors in the datastore)
 * Candidates outside [0, N) are dropped.  Each candidate, in that order: if it
 * is in the cache now, nothing happens; else it is written to slot len (and
 * len grows) while len < C, else to slot head, and head moves on cyclically.
 */
void ralm_oracle_cache_insert(int32_t *cache_ids, int32_t *cache_len, int32_t *cache_head, int32_t C,
                              int64_t R, const int32_t *truth, int64_t true_stride,
                              const int64_t *q_offsets, const int32_t *first_mismatch, int32_t p,
                              int32_t n_next, int64_t N)
{
    for (int64_t r = 0; r < R; ++r) {
        int32_t *c = cache_ids + r * (int64_t)C;
        int32_t len = cache_len[r], head = cache_head[r];
        int64_t s = q_offsets[r + 1] - q_offsets[r];
        int64_t n = s;
        if (first_mismatch && (int64_t)first_mismatch[r] + 1 < s) n = (int64_t)first_mismatch[r] + 1;
        for (int64_t i = 0; i < n; ++i) {
            for (int32_t j = 0; j < p; ++j) {
                int64_t t = truth[(q_offsets[r] + i) * true_stride + j];
                int32_t first = n_next > 0 ? 1 : 0, last = n_next > 0 ? n_next : 0;
                for (int32_t o = first; o <= last; ++o) {
                    int64_t e = t + o;
                    if (t < 0 || e < 0 || e >= N) continue;
                    int found = 0;
                    for (int32_t x = 0; x < len; ++x)
                        if (c[x] == (int32_t)e) { found = 1; break; }
                    if (found) continue;
                    if (len < C) {
                        c[len++] = (int32_t)e;
                    } else {
                        c[head] = (int32_t)e;
                        head = head + 1 == C ? 0 : head + 1;
                    }
                }
            }
        }
        cache_len[r] = len;
        cache_head[r] = head;
    }
}

/*
 * OS^3 (Section 4; Appendix A.2).  A speculation step matches with probability
 * gamma, independently.  With stride s the first mismatch is at step i (0-based)
 * with probability gamma^i (1 - gamma), i < s, and there is none with
 * probability gamma^s.  A mismatch at step i verifies i + 1 documents (the i
 * matches and the corrected one); no mismatch verifies s.  The expected number
 * of verified documents is the sum over these s + 1 outcomes.
 */
double ralm_oracle_os3_expected_verified(double gamma, int32_t s)
{
    double e = 0.0;
    for (int32_t i = 0; i < s; ++i) e += (double)(i + 1) * pow(gamma, (double)i) * (1.0 - gamma);
    e += (double)s * pow(gamma, (double)s);
    return e;
}

/*
 * Objective: expected verified documents per unit time.  a = latency of one
 * speculation step, b = latency of one verification step.  Synchronous
 * verification always takes s a + b.  Asynchronous verification overlaps the
 * verification with one more speculation step, (s-1) a + max(a, b), but only
 * when all s steps matched (probability gamma^s); otherwise s a + b.
 */
double ralm_oracle_os3_objective(double gamma, double a, double b, int32_t s, int32_t async)
{
    double all_match = pow(gamma, (double)s);
    double latency = (double)s * a + b;
    if (async)
        latency = all_match * ((double)(s - 1) * a + (a > b ? a : b)) + (1.0 - all_match) * ((double)s * a + b);
    return ralm_oracle_os3_expected_verified(gamma, s) / latency;
}

/* Best stride in [1, s_max] by trying each; the smallest on exact ties. */
int32_t ralm_oracle_os3_stride(double gamma, double a, double b, int32_t s_max, int32_t async)
{
    int32_t best = 1;
    for (int32_t s = 2; s <= s_max; ++s)
        if (ralm_oracle_os3_objective(gamma, a, b, s, async) > ralm_oracle_os3_objective(gamma, a, b, best, async))
            best = s;
    return best;
}

/*
 * Accuracy estimate (Appendix A.2, "Parameter estimation"): over the w most
 * recent verification steps, matched documents / (matched documents + number of
 * steps that ended in a mismatch), truncated at gamma_max.  This is the maximum
 * likelihood estimate for independent trials: every matched document is a
 * success, every step that stopped early contributes exactly one failure.
 */
double ralm_oracle_os3_gamma(const int32_t *strides, const int32_t *matched, int32_t w, double gamma_max)
{
    int64_t successes = 0, failures = 0;
    for (int32_t t = 0; t < w; ++t) {
        successes += matched[t];
        if (matched[t] < strides[t]) failures += 1;
    }
    if (successes + failures == 0) return 0.0;
    double g = (double)successes / (double)(successes + failures);
    return g > gamma_max ? gamma_max : g;
}

/*
 * KNN-LM neighbour distribution (Section 5.3: the k retrieved entries define a
 * distribution over their target tokens through their distances to the context
 * embedding).  Entry i of a query has retrieval score s_i (larger =
 * closer: the inner product, or minus the squared distance) and target token
 * values[ids_i].  Its weight is exp(s_i / T) / sum_j exp(s_j / T); the
 * probability of a token is the sum of the weights of the entries that carry
 * it.  Unfilled entries (id < 0) get token -1 and weight 0.
 *
 * Arithmetic: double; the largest score is subtracted before exp (this changes
 * nothing mathematically); sums run left to right in rank order; weights and
 * the top probability are rounded once to fp32.  top_token is the token with
 * the largest probability (compared in double), the smallest token id on ties;
 * -1 / 0 when the query has no filled entry.
 */
void ralm_oracle_knnlm_probs(const int32_t *ids, const float *scores, int64_t Q, int32_t k,
                             const int32_t *values, double T, int32_t *tokens, float *weights,
                             int32_t *top_token, float *top_prob)
{
    double *e = (double *)malloc(sizeof(double) * (size_t)(k > 0 ? k : 1));
    for (int64_t q = 0; q < Q; ++q) {
        const int32_t *id = ids + q * k;
        const float *sc = scores + q * k;
        int32_t *tok = tokens + q * k;
        float *w = weights + q * k;
        double best = -INFINITY;
        for (int32_t i = 0; i < k; ++i)
            if (id[i] >= 0 && (double)sc[i] > best) best = (double)sc[i];
        double Z = 0.0;
        for (int32_t i = 0; i < k; ++i) {
            e[i] = id[i] >= 0 ? exp(((double)sc[i] - best) / T) : 0.0;
            Z += e[i];
        }
        for (int32_t i = 0; i < k; ++i) {
            tok[i] = id[i] >= 0 ? values[id[i]] : -1;
            e[i] = Z > 0.0 ? e[i] / Z : 0.0;
            w[i] = (float)e[i];
        }
        int32_t arg = -1;
        double argp = 0.0;
        for (int32_t i = 0; i < k; ++i) {
            if (id[i] < 0) continue;
            int seen = 0;
            for (int32_t j = 0; j < i; ++j)
                if (id[j] >= 0 && tok[j] == tok[i]) { seen = 1; break; }
            if (seen) continue;
            double p = 0.0;
            for (int32_t j = i; j < k; ++j)
                if (id[j] >= 0 && tok[j] == tok[i]) p += e[j];
            if (arg < 0 || p > argp || (p == argp && tok[i] < arg)) { arg = tok[i]; argp = p; }
        }
        top_token[q] = arg;
        top_prob[q] = (float)argp;
    }
    free(e);
}

/*
 * Latencies a and b for OS^3 (Appendix A.2 estimates them from the profiled
 * latencies of recent steps; the number of steps is not stated: the same
 * window as for gamma is used): the arithmetic mean of the samples, 0 when
 * there is none.
 */
double ralm_oracle_os3_latency(const double *samples, int32_t n)
{
    if (n <= 0) return 0.0;
    double sum = 0.0;
    for (int32_t i = 0; i < n; ++i) sum += samples[i];
    return sum / (double)n;
}

/*
 * Speculative retrieval of k entries from the local cache (Section 5.3: for
 * KNN-LM the distribution over next tokens is formed from the k retrieved
 * entries, so the speculation step needs the k best CACHED entries, ranked
 * with the retriever's own metric like every cache retrieval: Section 3,
 * Fig. 2).  Per query: score every id the request has cached, sort all of them
 * by (score descending, id ascending), output the first k; ranks beyond the
 * number of cached ids get id -1 and score -inf.  Cached ids outside [0, N) are
 * ignored.
 */
int ralm_oracle_cache_lookup_topk(const int32_t *cache_ids, const int32_t *cache_len, int32_t C,
                                  int64_t R, const float *queries, const int64_t *q_offsets,
                                  const void *X, int dtype, int64_t N, int32_t d, int64_t ld,
                                  int metric, int32_t k, int32_t *out_ids, float *out_scores)
{
    if (R < 0 || C < 0 || d < 1 || ld < d || k < 1) return -1;
    scored_t *ranked = (scored_t *)malloc((size_t)(C > 0 ? C : 1) * sizeof(scored_t));
    if (!ranked) return -1;
    for (int64_t r = 0; r < R; ++r) {
        int32_t len = cache_len[r];
        if (len < 0 || len > C) { free(ranked); return -1; }
        for (int64_t i = q_offsets[r]; i < q_offsets[r + 1]; ++i) {
            const float *q = queries + i * (int64_t)d;
            int32_t n = 0;
            for (int32_t e = 0; e < len; ++e) {
                int32_t id = cache_ids[r * (int64_t)C + e];
                if (id < 0 || id >= N) continue;
                ranked[n].score = score_of(metric, q, X, dtype, id, ld, d);
                ranked[n].id = id;
                ++n;
            }
            qsort(ranked, (size_t)n, sizeof(scored_t), by_score_then_id);
            for (int32_t j = 0; j < k; ++j) {
                out_ids[i * k + j] = j < n ? ranked[j].id : -1;
                out_scores[i * k + j] = j < n ? ranked[j].score : -INFINITY;
            }
        }
    }
    free(ranked);
    return 0;
}
