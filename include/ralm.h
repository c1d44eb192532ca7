/*
 * ralm.h — C ABI of the MI355X (gfx950) retrieval hot path of RaLMSpec
 * (arXiv 2401.14021, "Accelerating Retrieval-augmented Language Model Serving
 * with Speculation").
 *
 * Four operations of the paper's serving loop (Alg. 1) are implemented:
 *
 *   C.retrieve(q_1..q_s)   batched exact knowledge-base retrieval, the
 *                          verification step        -> ralm_retrieve_topk[_ex]
 *   Q.retrieve(q_i)        speculative retrieval from the request's local
 *                          cache, top-1             -> ralm_cache_lookup
 *   m = argmin_i d^_i!=d_i first mis-speculated step -> ralm_verify
 *   Q.insert(C.retrieve(..)) cache update after verification -> ralm_cache_insert
 *
 * and, around that loop: the stride scheduler of Section 4 as host functions
 * (ralm_os3_*), and for KNN-LM datastores (Section 5.3) ranking by distance
 * (RALM_METRIC_L2) and the neighbour distribution (ralm_knnlm_probs).
 *
 * General conventions
 *   - Unless a parameter says "host", every data pointer is a DEVICE pointer
 *     owned by the caller.  The library keeps no reference after the call's
 *     work has run and never frees caller memory.
 *   - Calls enqueue work on the given HIP stream (a hipStream_t passed as
 *     void*; NULL = the default stream) and return without synchronising,
 *     except where stated.  Work of one call is ordered on that stream.
 *     Apart from ralm_retrieve_topk, ralm_workspace_overflows and
 *     ralm_workspace_counters, a call only
 *     launches kernels (no allocation, no memset or copy nodes), so after one
 *     ordinary call of the same shapes (the first launch of a kernel sets its
 *     attributes) it may be recorded into a HIP graph and replayed.
 *   - Matrices are row-major.  ids are int32 row numbers of the datastore
 *     (N <= 2^31 - 512); sizes are int64.  A call takes at most 2^20 queries
 *     and 2^22 requests (RALM_ERR_SHAPE beyond that).
 *   - The ranking is always (score descending, row id ascending): equal scores
 *     go to the lower id.  The paper does not define ties; this is this
 *     library's rule, at every stage.
 *   - The score is the inner product, or minus the squared distance (see
 *     ralm_metric).  Final scores (outputs) are the fp32 rounding of a sum
 *     formed in double from fp32 (or exactly widened fp16/bf16) inputs.
 *   - Argument errors are detected on the host before anything is launched and
 *     are reported as a status; ralm_last_error() gives the text.  Inputs are
 *     assumed finite (NaN/Inf: behaviour unspecified).
 */
#ifndef RALM_H
#define RALM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    RALM_OK = 0,
    RALM_ERR_NULL = 1,      /* a required pointer is NULL */
    RALM_ERR_SHAPE = 2,     /* Q, N, d, R, C or a stride is out of range */
    RALM_ERR_K = 3,         /* k < 1, k > N, k > RALM_MAX_K, k' < k or k' > RALM_MAX_K_PRIME */
    RALM_ERR_DTYPE = 4,     /* dtype tag unknown or not allowed in that slot */
    RALM_ERR_ALIGN = 5,     /* base pointer or row pitch not 16-byte aligned */
    RALM_ERR_WORKSPACE = 6, /* workspace NULL, misaligned or too small */
    RALM_ERR_RANGE = 7,     /* a count (Qt, true_stride) is negative or does not fit */
    RALM_ERR_DEVICE = 8,    /* a HIP call failed (text in ralm_last_error) */
    RALM_ERR_OVERFLOW = 9   /* a candidate buffer overflowed (degenerate input); see below */
} ralm_status;

typedef enum { RALM_F32 = 0, RALM_BF16 = 1, RALM_F16 = 2 } ralm_dtype;

/*
 * Score of a row x for a query q.  RALM_METRIC_IP: the inner product <q, x>
 * (dense passage retrieval).  RALM_METRIC_L2: minus the squared Euclidean
 * distance, -|q - x|^2 (KNN-LM datastores rank their entries by distance,
 * Section 5.3), so that a larger score is a better match under both.
 */
typedef enum { RALM_METRIC_IP = 0, RALM_METRIC_L2 = 1 } ralm_metric;

#define RALM_MAX_K 1024
#define RALM_MAX_K_PRIME 4096

/*
 * The knowledge base as the flat index of an exact dense retriever
 * (Section 5.1, "Retrievers"): N key vectors of dimension d.
 *
 *   exact  the keys that define the right answer: fp32 [N, d], or fp16 [N, d]
 *          (KNN-LM keys; widened exactly).  Scores returned to the caller are
 *          computed from this copy.
 *   scan   the copy the full scan reads: bf16 or fp16 roundings of the exact
 *          keys (build with ralm_build_scan_copy), or the exact copy itself
 *          (fp32 is rounded to bf16 on the fly: at or near the HBM rate for
 *          batches of up to 256 queries, at about half the speed of a bf16
 *          copy for larger ones; fp16 is used as is).
 *          NULL means "use the exact copy".
 *   *_stride  row pitch in ELEMENTS (0 = d).  Pitch in bytes and both base
 *          pointers must be multiples of 16.  d must be a multiple of 8.
 *   metric RALM_METRIC_IP (0) or RALM_METRIC_L2.  With RALM_METRIC_L2 the scan
 *          copy is mandatory, bf16 or fp16, and its rows have d + 8 columns:
 *          the d rounded elements, then the row's squared norm as the sum of
 *          two scan-dtype numbers, then six zeros (ralm_build_scan_copy_l2
 *          writes this layout; scan_stride 0 = d + 8, but a pitch that is a
 *          multiple of 64 elements keeps rows on 128-byte lines and scans
 *          ~20 % faster).  The scan then scores a
 *          row as 2<q, x> - |x|^2 on the matrix cores with no change to its
 *          kernels; final scores are -|q - x|^2 from the exact copy.
 */
typedef struct {
    const void *exact;
    int32_t exact_dtype;    /* RALM_F32 or RALM_F16 */
    const void *scan;       /* may be NULL */
    int32_t scan_dtype;     /* RALM_BF16, RALM_F16 or RALM_F32 */
    int64_t N;
    int32_t d;
    int64_t exact_stride;
    int64_t scan_stride;
    int32_t metric;         /* RALM_METRIC_IP or RALM_METRIC_L2 */
} ralm_datastore_t;

/*
 * Batched exact retrieval, simplest form (Alg. 1, the batched verification
 * step; exact dense retriever of Section 5.1).
 *
 *   queries    device fp32 [Q, d]
 *   datastore  device fp32 [N, d]; it is both the exact and the scanned copy
 *   out_ids    device int32 [Q, k]; out_scores device fp32 [Q, k]; each row
 *              ranked best first.
 *
 * Runs on the default stream and synchronises before returning.  It uses
 * buffers of its own, kept between calls and grown on demand (allocating tens
 * of gigabytes per call is slow); ralm_release_buffers() frees them: the
 * workspace and, for batches of more than 768 queries only, a bf16 copy of the
 * datastore for the scan (N*d*2 bytes, rebuilt on every call; skipped if the
 * device has no room for it).  Batches of up to 768 queries scan the fp32 rows
 * as they are (21M x 768: about 9.3 ms for up to 64 queries, the rate at which
 * HBM delivers the rows; 14 ms for 256, 25 ms for 512), and hold no copy.  Calls are serialised.  Meant for convenience; a caller that
 * retrieves large batches repeatedly keeps a scan copy and uses the full form.
 * A query that the full form would leave unanswered (see
 * ralm_retrieve_topk_ex) makes the call retry through ralm_retrieve_topk_seq;
 * if it is still unanswered the call returns RALM_ERR_OVERFLOW.
 */
ralm_status ralm_retrieve_topk(const float *queries, int64_t Q, const float *datastore, int64_t N,
                               int32_t d, int32_t k, int32_t *out_ids, float *out_scores);

/* Frees the device buffers that ralm_retrieve_topk keeps between calls (synchronises). */
void ralm_release_buffers(void);

/* Bytes of workspace ralm_retrieve_topk_ex needs for (Q, ds, k, k_prime); 0 on bad arguments. */
size_t ralm_workspace_bytes(int64_t Q, const ralm_datastore_t *ds, int32_t k, int32_t k_prime);

/*
 * Batched exact retrieval, full form.  How it gets the exact answer from a
 * low-precision scan: every row is scored in the scan dtype on the matrix
 * cores with fp32 accumulation; per query the k' (>= k) best scan scores are
 * kept; those k' rows are re-scored from the exact copy and the best k of them
 * are returned.  k_prime = 0 picks a default (64 for k <= 32, else the power
 * of two >= 2k).
 *
 * That answer is the exact one unless the scan's rounding pushed a true top-k
 * row out of the k' kept ones.  The library checks this per query, on the
 * device: the margin (see out_margin) must exceed 8x the root mean square of
 * the differences between scan score and exact score seen on the query's own k'
 * candidates (when all of those differences are zero, a margin of zero is
 * enough).  A query that fails the check, or whose candidate list lost entries
 * (below), is answered again in the same call by an exact pass: every row of
 * the exact copy is scored exactly (the arithmetic of the final scores) and the
 * best k of the rows that reach the exact rank-k score found so far are
 * returned, which is the exact top k by construction.  The pass is skipped
 * when no query needs it; it reads the exact copy once per 16 such queries
 * (inner product on the fp64 matrix cores; 21M x 768 fp32: about 11 ms per
 * pass), once per 8 for the squared distance and for row lengths that are not
 * a multiple of 64 (fp32) or 128 (fp16) elements (13 to 26 ms).  With k_prime = k there is
 * no margin to speak of and nearly every query takes that pass.
 * ralm_workspace_counters reports how many did.
 *
 *   queries     device fp32 [Q, d] (host code never reads it)
 *   ds          HOST struct of device pointers
 *   out_ids / out_scores  device [Q, k] as above
 *   out_margin  optional device fp32 [Q] (may be NULL): exact score of the
 *               rank-k row among the candidates minus the scan score of the
 *               k'-th kept candidate (brought to the same scale under
 *               RALM_METRIC_L2).  A row outside the candidates can belong in
 *               the top k only if the scan mis-scored it by at least this
 *               much.  Diagnostic: the library acts on it by itself (above).
 *               +inf when every row was a candidate (N < k').
 *   workspace   device scratch, 256-byte aligned, >= ralm_workspace_bytes();
 *               contents are undefined between calls; two calls that overlap
 *               in time must not share it.
 *   stream      hipStream_t
 *
 * The rows are visited in a fixed strided order, coarse samples first, and a
 * query's candidate list (a fixed number of slots in the workspace) takes only
 * scores that beat the k'-th best of the rows visited before.  Does not
 * synchronise.  If the list of some query overflows (only when the order of
 * the rows is correlated with that stride pattern, e.g. every other 256-row
 * tile holding the best matches), the list keeps what it has, the scan goes
 * on, and the query is answered by the exact pass, whose list holds only rows
 * that reach the exact rank-k score of the candidates that survived.  Only if
 * that list overflows too (more than 16384 rows beat that score, tie with it,
 * or fall short of it by no more than one fp32 step: the pass forms its double
 * sums in another order than the re-score and leaves that much room)
 * are the query's outputs set to id -1 / score NaN; ralm_workspace_overflows()
 * counts those.  (Such a datastore holds tens of thousands of rows that no
 * fp32 score separates from the query's k-th best; a larger k would be the
 * honest request.)
 */
ralm_status ralm_retrieve_topk_ex(const float *queries, int64_t Q, const ralm_datastore_t *ds,
                                  int32_t k, int32_t k_prime, int32_t *out_ids, float *out_scores,
                                  float *out_margin, void *workspace, size_t workspace_bytes,
                                  void *stream);

/*
 * Same arguments, same result as ralm_retrieve_topk_ex, computed block by
 * block over consecutive rows: every block is small enough that a list holds
 * its k' best so far plus every row of the block, so no list can overflow
 * whatever the order of the rows.  About N / 16000 small launches instead of a
 * dozen large ones (21M rows: ~50 ms); meant as the retry after an overflow.
 */
ralm_status ralm_retrieve_topk_seq(const float *queries, int64_t Q, const ralm_datastore_t *ds,
                                   int32_t k, int32_t k_prime, int32_t *out_ids, float *out_scores,
                                   float *out_margin, void *workspace, size_t workspace_bytes,
                                   void *stream);

/*
 * Number of queries of the LAST ralm_retrieve_topk_ex / _seq call on this workspace
 * that were left unanswered (id -1 / score NaN).  Synchronises `stream` and
 * copies one int to the host (*count is a host pointer).
 */
ralm_status ralm_workspace_overflows(const void *workspace, void *stream, int32_t *count);

/*
 * Counters of the LAST ralm_retrieve_topk_ex / _seq call on this workspace, all
 * numbers of queries (host struct; synchronises `stream`):
 *   unanswered        id -1 / score NaN (what ralm_workspace_overflows returns)
 *   ladder_overflows  candidate list lost entries during the scan; answered by
 *                     the exact pass
 *   hard_certified    margin above the deterministic bound of the scan's
 *                     rounding, (u_q + u_x + u_q u_x) |q| |x| + d 2^-24 |q| |x|
 *                     with unit roundoffs u = 2^-8 (bf16) or 2^-11 (fp16) of the
 *                     query and of the rows (0 for rows scanned as they are) and
 *                     |x| the longest of the query's candidates: a proof when
 *                     no row is longer than that, e.g. for unit-norm rows
 *   soft_certified    passed the check described at ralm_retrieve_topk_ex
 *                     (includes hard_certified)
 *   exact_pass        answered by the exact pass
 * soft_certified + exact_pass = Q.
 */
typedef struct {
    int32_t unanswered, ladder_overflows, hard_certified, soft_certified, exact_pass;
} ralm_counters_t;
ralm_status ralm_workspace_counters(const void *workspace, void *stream, ralm_counters_t *out);

/*
 * How full the candidate lists got in the LAST ralm_retrieve_topk_ex / _seq
 * call on this workspace: entries[i] = over all queries, the entries their
 * lists held when stage i of the ladder ended (the at most k' kept from the
 * stages before plus the scores the stage admitted), i < *n_stages; the other
 * elements are set to 0.  entries is a HOST array of RALM_MAX_LADDER_STAGES
 * elements; of a longer ladder (the sequential form) the first
 * RALM_MAX_LADDER_STAGES stages are reported.  Synchronises `stream`.  A
 * diagnostic: with rows in an order that the strided samples represent well a
 * stage that multiplies the rows scanned by g admits about k' (g - 1) scores
 * per query.
 */
#define RALM_MAX_LADDER_STAGES 40
ralm_status ralm_workspace_stage_entries(const void *workspace, void *stream, int32_t *n_stages,
                                         int64_t *entries);

/*
 * Build the low-precision scan copy of a datastore: dst[j, c] = round-to-
 * nearest-even(src[j, c]) in dst_dtype (RALM_BF16 or RALM_F16).  src is device
 * fp32 [N, d] with pitch src_stride elements, dst device [N, d] with pitch
 * dst_stride elements (0 = d for both).
 */
ralm_status ralm_build_scan_copy(const float *src, int64_t src_stride, void *dst, int32_t dst_dtype,
                                 int64_t dst_stride, int64_t N, int32_t d, void *stream);

/*
 * Scan copy for RALM_METRIC_L2: dst[j, 0..d) = round-to-nearest-even(src[j, c])
 * in dst_dtype; dst[j, d] + dst[j, d+1] = |src_j|^2 (summed in double, split
 * into a rounded head and the rounded remainder); dst[j, d+2 .. d+8) = 0.
 * src is device fp32 or fp16 [N, d] (src_dtype), dst device [N, d + 8] bf16 or
 * fp16; strides in elements (0 = d, d + 8).  src == dst is allowed for fp16
 * keys stored with a pitch of at least d + 8 that serve as their own scan
 * copy: then only the 8 extra columns are written.
 */
ralm_status ralm_build_scan_copy_l2(const void *src, int32_t src_dtype, int64_t src_stride, void *dst,
                                    int32_t dst_dtype, int64_t dst_stride, int64_t N, int32_t d,
                                    void *stream);

/*
 * Speculative retrieval from the per-request local caches (Alg. 1, the
 * speculative retrieval step; Section 3 "Speculative retrieval"; Fig. 2: the
 * cache is ranked with the retriever's own metric).  A cache holds datastore
 * row ids; the key is re-read from the exact datastore so that a cached
 * entry's score is the very number the knowledge-base retrieval would give it
 * (this is what makes the cache top-1 equal the knowledge-base top-1 whenever
 * the latter is cached).
 *
 *   cache_ids  device int32 [R, C]; request r owns entries [0, cache_len[r])
 *              of row r; every owned id must be in [0, N) (ids outside are
 *              skipped)
 *   cache_len  device int32 [R]; values are clamped to [0, C]
 *   queries    device fp32 [Qt, d]; request r owns rows q_offsets[r] ..
 *              q_offsets[r+1] (its speculation steps, in order)
 *   q_offsets  device int64 [R+1], non-decreasing, within [0, Qt].  Device
 *              data cannot be checked on the host: the kernel clamps each
 *              range to [0, Qt] and treats a decreasing pair as empty.
 *   spec_ids   device int32 [Qt]: top-1 cached id per query (-1 if the cache
 *              is empty);  spec_scores device fp32 [Qt] (-inf if empty).
 *              Rows of [0, Qt) that no request owns are left untouched.
 *   workspace  optional device scratch (may be NULL) of at least
 *              ralm_cache_lookup_workspace_bytes(Qt) = 8 bytes per query,
 *              8-byte aligned, contents undefined between calls.  Without it
 *              one workgroup serves a request, which leaves most of the chip
 *              idle when there are few requests (a single request with 4096
 *              cached rows then takes ~0.4 ms); with it the caches of fewer
 *              than 128 requests are each split over several workgroups that
 *              merge through the workspace (same results).
 */
size_t ralm_cache_lookup_workspace_bytes(int64_t Qt);
ralm_status ralm_cache_lookup(const int32_t *cache_ids, const int32_t *cache_len, int32_t C, int64_t R,
                              const float *queries, int64_t Qt, const int64_t *q_offsets,
                              const ralm_datastore_t *ds, int32_t *spec_ids, float *spec_scores,
                              void *workspace, size_t workspace_bytes, void *stream);

/*
 * ralm_cache_lookup for callers that can neither allocate device memory nor
 * pass a workspace: code recorded under HIP graph capture, tight serving loops,
 * harnesses that forbid allocation.  Same arguments and same results as
 * ralm_cache_lookup called with a workspace; the merge slots (8 bytes per
 * query) live in an array inside the library instead, 512 KiB per GPU, held
 * until the process ends.  Limit: Qt <= 65536 (RALM_ERR_RANGE beyond it).  The
 * call allocates nothing and only launches kernels (the slots are cleared by a
 * kernel).  All calls on one GPU share that array: two calls that overlap in
 * time on the same GPU (different streams or threads) race; calls ordered on
 * one stream are fine.
 */
#define RALM_STATIC_LOOKUP_MAX_QT 65536
ralm_status ralm_cache_lookup_static(const int32_t *cache_ids, const int32_t *cache_len, int32_t C, int64_t R,
                                     const float *queries, int64_t Qt, const int64_t *q_offsets,
                                     const ralm_datastore_t *ds, int32_t *spec_ids, float *spec_scores,
                                     void *stream);

/*
 * Speculative retrieval of k entries from the local caches (Section 5.3: KNN-LM
 * forms its next-token distribution from k retrieved entries, so its
 * speculation step needs the k best CACHED entries; ranked with the
 * retriever's own metric like every cache retrieval, Section 3 / Fig. 2).
 * Arguments as ralm_cache_lookup, plus
 *
 *   k           1 <= k <= min(C, RALM_MAX_K); C <= RALM_MAX_K_PRIME
 *   out_ids / out_scores  device [Qt, k], best first; ranks beyond the number
 *               of (valid) cached ids get id -1 / score -inf, as do queries
 *               that no request owns
 *   workspace   device scratch, 256-byte aligned, at least
 *               ralm_cache_lookup_topk_workspace_bytes(Qt, C)
 *
 * Cached ids must be distinct within a request (a repeated id is returned
 * repeatedly).  Feeds ralm_knnlm_probs directly.
 */
size_t ralm_cache_lookup_topk_workspace_bytes(int64_t Qt, int32_t C);
ralm_status ralm_cache_lookup_topk(const int32_t *cache_ids, const int32_t *cache_len, int32_t C, int64_t R,
                                   const float *queries, int64_t Qt, const int64_t *q_offsets,
                                   const ralm_datastore_t *ds, int32_t k, int32_t *out_ids,
                                   float *out_scores, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Verification compare (Alg. 1: m = argmin_i d^_i != d_i).  For request r with
 * stride s_r = q_offsets[r+1] - q_offsets[r]:
 *   first_mismatch[r] = min { i in [0, s_r) : spec_ids[q_offsets[r] + i] !=
 *                             true_ids[(q_offsets[r] + i) * true_stride] }
 * or s_r when every step matches (0-based; s_r = 0 gives 0).  true_stride = k
 * reads the rank-0 column of a [Q, k] retrieval result in place.
 *
 *   spec_ids   device int32 [Qt];  true_ids device int32 [Qt * true_stride];
 *   q_offsets  device int64 [R+1] (clamped as in ralm_cache_lookup);
 *   first_mismatch  device int32 [R]
 */
ralm_status ralm_verify(const int32_t *spec_ids, const int32_t *true_ids, int64_t true_stride,
                        int64_t Qt, const int64_t *q_offsets, int64_t R, int32_t *first_mismatch,
                        void *stream);

/*
 * Cache update after a verification step (Alg. 1, Q.insert(C.retrieve(..));
 * Section 3 "Batched verification": top-1 update and top-k update =
 * prefetching, Fig. 2; Section 5.3: for KNN-LM the next n entries after a
 * retrieved one).  The paper's cache has no stated capacity; here a request's
 * cache is a ring of C ids: an id that is already cached is not inserted
 * again, and once all C slots are used the oldest inserted id is overwritten.
 *
 *   cache_ids / cache_len   device int32 [R, C] / [R], as in ralm_cache_lookup;
 *                           updated in place.  Owned ids must be distinct.
 *   cache_head  device int32 [R]: the slot that the next insertion into a FULL
 *               cache overwrites; start with zeros; updated in place.
 *   true_ids    device int32: rank-j id of query q at true_ids[q * true_stride
 *               + j] (the out_ids of a retrieval with k = true_stride)
 *   q_offsets   device int64 [R+1] (clamped as in ralm_cache_lookup)
 *   first_mismatch  device int32 [R] from ralm_verify, or NULL.  Given: only
 *               the steps 0 .. min(first_mismatch[r], s_r - 1) of request r are
 *               taken (the later ones were retrieved for a context that is
 *               rolled back).  NULL: all s_r steps.
 *   p           ranks 0 .. p-1 of each taken step are taken (1 = top-1 update,
 *               20 = the paper's prefetch size); 1 <= p <= true_stride
 *   n_next      0: a taken id t is itself the candidate; n > 0: its successors
 *               t+1 .. t+n are (spatial locality of KNN-LM datastores)
 *   N           candidates outside [0, N) are dropped, as are negative ids
 *
 * Candidates are inserted in the order step, rank, successor; the result is
 * that of doing so one at a time.  Requests are independent (one wave each).
 * Cost per candidate grows with the number of cached ids (linear membership
 * test over the row in LDS); C <= 16384.
 */
ralm_status ralm_cache_insert(int32_t *cache_ids, int32_t *cache_len, int32_t *cache_head, int32_t C,
                              int64_t R, const int32_t *true_ids, int64_t true_stride, int64_t Qt,
                              const int64_t *q_offsets, const int32_t *first_mismatch, int32_t p,
                              int32_t n_next, int64_t N, void *stream);

/*
 * KNN-LM neighbour distribution (Section 5.3: a distribution over the target
 * tokens of the k retrieved entries, computed from their distances).  Input is
 * the output of a retrieval: ids / scores device [Q, k], a larger score being a
 * closer entry.
 *
 *   values       device int32 [N]: target token of every datastore entry
 *   temperature  T > 0; weight_i = exp(score_i / T) / sum_j exp(score_j / T)
 *   out_tokens   device int32 [Q, k]: values[ids]  (-1 for an unfilled entry:
 *                id < 0 or >= N; its weight is 0)
 *   out_weights  device fp32 [Q, k], each row sums to 1
 *   out_top_token / out_top_prob  optional device [Q] (either may be NULL): the
 *                token with the largest summed weight and that sum; the smaller
 *                token id on ties; -1 / 0 for a query without filled entries.
 * Sums and exponentials are formed in double and rounded once to fp32.
 */
ralm_status ralm_knnlm_probs(const int32_t *ids, const float *scores, int64_t Q, int32_t k,
                             const int32_t *values, int64_t N, float temperature, int32_t *out_tokens,
                             float *out_weights, int32_t *out_top_token, float *out_top_prob,
                             void *stream);

/*
 * Optimal speculation stride scheduler, OS^3 (Section 4; estimation of its
 * parameters: Appendix A.2, "Parameter estimation").  Host-only scalar
 * functions; every pointer is a HOST pointer; nothing is launched.
 *
 * ralm_os3_gamma: estimate of the speculation accuracy gamma from the w most
 *   recent verification steps of a request: strides[t] = s(t), matched[t] =
 *   M(s(t)) = number of speculated documents that matched before the first
 *   mismatch (the first_mismatch of ralm_verify):
 *       gamma^ = sum_t M(t) / ( sum_t M(t) + #{t : M(t) < s(t)} ),
 *   truncated at gamma_max (the paper uses w = 5, gamma_max = 0.6).  0 when
 *   there is no history (w <= 0) or nothing matched.
 * ralm_os3_objective: expected verified documents per unit time for stride s,
 *       (1 - gamma^s) / (1 - gamma) / latency(s),
 *   latency(s) = s a + b (synchronous verification; async == 0), or
 *   gamma^s ((s-1) a + max(a, b)) + (1 - gamma^s)(s a + b) (asynchronous),
 *   with a = latency of a speculation step, b = latency of a verification
 *   step.  The expectation is formed as the sum of gamma^i, i < s, so gamma = 1
 *   needs no special case.  NaN for s < 1, negative a or b, gamma outside [0, 1].
 * ralm_os3_stride: the s in [1, s_max] with the largest objective; the
 *   smallest such s on ties.
 * ralm_os3_latency: a (or b) as the mean of the n most recent measurements
 *   (Appendix A.2 estimates both from recent profiling and fixes no window
 *   length); 0 for n <= 0.
 * ralm_os3_next_stride: the stride for the next round from a request's history:
 *   gamma^ from (strides, matched, w), a and b from their samples, then
 *   ralm_os3_stride.  1 while any of the three histories is empty (the paper
 *   starts with s = 1).
 */
double ralm_os3_gamma(const int32_t *strides, const int32_t *matched, int32_t w, double gamma_max);
double ralm_os3_objective(double gamma, double a, double b, int32_t s, int32_t async);
int32_t ralm_os3_stride(double gamma, double a, double b, int32_t s_max, int32_t async);
double ralm_os3_latency(const double *samples, int32_t n);
int32_t ralm_os3_next_stride(const int32_t *strides, const int32_t *matched, int32_t w,
                             const double *a_samples, int32_t n_a, const double *b_samples, int32_t n_b,
                             double gamma_max, int32_t s_max, int32_t async);

/*
 * Asynchronous verification (Section 3, "Asynchronous verification"; latency
 * model of Section 4: a verification that overlaps the next speculation step
 * costs (s-1) a + max(a, b) instead of s a + b).  Every call here is ordered on
 * the caller's stream only, so the batched retrieval of step t and the cache
 * lookup of step t+1 can be issued on two streams.  The scan, however, runs as
 * a persistent grid with one workgroup per compute unit whose LDS it fills, so
 * a kernel on another stream finds no free unit until a scan launch ends.
 * ralm_scan_reserve_cus(n) makes every later retrieval call of the process
 * leave n compute units free (n = 8: one per XCD; 0 restores the default); the
 * scan slows down by about n / 256 and the other stream's kernels run beside
 * it.  Process-wide setting, read when a call is issued.
 */
void ralm_scan_reserve_cus(int32_t n);

/*
 * Timing aid for benchmarks.  While enabled, ralm_retrieve_topk_ex brackets
 * each launch of its scan kernel (a call makes several: together they read
 * every row of the datastore exactly once) with HIP events on the call's
 * stream.  ralm_profile_scan_ms synchronises those events and returns the
 * total milliseconds and the number of bracketed launches since the last
 * reset (host pointers), then resets.  At most 2048 launches are recorded
 * between resets.  Not thread-safe; off by default.
 */
void ralm_profile_enable(int32_t on);
ralm_status ralm_profile_scan_ms(float *total_ms, int32_t *launches);

/* Text of the calling thread's last error (static storage; never NULL). */
const char *ralm_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* RALM_H */
