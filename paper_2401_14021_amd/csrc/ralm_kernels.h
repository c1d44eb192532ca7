// Launchers of the retrieval kernels (internal to libralm.so).  Every launcher only
// enqueues work on `stream`; argument validation happens in the C-ABI layer.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ralm {

typedef unsigned long long u64;

constexpr int SCAN_BM = 256;       // datastore rows per tile of the stage ladder (a workgroup takes one, or half of one)
constexpr int SCAN_BK = 64;        // reduction elements staged per pipeline step
constexpr int SCAN_QPAD = 256;     // query matrix is zero-padded to a multiple of this

struct ScanParams {
    const void *X;          // scan copy [N, ldx]
    int64_t ldx;            // elements
    int64_t N;
    int32_t d;              // reduction length: columns of X that are scored (multiple of 8)
    int32_t in_dtype;       // DT_* of X
    const uint16_t *Qs;     // converted queries [Qpad, dpad], zero padded
    int32_t dpad;           // multiple of SCAN_BK
    int32_t Q;
    const u64 *tau;         // [Q] admission keys (0 = admit everything)
    u64 *cand;              // [Q, cap]
    uint32_t *cnt;          // [Q]
    uint32_t cap;
    int64_t n_row_tiles;    // tiles visited in this stage
    int64_t tile_stride;    // visited tile t is datastore tile (tile_begin + m(t)) * tile_stride, where m(t) = t
    int32_t tile_skip;      // if tile_skip == 0, else the t-th positive integer that is no multiple of tile_skip
    int64_t tile_begin;
    int32_t park_pushes;    // 1: thresholds are selective, collect admitted scores in LDS first
    int32_t lists_empty;    // 1 (with park_pushes == 0): every list is empty and every score of this launch is
                            // kept, so list positions follow from the row's place in the launch (no atomics)
};

// query tile width chosen for Q
int scan_bn_for(int64_t Q);
hipError_t launch_scan(const ScanParams &p, int n_cu, hipStream_t stream);

hipError_t launch_fill_u32(uint32_t *p, uint32_t v, int64_t n, hipStream_t stream);
hipError_t launch_fill_u64(u64 *p, u64 v, int64_t n, hipStream_t stream);

// fp32 [Q, d] -> scan dtype [Qpad, dpad], zero padded
// also clears the n0 words at z0 and the n1 words at z1
hipError_t launch_query_prep(const float *q, int64_t Q, int32_t d, uint16_t *out, int64_t Qpad,
                             int32_t dpad, int32_t scan_dtype, int32_t metric, uint32_t *z0, int64_t n0,
                             uint32_t *z1, int64_t n1, hipStream_t stream);
hipError_t launch_l2_scan_copy(const void *src, int32_t src_dtype, int64_t src_ld, void *dst, int32_t dst_dtype,
                               int64_t dst_ld, int64_t N, int32_t d, hipStream_t stream);

hipError_t launch_convert_rows(const float *src, int64_t src_ld, void *dst, int32_t dst_dtype,
                               int64_t dst_ld, int64_t N, int32_t d, hipStream_t stream);

// A retrieval call's flag block (first FLAG_BLOCK_BYTES of its workspace): 32-bit words FLAG_*,
// counts of queries; from byte STAGE_SUMS_BYTE on, one 64-bit sum per ladder stage (entries that
// the lists held when the stage ended, over all queries).
constexpr int FLAG_BLOCK_BYTES = 1024, STAGE_SUMS_BYTE = 256, MAX_STAGE_SUMS = 40;
enum {
    FLAG_UNANSWERED = 0,        // answered with id -1 / score NaN
    FLAG_LADDER_OVERFLOWS = 1,  // candidate list lost entries during the scan (answered by the exact pass)
    FLAG_HARD_CERTIFIED = 2,    // margin above the deterministic rounding bound
    FLAG_SOFT_CERTIFIED = 3,    // margin above 8x the rounding spread seen on the candidates (includes the above)
    FLAG_FALLBACKS = 4,         // answered by the exact pass
    FLAG_STAGES = 5             // stages of the ladder whose sums were recorded
};

// What the re-score needs to check its own result and to queue a query for the exact pass; all
// pointers NULL: no check (flags == NULL decides).
struct CertifyParams {
    int32_t *flags;        // flag block
    const uint32_t *lost;  // [Q] != 0: the query's list lost entries during the scan
    uint32_t *cnt_rw;      // [Q] list lengths, reset for queued queries
    u64 *tau_exact;        // [Q] out: exact rank-k key of the queued query
    int32_t *fb_list;      // [Q] out: queued queries
    float u_query, u_rows; // unit roundoff applied by the scan to the query / to the rows (0: not rounded)
};

// per query: k'-th best key of cand[q, 0..cnt[q]) -> tau[q]; the list is then cut down, in place,
// to its k' best keys (cnt[q] <- min(cnt[q], k')).  tmp is scratch of [Q, k'] keys.  A list
// that was sent more than cap keys holds the first cap of them: lost[q] is set and the query
// counted once in flags[FLAG_LADDER_OVERFLOWS].
// stage >= 0: the lists' lengths before the cut are added to the stage's sum in the flag block.
hipError_t launch_select(u64 *cand, uint32_t *cnt, uint32_t cap, int32_t k_prime, int64_t Q, u64 *tau,
                         u64 *tmp, uint32_t *lost, int32_t *flags, int32_t stage, hipStream_t stream);

// per query: exact scores of the (at most k') rows left in its list, final ranking, top k out;
// with cert.flags: the result is checked and queries that fail are queued for launch_exact_pass
hipError_t launch_rescore(const u64 *cand, const uint32_t *cnt, uint32_t cap, int32_t k_prime,
                          const float *queries, int64_t Q, const void *exact, int32_t exact_dtype, int64_t ld,
                          int32_t d, int32_t metric, int32_t k, int32_t *out_ids, float *out_scores,
                          float *out_margin, const CertifyParams &cert, hipStream_t stream);

// exact scan + final ranking for the queries queued by the re-score (two launches that return at
// once when none is queued)
hipError_t launch_exact_pass(const float *queries, int64_t Q, const void *exact, int32_t exact_dtype, int64_t ld,
                             int64_t N, int32_t d, int32_t metric, int32_t k, const int32_t *fb_list, int32_t *flags,
                             const u64 *tau_exact, u64 *cand, uint32_t *cnt, uint32_t cap, int32_t *out_ids,
                             float *out_scores, int n_cu, hipStream_t stream);

hipError_t launch_cache_lookup(const int32_t *cache_ids, const int32_t *cache_len, int32_t C, int64_t R,
                               const float *queries, int64_t Qt, const int64_t *q_offsets,
                               const void *exact, int32_t exact_dtype, int64_t ld, int64_t N, int32_t d,
                               int32_t metric, int32_t *spec_ids, float *spec_scores, u64 *partial,
                               hipStream_t stream);

constexpr int CACHE_INSERT_MAX_C = 16384;   // a request's cache row is held in LDS during an update
hipError_t launch_cache_insert(int32_t *cache_ids, int32_t *cache_len, int32_t *cache_head, int32_t C, int64_t R,
                               const int32_t *truth, int64_t true_stride, int64_t Qt, const int64_t *q_offsets,
                               const int32_t *first_mismatch, int32_t p, int32_t n_next, int64_t N,
                               hipStream_t stream);
hipError_t launch_knnlm_probs(const int32_t *ids, const float *scores, int64_t Q, int32_t k, const int32_t *values,
                              int64_t N, double T, int32_t *tokens, float *weights, int32_t *top_token,
                              float *top_prob, hipStream_t stream);
// keys[q, 0..cnt[q]) = ranking keys (score 0) of the valid ids cached by the request that owns query q
hipError_t launch_cache_keys(const int32_t *cache_ids, const int32_t *cache_len, int32_t C, int64_t R, int64_t Qt,
                             const int64_t *q_offsets, int64_t N, u64 *keys, uint32_t *cnt, hipStream_t stream);
hipError_t launch_verify(const int32_t *spec, const int32_t *truth, int64_t true_stride, int64_t Qt,
                         const int64_t *q_offsets, int64_t R, int32_t *first_mismatch,
                         hipStream_t stream);

}  // namespace ralm
