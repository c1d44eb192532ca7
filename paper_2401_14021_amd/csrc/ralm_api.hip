// C ABI of the retrieval library: argument checks (all on the host, before any launch),
// workspace carve-up, stage planning and kernel sequencing.  See include/ralm.h for the
// contract of every entry point.
//
// How one ralm_retrieve_topk_ex call runs (everything on the caller's stream):
//   1. queries are rounded to the scan dtype into a zero-padded matrix;
//   2. the datastore's 256-row tiles are scanned exactly once, in a ladder of stages that
//      visit them in a progressively finer strided order: stage 0 visits every s0-th tile and
//      keeps every score (s0 is chosen so that they fit the candidate lists); stage i visits
//      the tiles at stride s0/g^i that no earlier stage visited.  After each stage the exact
//      k'-th best key of everything scanned so far becomes the admission key of the next
//      stage (a valid lower bound on the final k'-th best, because the scanned rows are a
//      subset of all rows) and each list is cut down to its k' best.  Every stage's rows are
//      a representative sample, so a stage admits only about k'*(g-1) scores per query.
//   3. the k' keys left in each list are re-scored from the exact copy and ranked.
#include <hip/hip_runtime.h>
#include <atomic>
#include <mutex>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include "../../include/ralm.h"
#include "ralm_common.h"
#include "ralm_kernels.h"

using namespace ralm;

namespace {

thread_local char g_err[512] = "";

ralm_status fail(ralm_status st, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return st;
}

#define RALM_HIP(call)                                                                          \
    do {                                                                                        \
        hipError_t e_ = (call);                                                                 \
        if (e_ != hipSuccess)                                                                   \
            return fail(RALM_ERR_DEVICE, "%s failed: %s", #call, hipGetErrorString(e_));        \
    } while (0)

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
size_t up256(size_t x) { return (x + 255) & ~(size_t)255; }
int elem_bytes(int dt) { return dt == RALM_F32 ? 4 : 2; }

// ---- stage plan ---------------------------------------------------------------------------
struct Plan {
    int32_t k_prime;
    uint32_t cap;         // candidate slots per query
    int64_t Qpad;
    int32_t dpad;
    int n_stages;
    int64_t stride[40];   // tile stride of each stage, first = coarsest, last = 1
    // workspace offsets
    size_t off_q, off_tau, off_cnt, off_lost, off_fb, off_flags, off_cand, off_sel, total;
};

// columns of a scan-copy row: the squared-distance metric keeps the row's squared norm behind it
// one workgroup per request (or per four): keeps every launch below 2^32 work-items
constexpr int64_t MAX_REQUESTS = 1 << 22;

int32_t scan_cols(const ralm_datastore_t *ds) { return ds->d + (ds->metric == RALM_METRIC_L2 ? L2_EXTRA_COLS : 0); }

int32_t default_k_prime(int32_t k)
{
    if (k <= 32) return 64;
    int32_t kp = 64;
    while (kp < 2 * k) kp <<= 1;
    return kp;
}

ralm_status make_plan(int64_t Q, const ralm_datastore_t *ds, int32_t k, int32_t k_prime, Plan &pl)
{
    if (k_prime == 0) k_prime = default_k_prime(k);
    if (k < 1 || k > RALM_MAX_K || (int64_t)k > ds->N)
        return fail(RALM_ERR_K, "k=%d must be in [1, min(N, %d)]", k, RALM_MAX_K);
    if (k_prime < k || k_prime > RALM_MAX_K_PRIME)
        return fail(RALM_ERR_K, "k_prime=%d must be in [k, %d]", k_prime, RALM_MAX_K_PRIME);
    pl.k_prime = k_prime;
    // Stage strides, finest first: 1, then multiplied by the stage's growth until a stage is
    // small enough to keep every score (that one is stage 0).  A stage that refines by g is
    // expected to admit k'*(g-1) scores per query.  Large batches are limited by the matrix
    // cores and by the rare path of the selection, so their big last stages refine in steps
    // of 2; small batches are limited by HBM and prefer few launches.
    // With a large k' (KNN-LM: 2048) a stage that refines by 8 admits 7 k' scores per query, more
    // than its rows are worth: such batches refine by 2 throughout (100M x 1024, Q = 256: 2 %
    // faster although the ladder has 14 stages instead of 7).
    const int32_t g_fine = 2, g_coarse = Q > 64 ? (k_prime > 256 ? 2 : 8) : (k_prime <= 256 ? 64 : 32);
    const int64_t fine_until = Q > 64 ? 8 : 1;    // strides below this refine by g_fine
    // the slots leave 4x (2x for large k') head room over that expectation, far beyond the
    // spread of the count for rows in random order, and are never fewer than 16384 so that
    // stage 0 can be a real sample
    const int64_t safety = k_prime <= 256 ? 4 : 2;
    pl.cap = (uint32_t)(safety * k_prime * (g_coarse - 1) + k_prime);
    if (pl.cap < 16384u) pl.cap = 16384u;
    pl.cap = (pl.cap + 1u) & ~1u;   // even: lists start on 16-byte boundaries
    pl.Qpad = (Q + SCAN_QPAD - 1) / SCAN_QPAD * SCAN_QPAD;
    pl.dpad = (scan_cols(ds) + SCAN_BK - 1) / SCAN_BK * SCAN_BK;

    const int64_t tiles = (ds->N + SCAN_BM - 1) / SCAN_BM;
    auto fits = [&](int64_t s) { return ((tiles + s - 1) / s) * SCAN_BM <= (int64_t)pl.cap; };
    int64_t rev[40];
    int n = 0;
    int64_t s = 1;
    rev[n++] = s;
    while (!fits(s)) {
        const int32_t g = s < fine_until ? g_fine : g_coarse;
        int32_t f = 2;
        while (f < g && !fits(s * f)) ++f;     // the coarsest step may be shorter
        s *= f;
        rev[n++] = s;
    }
    pl.n_stages = n;
    for (int i = 0; i < n; ++i) pl.stride[i] = rev[n - 1 - i];

    size_t off = 0;
    pl.off_flags = off;  off += FLAG_BLOCK_BYTES;   // always first: the counters of the last call (FLAG_*)
    pl.off_q = off;      off += up256((size_t)pl.Qpad * pl.dpad * 2);
    pl.off_tau = off;    off += up256((size_t)pl.Qpad * 8);
    pl.off_cnt = off;    off += up256((size_t)pl.Qpad * 4);
    pl.off_lost = off;   off += up256((size_t)pl.Qpad * 4);   // directly behind cnt: cleared together
    pl.off_fb = off;     off += up256((size_t)pl.Qpad * 4);
    pl.off_cand = off;   off += up256((size_t)Q * pl.cap * 8);
    pl.off_sel = off;    off += up256((size_t)Q * k_prime * 8);   // scratch of the select kernel
    pl.total = off;
    return RALM_OK;
}

ralm_status check_datastore(const ralm_datastore_t *ds, bool need_scan)
{
    if (!ds) return fail(RALM_ERR_NULL, "datastore descriptor is NULL");
    if (!ds->exact) return fail(RALM_ERR_NULL, "datastore.exact is NULL");
    // row numbers of a padded last tile must still fit int32
    if (ds->N < 1 || ds->N > 0x7fffffffLL - 512) return fail(RALM_ERR_SHAPE, "N=%lld out of [1, 2^31 - 512]", (long long)ds->N);
    if (ds->d < 8 || ds->d % 8 != 0 || ds->d > 16384)
        return fail(RALM_ERR_SHAPE, "d=%d must be a multiple of 8 in [8, 16384]", ds->d);
    if (ds->exact_dtype != RALM_F32 && ds->exact_dtype != RALM_F16)
        return fail(RALM_ERR_DTYPE, "exact_dtype must be RALM_F32 or RALM_F16");
    const int64_t es = ds->exact_stride ? ds->exact_stride : ds->d;
    if (es < ds->d) return fail(RALM_ERR_SHAPE, "exact_stride < d");
    if (!aligned16(ds->exact) || (es * elem_bytes(ds->exact_dtype)) % 16)
        return fail(RALM_ERR_ALIGN, "exact copy: base and row pitch must be multiples of 16 bytes");
    // without a scan copy the exact copy is scanned, and the scan's 24-bit offset arithmetic applies to it
    if (need_scan && !ds->scan && es * elem_bytes(ds->exact_dtype) >= (1 << 24))
        return fail(RALM_ERR_SHAPE, "exact_stride: row pitch of a scanned copy must be below 16 MiB");
    if (ds->metric != RALM_METRIC_IP && ds->metric != RALM_METRIC_L2) return fail(RALM_ERR_DTYPE, "metric unknown");
    if (need_scan && ds->metric == RALM_METRIC_L2) {
        if (!ds->scan) return fail(RALM_ERR_NULL, "the squared-distance metric needs a scan copy built by ralm_build_scan_copy_l2");
        if (ds->scan_dtype != RALM_BF16 && ds->scan_dtype != RALM_F16)
            return fail(RALM_ERR_DTYPE, "the squared-distance metric needs a bf16 or fp16 scan copy");
    }
    if (need_scan && ds->scan) {
        if (ds->scan_dtype != RALM_BF16 && ds->scan_dtype != RALM_F16 && ds->scan_dtype != RALM_F32)
            return fail(RALM_ERR_DTYPE, "scan_dtype unknown");
        const int64_t sd = scan_cols(ds);
        const int64_t ss = ds->scan_stride ? ds->scan_stride : sd;
        if (ss < sd) return fail(RALM_ERR_SHAPE, "scan_stride < d (+ 8 norm columns for the squared-distance metric)");
        if (!aligned16(ds->scan) || (ss * elem_bytes(ds->scan_dtype)) % 16)
            return fail(RALM_ERR_ALIGN, "scan copy: base and row pitch must be multiples of 16 bytes");
        // the pipelined scan forms per-lane byte offsets (row in tile) * pitch with a 24-bit multiply
        if (ss * elem_bytes(ds->scan_dtype) >= (1 << 24))
            return fail(RALM_ERR_SHAPE, "scan_stride: row pitch of the scan copy must be below 16 MiB");
    }
    return RALM_OK;
}

int device_cus()
{
    static int cus = 0;
    if (cus == 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
            cus = n;
        else
            cus = 256;
    }
    return cus;
}

// compute units that the scan's persistent grids leave free (ralm_scan_reserve_cus)
std::atomic<int> g_scan_reserve{0};

// ---- scan timing aid ------------------------------------------------------------------------
constexpr int MAX_PROF = 2048;
bool g_prof_on = false;
int g_prof_n = 0;
hipEvent_t g_prof_ev[MAX_PROF][2];
int g_prof_made = 0;

}  // namespace

extern "C" {

const char *ralm_last_error(void) { return g_err; }

size_t ralm_workspace_bytes(int64_t Q, const ralm_datastore_t *ds, int32_t k, int32_t k_prime)
{
    if (Q < 1 || check_datastore(ds, true) != RALM_OK) return 0;
    Plan pl;
    if (make_plan(Q, ds, k, k_prime, pl) != RALM_OK) return 0;
    return pl.total;
}

}  // extern "C"

namespace {

// sequential == false: the strided ladder described at the top of this file.
// sequential == true: consecutive blocks of tiles, each small enough that a list holds its k'
// best so far plus every row of the block, so that no list can overflow whatever the order of
// the rows; about N / cap launches.
ralm_status retrieve_impl(const float *queries, int64_t Q, const ralm_datastore_t *ds, int32_t k, int32_t k_prime,
                          int32_t *out_ids, float *out_scores, float *out_margin, void *workspace,
                          size_t workspace_bytes, void *stream_, bool sequential)
{
    if (!queries || !out_ids || !out_scores) return fail(RALM_ERR_NULL, "queries/out_ids/out_scores is NULL");
    if (Q < 1 || Q > (1 << 20)) return fail(RALM_ERR_SHAPE, "Q=%lld out of [1, 2^20]", (long long)Q);
    ralm_status st = check_datastore(ds, true);
    if (st != RALM_OK) return st;
    if (!aligned16(queries)) return fail(RALM_ERR_ALIGN, "queries must be 16-byte aligned");
    Plan pl;
    st = make_plan(Q, ds, k, k_prime, pl);
    if (st != RALM_OK) return st;
    // the scan kernels count (row tile, query tile) work items in 32 bits
    if (((ds->N + SCAN_BM - 1) / SCAN_BM) * 2 * ((Q + 31) / 32) > 0x7fffffffLL)
        return fail(RALM_ERR_SHAPE, "Q=%lld x N=%lld: more than 2^31 tile pairs in one call; split the batch",
                    (long long)Q, (long long)ds->N);
    if (!workspace) return fail(RALM_ERR_WORKSPACE, "workspace is NULL");
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return fail(RALM_ERR_WORKSPACE, "workspace must be 256-byte aligned");
    if (workspace_bytes < pl.total)
        return fail(RALM_ERR_WORKSPACE, "workspace too small: %zu < %zu bytes", workspace_bytes, pl.total);

    hipStream_t stream = static_cast<hipStream_t>(stream_);
    unsigned char *ws = static_cast<unsigned char *>(workspace);
    uint16_t *qs = reinterpret_cast<uint16_t *>(ws + pl.off_q);
    u64 *tau = reinterpret_cast<u64 *>(ws + pl.off_tau);
    uint32_t *cnt = reinterpret_cast<uint32_t *>(ws + pl.off_cnt);
    uint32_t *lost = reinterpret_cast<uint32_t *>(ws + pl.off_lost);
    int32_t *fb_list = reinterpret_cast<int32_t *>(ws + pl.off_fb);
    int32_t *flags = reinterpret_cast<int32_t *>(ws + pl.off_flags);
    u64 *cand = reinterpret_cast<u64 *>(ws + pl.off_cand);
    u64 *sel = reinterpret_cast<u64 *>(ws + pl.off_sel);

    const void *scan = ds->scan ? ds->scan : ds->exact;
    const int scan_dt = ds->scan ? ds->scan_dtype : ds->exact_dtype;
    const int64_t scan_ld = ds->scan ? (ds->scan_stride ? ds->scan_stride : scan_cols(ds))
                                     : (ds->exact_stride ? ds->exact_stride : ds->d);
    const int mma_dt = scan_dt == RALM_F16 ? RALM_F16 : RALM_BF16;   // fp32 rows are rounded to bf16
    // the scan's grids are persistent: one workgroup per CU (two for the small tiles), minus the reserve
    int n_cu = device_cus() - g_scan_reserve.load(std::memory_order_relaxed);
    if (n_cu < 8) n_cu = 8;

    // the same launch clears the flag block and, behind the queries, the admission keys, the list
    // lengths and the lost marks (contiguous in the workspace)
    RALM_HIP(launch_query_prep(queries, Q, ds->d, qs, pl.Qpad, pl.dpad, mma_dt, ds->metric,
                               reinterpret_cast<uint32_t *>(flags), FLAG_BLOCK_BYTES / 4,
                               reinterpret_cast<uint32_t *>(tau), (int64_t)(pl.off_fb - pl.off_tau) / 4, stream));

    ScanParams sp;
    sp.X = scan; sp.ldx = scan_ld; sp.N = ds->N; sp.d = scan_cols(ds); sp.in_dtype = scan_dt;
    sp.Qs = qs; sp.dpad = pl.dpad; sp.Q = (int32_t)Q;
    sp.tau = tau; sp.cand = cand; sp.cnt = cnt; sp.cap = pl.cap;
    sp.lists_empty = 0;
    // one stage: scan the tiles sp describes, then cut every list down to its k' best
    int32_t stage_no = 0;
    auto run_stage = [&]() -> ralm_status {
        if (sp.n_row_tiles <= 0) return RALM_OK;
        const bool prof = g_prof_on && g_prof_n < MAX_PROF;
        if (prof) {
            while (g_prof_made <= g_prof_n) {
                RALM_HIP(hipEventCreate(&g_prof_ev[g_prof_made][0]));
                RALM_HIP(hipEventCreate(&g_prof_ev[g_prof_made][1]));
                ++g_prof_made;
            }
            RALM_HIP(hipEventRecord(g_prof_ev[g_prof_n][0], stream));
        }
        RALM_HIP(launch_scan(sp, n_cu, stream));
        if (prof) {
            RALM_HIP(hipEventRecord(g_prof_ev[g_prof_n][1], stream));
            ++g_prof_n;
        }
        RALM_HIP(launch_select(cand, cnt, pl.cap, pl.k_prime, Q, tau, sel, lost, flags, stage_no++, stream));
        return RALM_OK;
    };

    const int64_t tiles = (ds->N + SCAN_BM - 1) / SCAN_BM;
    if (sequential) {
        const int64_t block = ((int64_t)pl.cap - pl.k_prime) / SCAN_BM;   // >= 1: cap >= 16384, k' <= 4096
        sp.tile_stride = 1;
        sp.tile_skip = 0;
        sp.park_pushes = 0;
        for (int64_t t0 = 0; t0 < tiles; t0 += block) {
            sp.tile_begin = t0;
            sp.n_row_tiles = tiles - t0 < block ? tiles - t0 : block;
            st = run_stage();
            if (st != RALM_OK) return st;
        }
    } else {
        sp.tile_begin = 0;
        for (int s = 0; s < pl.n_stages; ++s) {
            const int64_t stride = pl.stride[s];
            sp.tile_stride = stride;
            if (s == 0) {
                sp.tile_skip = 0;                                   // every multiple of the stride
                sp.n_row_tiles = (tiles + stride - 1) / stride;
                sp.park_pushes = 0;                                 // admits everything
                sp.lists_empty = 1;
            } else {
                const int64_t m_max = (tiles + stride - 1) / stride - 1;   // multiples m >= 1 with m*stride < tiles
                const int64_t g = pl.stride[s - 1] / stride;        // ... that no earlier stage visited
                sp.tile_skip = (int32_t)g;
                sp.n_row_tiles = m_max - m_max / g;
                sp.park_pushes = 1;
                sp.lists_empty = 0;
            }
            st = run_stage();
            if (st != RALM_OK) return st;
        }
    }
    const int64_t exact_ld = ds->exact_stride ? ds->exact_stride : ds->d;
    // The re-score checks each query's result against the scan's rounding; the queries that fail
    // (and those whose list lost entries) are answered again by an exact pass over the exact copy.
    // tau is free by now and takes the exact rank-k keys.
    CertifyParams cert;
    cert.flags = flags;
    cert.lost = lost;
    cert.cnt_rw = cnt;
    cert.tau_exact = tau;
    cert.fb_list = fb_list;
    const float u = mma_dt == RALM_F16 ? 1.f / 2048.f : 1.f / 256.f;   // 11 / 8 significant bits
    cert.u_query = u;
    cert.u_rows = (scan == ds->exact && scan_dt == ds->exact_dtype && scan_dt != RALM_F32) ? 0.f : u;
    RALM_HIP(launch_rescore(cand, cnt, pl.cap, pl.k_prime, queries, Q, ds->exact, ds->exact_dtype, exact_ld, ds->d,
                            ds->metric, k, out_ids, out_scores, out_margin, cert, stream));
    RALM_HIP(launch_exact_pass(queries, Q, ds->exact, ds->exact_dtype, exact_ld, ds->N, ds->d, ds->metric, k, fb_list,
                               flags, tau, cand, cnt, pl.cap, out_ids, out_scores, n_cu, stream));
    return RALM_OK;
}

}  // namespace

extern "C" {

ralm_status ralm_retrieve_topk_ex(const float *queries, int64_t Q, const ralm_datastore_t *ds, int32_t k,
                                  int32_t k_prime, int32_t *out_ids, float *out_scores, float *out_margin,
                                  void *workspace, size_t workspace_bytes, void *stream)
{
    return retrieve_impl(queries, Q, ds, k, k_prime, out_ids, out_scores, out_margin, workspace, workspace_bytes,
                         stream, false);
}

ralm_status ralm_retrieve_topk_seq(const float *queries, int64_t Q, const ralm_datastore_t *ds, int32_t k,
                                   int32_t k_prime, int32_t *out_ids, float *out_scores, float *out_margin,
                                   void *workspace, size_t workspace_bytes, void *stream)
{
    return retrieve_impl(queries, Q, ds, k, k_prime, out_ids, out_scores, out_margin, workspace, workspace_bytes,
                         stream, true);
}

ralm_status ralm_workspace_overflows(const void *workspace, void *stream_, int32_t *count)
{
    if (!workspace || !count) return fail(RALM_ERR_NULL, "workspace/count is NULL");
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    RALM_HIP(hipStreamSynchronize(stream));
    RALM_HIP(hipMemcpy(count, static_cast<const int32_t *>(workspace) + FLAG_UNANSWERED, sizeof(int32_t),
                       hipMemcpyDeviceToHost));
    return RALM_OK;
}

static_assert(MAX_STAGE_SUMS == RALM_MAX_LADDER_STAGES, "the flag block holds one sum per reported stage");

ralm_status ralm_workspace_stage_entries(const void *workspace, void *stream_, int32_t *n_stages, int64_t *entries)
{
    if (!workspace || !n_stages || !entries) return fail(RALM_ERR_NULL, "workspace/n_stages/entries is NULL");
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    unsigned char block[FLAG_BLOCK_BYTES];
    RALM_HIP(hipStreamSynchronize(stream));
    RALM_HIP(hipMemcpy(block, workspace, sizeof(block), hipMemcpyDeviceToHost));
    int32_t n = reinterpret_cast<const int32_t *>(block)[FLAG_STAGES];
    n = n < 0 ? 0 : (n > MAX_STAGE_SUMS ? MAX_STAGE_SUMS : n);
    *n_stages = n;
    const unsigned long long *sums = reinterpret_cast<const unsigned long long *>(block + STAGE_SUMS_BYTE);
    for (int i = 0; i < RALM_MAX_LADDER_STAGES; ++i) entries[i] = i < n ? (int64_t)sums[i] : 0;
    return RALM_OK;
}

ralm_status ralm_workspace_counters(const void *workspace, void *stream_, ralm_counters_t *out)
{
    if (!workspace || !out) return fail(RALM_ERR_NULL, "workspace/out is NULL");
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    int32_t words[8];
    RALM_HIP(hipStreamSynchronize(stream));
    RALM_HIP(hipMemcpy(words, workspace, sizeof(words), hipMemcpyDeviceToHost));
    out->unanswered = words[FLAG_UNANSWERED];
    out->ladder_overflows = words[FLAG_LADDER_OVERFLOWS];
    out->hard_certified = words[FLAG_HARD_CERTIFIED];
    out->soft_certified = words[FLAG_SOFT_CERTIFIED];
    out->exact_pass = words[FLAG_FALLBACKS];
    return RALM_OK;
}

}  // extern "C"

namespace {

// Buffers of the simple entry point, kept between calls and grown on demand: allocating and
// freeing tens of gigabytes on every call is slow (and gets slower with repetition).
std::mutex g_simple_mutex;
void *g_simple_ws = nullptr, *g_simple_scan = nullptr;
size_t g_simple_ws_bytes = 0, g_simple_scan_bytes = 0;

// true if *buf holds at least `bytes` afterwards; on failure *buf is NULL
bool simple_reserve(void **buf, size_t *have, size_t bytes)
{
    if (*buf && *have >= bytes) return true;
    if (*buf) (void)hipFree(*buf);
    *buf = nullptr;
    *have = 0;
    if (hipMalloc(buf, bytes) != hipSuccess) {
        (void)hipGetLastError();
        *buf = nullptr;
        return false;
    }
    *have = bytes;
    return true;
}

}  // namespace

extern "C" {

void ralm_release_buffers(void)
{
    std::lock_guard<std::mutex> lock(g_simple_mutex);
    if (g_simple_ws) (void)hipFree(g_simple_ws);
    if (g_simple_scan) (void)hipFree(g_simple_scan);
    g_simple_ws = g_simple_scan = nullptr;
    g_simple_ws_bytes = g_simple_scan_bytes = 0;
}

ralm_status ralm_retrieve_topk(const float *queries, int64_t Q, const float *datastore, int64_t N, int32_t d,
                               int32_t k, int32_t *out_ids, float *out_scores)
{
    if (!queries || !datastore || !out_ids || !out_scores) return fail(RALM_ERR_NULL, "a pointer is NULL");
    ralm_datastore_t ds;
    memset(&ds, 0, sizeof(ds));
    ds.exact = datastore;
    ds.exact_dtype = RALM_F32;
    ds.scan = nullptr;
    ds.N = N;
    ds.d = d;
    if (Q < 1 || Q > (1 << 20)) return fail(RALM_ERR_SHAPE, "Q=%lld out of [1, 2^20]", (long long)Q);
    ralm_status st = check_datastore(&ds, true);
    if (st != RALM_OK) return st;
    Plan pl;
    st = make_plan(Q, &ds, k, 0, pl);
    if (st != RALM_OK) return st;
    std::lock_guard<std::mutex> lock(g_simple_mutex);
    if (!simple_reserve(&g_simple_ws, &g_simple_ws_bytes, pl.total))
        return fail(RALM_ERR_DEVICE, "no device memory for %zu bytes of workspace", pl.total);
    // Batches of up to 768 queries (three query tiles) scan the fp32 rows as they are: one pass over
    // 4 bytes per element, 9 to 14 ms per query tile at 21M x 768, beats a conversion pass (19.5 ms)
    // plus a scan of the copy (6.5 ms per tile), and no copy is held.  Larger batches are limited
    // by the matrix cores, which the
    // pipelined bf16 kernel feeds far better: they get a bf16 copy (one read, one write, redone on
    // every call: the rows may have changed), kept between calls; if the device has no room for
    // it the rows are scanned as they are by the staged kernel.  Same result either way.
    if (Q > 768 && simple_reserve(&g_simple_scan, &g_simple_scan_bytes, (size_t)N * d * 2) &&
        launch_convert_rows(datastore, d, g_simple_scan, RALM_BF16, d, N, d, nullptr) == hipSuccess) {
        ds.scan = g_simple_scan;
        ds.scan_dtype = RALM_BF16;
    }
    void *ws = g_simple_ws;
    st = ralm_retrieve_topk_ex(queries, Q, &ds, k, 0, out_ids, out_scores, nullptr, ws, pl.total, nullptr);
    int32_t overflows = 0;
    if (st == RALM_OK) st = ralm_workspace_overflows(ws, nullptr, &overflows);
    if (st == RALM_OK && overflows > 0) {
        // rows in an order that defeats the strided samples: redo the call block by block
        st = ralm_retrieve_topk_seq(queries, Q, &ds, k, 0, out_ids, out_scores, nullptr, ws, pl.total, nullptr);
        if (st == RALM_OK) st = ralm_workspace_overflows(ws, nullptr, &overflows);
    }
    if (st == RALM_OK && overflows > 0)
        return fail(RALM_ERR_OVERFLOW, "%d queries overflowed their candidate buffers", overflows);
    return st;
}

ralm_status ralm_build_scan_copy(const float *src, int64_t src_stride, void *dst, int32_t dst_dtype,
                                 int64_t dst_stride, int64_t N, int32_t d, void *stream)
{
    if (!src || !dst) return fail(RALM_ERR_NULL, "src/dst is NULL");
    if (N < 1 || d < 8 || d % 8) return fail(RALM_ERR_SHAPE, "N >= 1 and d a multiple of 8 required");
    if (dst_dtype != RALM_BF16 && dst_dtype != RALM_F16) return fail(RALM_ERR_DTYPE, "dst_dtype must be RALM_BF16 or RALM_F16");
    if (src_stride == 0) src_stride = d;
    if (dst_stride == 0) dst_stride = d;
    if (src_stride < d || dst_stride < d) return fail(RALM_ERR_SHAPE, "stride < d");
    if (!aligned16(src) || !aligned16(dst) || (src_stride * 4) % 16 || (dst_stride * 2) % 16)
        return fail(RALM_ERR_ALIGN, "bases and row pitches must be multiples of 16 bytes");
    RALM_HIP(launch_convert_rows(src, src_stride, dst, dst_dtype, dst_stride, N, d, static_cast<hipStream_t>(stream)));
    return RALM_OK;
}

ralm_status ralm_build_scan_copy_l2(const void *src, int32_t src_dtype, int64_t src_stride, void *dst,
                                    int32_t dst_dtype, int64_t dst_stride, int64_t N, int32_t d, void *stream)
{
    if (!src || !dst) return fail(RALM_ERR_NULL, "src/dst is NULL");
    if (N < 1 || d < 8 || d % 8) return fail(RALM_ERR_SHAPE, "N >= 1 and d a multiple of 8 required");
    if (src_dtype != RALM_F32 && src_dtype != RALM_F16) return fail(RALM_ERR_DTYPE, "src_dtype must be RALM_F32 or RALM_F16");
    if (dst_dtype != RALM_BF16 && dst_dtype != RALM_F16) return fail(RALM_ERR_DTYPE, "dst_dtype must be RALM_BF16 or RALM_F16");
    if (src_stride == 0) src_stride = d;
    if (dst_stride == 0) dst_stride = d + L2_EXTRA_COLS;
    if (src_stride < d || dst_stride < d + L2_EXTRA_COLS) return fail(RALM_ERR_SHAPE, "src_stride < d or dst_stride < d + 8");
    if (src == dst && (src_dtype != dst_dtype || src_stride != dst_stride))
        return fail(RALM_ERR_SHAPE, "in place (src == dst) needs equal dtypes and strides");
    if (!aligned16(src) || !aligned16(dst) || (src_stride * elem_bytes(src_dtype)) % 16 || (dst_stride * 2) % 16)
        return fail(RALM_ERR_ALIGN, "bases and row pitches must be multiples of 16 bytes");
    RALM_HIP(launch_l2_scan_copy(src, src_dtype, src_stride, dst, dst_dtype, dst_stride, N, d,
                                 static_cast<hipStream_t>(stream)));
    return RALM_OK;
}

}  // extern "C"

namespace {

// argument checks shared by the two forms of the cache lookup (host only)
ralm_status check_cache_lookup(const int32_t *cache_ids, const int32_t *cache_len, int32_t C, int64_t R,
                               const float *queries, int64_t Qt, const int64_t *q_offsets,
                               const ralm_datastore_t *ds, const int32_t *spec_ids, const float *spec_scores)
{
    if (!cache_ids || !cache_len || !queries || !q_offsets || !spec_ids || !spec_scores)
        return fail(RALM_ERR_NULL, "a pointer is NULL");
    if (R < 0 || R > MAX_REQUESTS || C < 1) return fail(RALM_ERR_SHAPE, "R=%lld, C=%d out of range", (long long)R, C);
    if (Qt < 0) return fail(RALM_ERR_RANGE, "Qt=%lld is negative", (long long)Qt);
    ralm_status st = check_datastore(ds, false);
    if (st != RALM_OK) return st;
    if (ds->d > 2048) return fail(RALM_ERR_SHAPE, "cache lookup supports d <= 2048");
    if (!aligned16(queries)) return fail(RALM_ERR_ALIGN, "queries must be 16-byte aligned");
    return RALM_OK;
}

}  // namespace

extern "C" {

size_t ralm_cache_lookup_workspace_bytes(int64_t Qt) { return Qt < 0 ? 0 : up256((size_t)(Qt > 0 ? Qt : 1) * 8); }

ralm_status ralm_cache_lookup(const int32_t *cache_ids, const int32_t *cache_len, int32_t C, int64_t R,
                              const float *queries, int64_t Qt, const int64_t *q_offsets,
                              const ralm_datastore_t *ds, int32_t *spec_ids, float *spec_scores, void *workspace,
                              size_t workspace_bytes, void *stream)
{
    ralm_status st = check_cache_lookup(cache_ids, cache_len, C, R, queries, Qt, q_offsets, ds, spec_ids, spec_scores);
    if (st != RALM_OK) return st;
    if (workspace && ((reinterpret_cast<uintptr_t>(workspace) & 7u) || workspace_bytes < (size_t)Qt * 8))
        return fail(RALM_ERR_WORKSPACE, "workspace must be 8-byte aligned and hold 8 bytes per query");
    const int64_t ld = ds->exact_stride ? ds->exact_stride : ds->d;
    RALM_HIP(launch_cache_lookup(cache_ids, cache_len, C, R, queries, Qt, q_offsets, ds->exact, ds->exact_dtype, ld,
                                 ds->N, ds->d, ds->metric, spec_ids, spec_scores, static_cast<u64 *>(workspace),
                                 static_cast<hipStream_t>(stream)));
    return RALM_OK;
}

}  // extern "C"

// Scratch of ralm_cache_lookup_static: one merge slot (8 bytes) per query, held by every GPU the
// library runs on until the process ends.  In host code the array's name is only a stand-in for
// the symbol; the device address is looked up once per device and used from then on.
constexpr int64_t STATIC_LOOKUP_MAX_QT = 65536;
static __device__ __align__(256) unsigned long long scratch[STATIC_LOOKUP_MAX_QT];

namespace {

constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[MAX_DEVICES] = {};

// device address of `scratch` on the current device (looked up on the first call per device)
ralm_status static_scratch(void **out)
{
    int dev = -1;
    RALM_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES) return fail(RALM_ERR_DEVICE, "device ordinal %d out of range", dev);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        RALM_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return fail(RALM_ERR_DEVICE, "hipGetSymbolAddress returned a null address");
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return RALM_OK;
}

}  // namespace

extern "C" {

ralm_status ralm_cache_lookup_static(const int32_t *cache_ids, const int32_t *cache_len, int32_t C, int64_t R,
                                     const float *queries, int64_t Qt, const int64_t *q_offsets,
                                     const ralm_datastore_t *ds, int32_t *spec_ids, float *spec_scores,
                                     void *stream)
{
    // every argument error is reported before the device is touched
    ralm_status st = check_cache_lookup(cache_ids, cache_len, C, R, queries, Qt, q_offsets, ds, spec_ids, spec_scores);
    if (st != RALM_OK) return st;
    if (Qt > STATIC_LOOKUP_MAX_QT)
        return fail(RALM_ERR_RANGE, "Qt=%lld exceeds the %lld queries the built-in scratch holds; use "
                    "ralm_cache_lookup with a workspace", (long long)Qt, (long long)STATIC_LOOKUP_MAX_QT);
    void *ptr = nullptr;
    st = static_scratch(&ptr);
    if (st != RALM_OK) return st;
    return ralm_cache_lookup(cache_ids, cache_len, C, R, queries, Qt, q_offsets, ds, spec_ids, spec_scores, ptr,
                             (size_t)STATIC_LOOKUP_MAX_QT * 8, stream);
}

ralm_status ralm_cache_insert(int32_t *cache_ids, int32_t *cache_len, int32_t *cache_head, int32_t C, int64_t R,
                              const int32_t *true_ids, int64_t true_stride, int64_t Qt, const int64_t *q_offsets,
                              const int32_t *first_mismatch, int32_t p, int32_t n_next, int64_t N, void *stream)
{
    if (!cache_ids || !cache_len || !cache_head || !true_ids || !q_offsets)
        return fail(RALM_ERR_NULL, "a pointer is NULL");
    if (R < 0 || R > MAX_REQUESTS || C < 1 || C > CACHE_INSERT_MAX_C)
        return fail(RALM_ERR_SHAPE, "R=%lld, C=%d out of range (C <= %d)", (long long)R, C, CACHE_INSERT_MAX_C);
    if (N < 1 || N > 0x7fffffffLL) return fail(RALM_ERR_SHAPE, "N=%lld out of [1, 2^31)", (long long)N);
    if (Qt < 0 || true_stride < 1) return fail(RALM_ERR_RANGE, "Qt >= 0 and true_stride >= 1 required");
    if (p < 1 || (int64_t)p > true_stride) return fail(RALM_ERR_K, "p=%d must be in [1, true_stride]", p);
    if (n_next < 0 || n_next > 65536) return fail(RALM_ERR_RANGE, "n_next=%d out of [0, 65536]", n_next);
    RALM_HIP(launch_cache_insert(cache_ids, cache_len, cache_head, C, R, true_ids, true_stride, Qt, q_offsets,
                                 first_mismatch, p, n_next, N, static_cast<hipStream_t>(stream)));
    return RALM_OK;
}

ralm_status ralm_knnlm_probs(const int32_t *ids, const float *scores, int64_t Q, int32_t k, const int32_t *values,
                             int64_t N, float temperature, int32_t *out_tokens, float *out_weights,
                             int32_t *out_top_token, float *out_top_prob, void *stream)
{
    if (!ids || !scores || !values || !out_tokens || !out_weights) return fail(RALM_ERR_NULL, "a pointer is NULL");
    if (Q < 0 || Q > (1 << 20)) return fail(RALM_ERR_SHAPE, "Q=%lld out of [0, 2^20]", (long long)Q);
    if (N < 1 || N > 0x7fffffffLL) return fail(RALM_ERR_SHAPE, "N=%lld out of [1, 2^31)", (long long)N);
    if (k < 1 || k > RALM_MAX_K) return fail(RALM_ERR_K, "k=%d must be in [1, %d]", k, RALM_MAX_K);
    if (!(temperature > 0.f) || !(temperature < __builtin_inff()))
        return fail(RALM_ERR_RANGE, "temperature must be positive and finite");
    RALM_HIP(launch_knnlm_probs(ids, scores, Q, k, values, N, (double)temperature, out_tokens, out_weights,
                                out_top_token, out_top_prob, static_cast<hipStream_t>(stream)));
    return RALM_OK;
}

size_t ralm_cache_lookup_topk_workspace_bytes(int64_t Qt, int32_t C)
{
    if (Qt < 0 || C < 1) return 0;
    const size_t q = (size_t)(Qt > 0 ? Qt : 1);
    return up256(q * (size_t)C * 8) + up256(q * 4);
}

ralm_status ralm_cache_lookup_topk(const int32_t *cache_ids, const int32_t *cache_len, int32_t C, int64_t R,
                                   const float *queries, int64_t Qt, const int64_t *q_offsets,
                                   const ralm_datastore_t *ds, int32_t k, int32_t *out_ids, float *out_scores,
                                   void *workspace, size_t workspace_bytes, void *stream_)
{
    if (!cache_ids || !cache_len || !queries || !q_offsets || !out_ids || !out_scores)
        return fail(RALM_ERR_NULL, "a pointer is NULL");
    if (R < 0 || R > MAX_REQUESTS || C < 1 || C > RALM_MAX_K_PRIME)
        return fail(RALM_ERR_SHAPE, "R=%lld, C=%d out of range (C <= %d)", (long long)R, C, RALM_MAX_K_PRIME);
    if (Qt < 0 || Qt > (1 << 20)) return fail(RALM_ERR_RANGE, "Qt=%lld out of [0, 2^20]", (long long)Qt);
    if (k < 1 || k > RALM_MAX_K || k > C) return fail(RALM_ERR_K, "k=%d must be in [1, min(C, %d)]", k, RALM_MAX_K);
    ralm_status st = check_datastore(ds, false);
    if (st != RALM_OK) return st;
    if (!aligned16(queries)) return fail(RALM_ERR_ALIGN, "queries must be 16-byte aligned");
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) ||
        workspace_bytes < ralm_cache_lookup_topk_workspace_bytes(Qt, C))
        return fail(RALM_ERR_WORKSPACE, "workspace NULL, not 256-byte aligned or too small");
    if (Qt == 0) return RALM_OK;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    u64 *keys = static_cast<u64 *>(workspace);
    uint32_t *cnt = reinterpret_cast<uint32_t *>(static_cast<unsigned char *>(workspace) + up256((size_t)Qt * C * 8));
    RALM_HIP(launch_cache_keys(cache_ids, cache_len, C, R, Qt, q_offsets, ds->N, keys, cnt, stream));
    // the cached rows are the candidates: exact scores, ranking and the first k, as after a scan
    const int64_t ld = ds->exact_stride ? ds->exact_stride : ds->d;
    CertifyParams no_check;
    memset(&no_check, 0, sizeof(no_check));
    RALM_HIP(launch_rescore(keys, cnt, (uint32_t)C, C, queries, Qt, ds->exact, ds->exact_dtype, ld, ds->d, ds->metric,
                            k, out_ids, out_scores, nullptr, no_check, stream));
    return RALM_OK;
}

ralm_status ralm_verify(const int32_t *spec_ids, const int32_t *true_ids, int64_t true_stride, int64_t Qt,
                        const int64_t *q_offsets, int64_t R, int32_t *first_mismatch, void *stream)
{
    if (!spec_ids || !true_ids || !q_offsets || !first_mismatch) return fail(RALM_ERR_NULL, "a pointer is NULL");
    if (R < 0 || R > MAX_REQUESTS) return fail(RALM_ERR_SHAPE, "R=%lld out of range", (long long)R);
    if (Qt < 0 || true_stride < 1) return fail(RALM_ERR_RANGE, "Qt >= 0 and true_stride >= 1 required");
    RALM_HIP(launch_verify(spec_ids, true_ids, true_stride, Qt, q_offsets, R, first_mismatch,
                           static_cast<hipStream_t>(stream)));
    return RALM_OK;
}

void ralm_scan_reserve_cus(int32_t n)
{
    g_scan_reserve.store(n < 0 ? 0 : n, std::memory_order_relaxed);
}

void ralm_profile_enable(int32_t on)
{
    g_prof_on = on != 0;
}

ralm_status ralm_profile_scan_ms(float *total_ms, int32_t *launches)
{
    if (!total_ms || !launches) return fail(RALM_ERR_NULL, "total_ms/launches is NULL");
    float total = 0.f;
    for (int i = 0; i < g_prof_n; ++i) {
        RALM_HIP(hipEventSynchronize(g_prof_ev[i][1]));
        float ms = 0.f;
        RALM_HIP(hipEventElapsedTime(&ms, g_prof_ev[i][0], g_prof_ev[i][1]));
        total += ms;
    }
    *total_ms = total;
    *launches = g_prof_n;
    g_prof_n = 0;
    return RALM_OK;
}

}  // extern "C"
