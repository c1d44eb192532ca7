// Per-query selection and exact re-scoring (gfx950).
//
//  select_kernel   exact k'-th best of a query's candidate keys by an 8-bit radix descent
//                  over the 64-bit ranking key; writes it as the admission key for the next
//                  scan stage and cuts the list down to its k' best keys in place.
//  rescore_kernel  for the k' rows kept by the scan: inner product with the fp32 query from
//                  the EXACT datastore copy, products and sum in double, one rounding to
//                  fp32; final ranking (score descending, id ascending); first k written.
//                  This is what makes the result that of the paper's exact dense retriever
//                  (Section 5.1) although the scan ran in bf16/fp16.  It also checks that
//                  result: the gap between the exact rank-k score and the scan's score of the
//                  worst kept candidate must exceed what the scan's rounding can do to a
//                  score (judged from the rounding errors seen on the candidates themselves);
//                  a query that fails the check, or whose list lost entries, is queued for
//  exact_scan_kernel / exact_finish_kernel: every row of the exact copy is scored exactly
//                  against the queued queries, the rows that reach the query's exact rank-k
//                  key are collected, and the best k of them are the answer.  Both kernels
//                  are always launched and return at once when nothing is queued.
#include <atomic>

#include "ralm_common.h"
#include "ralm_kernels.h"

namespace ralm {

namespace {

constexpr int SEL_THREADS = 1024;

// Exact rank-th best (1-based) key of c[0, n), n >= rank >= 1, by a radix descent over the 64-bit
// ranking key, 8 bits per pass from the top.  A pass histograms the digit of the keys that match
// the prefix found so far; wave 0 walks the 256 bins from the best digit down to the one that
// holds the wanted key.  As soon as that bin holds a single key the descent stops and one more
// pass over the list fetches that key (scores are mostly distinct, so this usually happens
// before the id bits are reached).  Called by all SEL_THREADS threads of a workgroup; keys must
// be distinct.
struct RadixShared {
    uint32_t hist[256];
    uint32_t digit, remaining, bin;
    u64 kth;
};

__device__ u64 radix_kth(const u64 *__restrict__ c, uint32_t n, uint32_t rank, RadixShared &sh)
{
    const int tid = threadIdx.x, lane = tid & 63;
    u64 prefix = 0, mask = 0;
    uint32_t remaining = rank;
    bool single = false;
    for (int shift = 56; shift >= 0; shift -= 8) {
        if (tid < 256) sh.hist[tid] = 0;
        __syncthreads();
        for (uint32_t i = tid; i < n; i += SEL_THREADS) {
            const u64 key = c[i];
            if ((key & mask) == prefix) atomicAdd(&sh.hist[(uint32_t)(key >> shift) & 255u], 1u);
        }
        __syncthreads();
        if (tid < 64) {
            // lane l owns digits 255-4l .. 252-4l, best first
            uint32_t h[4], tot = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                h[j] = sh.hist[255 - 4 * lane - j];
                tot += h[j];
            }
            uint32_t incl = tot;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const uint32_t y = __shfl_up(incl, o, 64);
                if (lane >= o) incl += y;
            }
            uint32_t run = incl - tot;   // keys in better digits than this lane's
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (run < remaining && run + h[j] >= remaining) {
                    sh.digit = 255 - 4 * lane - j;
                    sh.remaining = remaining - run;
                    sh.bin = h[j];
                }
                run += h[j];
            }
        }
        __syncthreads();
        prefix |= (u64)sh.digit << shift;
        mask |= 0xffull << shift;
        remaining = sh.remaining;
        if (sh.bin == 1) {
            single = shift > 0;
            break;
        }
    }
    u64 kth = prefix;
    if (single) {   // the only key under the prefix is the wanted one
        for (uint32_t i = tid; i < n; i += SEL_THREADS) {
            const u64 key = c[i];
            if ((key & mask) == prefix) sh.kth = key;
        }
        __syncthreads();
        kth = sh.kth;
    }
    __syncthreads();   // sh may be reused by the caller's next call
    return kth;
}

// Per query: the k'-th best key of its list becomes the admission key of the next scan stage
// and the list is cut down to its k' best keys in place.  A list that was sent more keys than
// it has slots kept only the first `cap` of them: it is processed as it is (its k'-th best key
// is still a valid lower bound, the rows behind those keys were all scanned) and the query is
// marked in `lost`, so that it is answered by the exact pass at the end of the call.
__global__ __launch_bounds__(SEL_THREADS) void select_kernel(u64 *__restrict__ cand, uint32_t *__restrict__ cnt,
                                                             uint32_t cap, int k_prime, u64 *__restrict__ tau,
                                                             u64 *__restrict__ tmp, uint32_t *__restrict__ lost,
                                                             int32_t *__restrict__ flags, int stage)
{
    __shared__ RadixShared sh;
    __shared__ uint32_t s_out;

    const int64_t q = blockIdx.x;
    const int tid = threadIdx.x;
    uint32_t n = cnt[q];
    u64 *c = cand + q * (int64_t)cap;
    // entries the scan sent to this list in the stage that just ended, plus the (at most k') kept before
    if (tid == 0 && stage >= 0 && stage < MAX_STAGE_SUMS) {
        unsigned long long *sums = reinterpret_cast<unsigned long long *>(reinterpret_cast<unsigned char *>(flags) + STAGE_SUMS_BYTE);
        atomicAdd(sums + stage, (unsigned long long)n);
        if (q == 0) flags[FLAG_STAGES] = stage + 1;
    }

    if (n > cap) {
        n = cap;
        if (tid == 0) {
            if (lost[q] == 0) atomicAdd(flags + FLAG_LADDER_OVERFLOWS, 1);
            lost[q] = 1;
        }
    }
    if (n < (uint32_t)k_prime) {    // fewer than k' candidates exist so far: keep admitting everything
        if (tid == 0) {
            tau[q] = 0ull;
            cnt[q] = n;
        }
        return;
    }

    const u64 kth = radix_kth(c, n, (uint32_t)k_prime, sh);
    // keys are distinct: exactly k' of them are >= kth

    // cut the list down to those k' keys, in place (via tmp)
    if (tid == 0) s_out = 0;
    __syncthreads();
    u64 *t = tmp + q * (int64_t)k_prime;
    for (uint32_t i = tid; i < n; i += SEL_THREADS) {
        const u64 key = c[i];
        if (key >= kth) {
            const uint32_t at = atomicAdd(&s_out, 1u);
            if (at < (uint32_t)k_prime) t[at] = key;
        }
    }
    __syncthreads();
    for (int i = tid; i < k_prime; i += SEL_THREADS) c[i] = t[i];
    if (tid == 0) {
        tau[q] = kth;
        cnt[q] = (uint32_t)k_prime;
    }
}

// every exact score ends in this sum over the wave's 64 lane sums (fixed order: the re-score and
// the exact pass must give a row the same number)
__device__ __forceinline__ double wave_sum(double x) { return wave64_sum(x); }

// The exact score, as the re-score and the exact pass form it: lane l of a wave takes the
// elements 4l .. 4l+3, 256+4l .., adds their products (squared differences) to its sum in that
// order, and the 64 lane sums are added in a fixed order (wave_sum).  Products and sums in double;
// the caller rounds the total once to fp32.
template <bool L2>
__device__ __forceinline__ void exact_accum4(double &sum, const float4 &x, const float4 &y)
{
    if constexpr (L2) {
        const double d0 = (double)y.x - (double)x.x, d1 = (double)y.y - (double)x.y;
        const double d2 = (double)y.z - (double)x.z, d3 = (double)y.w - (double)x.w;
        sum += d0 * d0;
        sum += d1 * d1;
        sum += d2 * d2;
        sum += d3 * d3;
    } else {
        sum += (double)x.x * (double)y.x;
        sum += (double)x.y * (double)y.y;
        sum += (double)x.z * (double)y.z;
        sum += (double)x.w * (double)y.w;
    }
}

// elements j .. j+3 of a row of the exact copy, widened exactly to fp32
template <int EX>
__device__ __forceinline__ float4 exact_load4(const void *__restrict__ exact, int64_t row_off, int j)
{
    if constexpr (EX == DT_F32) {
        return *reinterpret_cast<const float4 *>(static_cast<const float *>(exact) + row_off + j);
    } else {
        const uint2 h = *reinterpret_cast<const uint2 *>(static_cast<const uint16_t *>(exact) + row_off + j);
        return make_float4(f16_bits_to_f32(h.x & 0xffffu), f16_bits_to_f32(h.x >> 16), f16_bits_to_f32(h.y & 0xffffu),
                           f16_bits_to_f32(h.y >> 16));
    }
}

constexpr int RS_THREADS = 1024, RS_WAVES = RS_THREADS / 64;

// Re-score of the candidates, final ranking, and the check of the result (see CertifyParams).
// EX: DT_F32 or DT_F16 exact rows.  L2: the score is minus the squared distance; the scan's
// score of a row is then 2<q, x> - |x|^2, so |q|^2 is subtracted from it wherever the two are
// compared.
template <int EX, bool L2>
__global__ __launch_bounds__(RS_THREADS) void rescore_kernel(const u64 *__restrict__ cand,
                                                      const uint32_t *__restrict__ cnt, uint32_t cap,
                                                      int k_prime, int kp2, const float *__restrict__ queries,
                                                      const void *__restrict__ exact, int64_t ld, int d,
                                                      int k, int32_t *__restrict__ out_ids,
                                                      float *__restrict__ out_scores,
                                                      float *__restrict__ out_margin, const CertifyParams cert)
{
    extern __shared__ __align__(16) unsigned char smem[];
    u64 *keys = reinterpret_cast<u64 *>(smem);   // [kp2]
    __shared__ u64 s_min_scan[RS_WAVES];
    __shared__ double s_e2[RS_WAVES], s_x2[RS_WAVES], s_q2[RS_WAVES];

    const int64_t q = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t n_raw = cnt[q];
    const int n = (int)(n_raw < (uint32_t)k_prime ? n_raw : (uint32_t)k_prime);
    const u64 *mine = cand + q * (int64_t)cap;
    const float *qv = queries + q * (int64_t)d;
    const bool stats = out_margin || cert.flags;   // wave-uniform

    // |q|^2: part of the scan's score under L2, and of the rounding bound
    double q2 = 0.0;
    if (stats) {
        for (int j = tid; j < d; j += RS_THREADS) q2 += (double)qv[j] * (double)qv[j];
        q2 = wave_sum(q2);
        if (lane == 0) s_q2[wave] = q2;
    }
    __syncthreads();
    if (stats) {
        q2 = 0.0;
        for (int w = 0; w < RS_WAVES; ++w) q2 += s_q2[w];
    }
    const float q_sq = L2 ? (float)q2 : 0.f;

    u64 min_scan = ~0ull;
    double e2 = 0.0, x2max = 0.0;   // sum of squared scan errors, largest squared row norm (lane 0)
    for (int c = wave; c < n; c += RS_WAVES) {
        const u64 skey = mine[c];
        min_scan = skey < min_scan ? skey : min_scan;
        const int32_t id = key_id(skey);
        const int64_t row_off = (int64_t)id * ld;
        double sum = 0.0, x2 = 0.0;
        for (int j = lane * 4; j < d; j += 256) {
            const float4 x = exact_load4<EX>(exact, row_off, j);
            const float4 y = *reinterpret_cast<const float4 *>(qv + j);
            exact_accum4<L2>(sum, x, y);
            if (stats)
                x2 += (double)x.x * (double)x.x + (double)x.y * (double)x.y + (double)x.z * (double)x.z +
                      (double)x.w * (double)x.w;
        }
        sum = wave_sum(sum);
        const float score = L2 ? (float)(-sum) : (float)sum;
        if (stats) {
            x2 = wave_sum(x2);
            const double e = (double)(key_score(skey) - q_sq) - (double)score;
            e2 += e * e;
            x2max = x2 > x2max ? x2 : x2max;
        }
        if (lane == 0) keys[c] = make_key(score, id);
    }
    for (int c = n + tid; c < kp2; c += RS_THREADS) keys[c] = 0ull;
    if (lane == 0) {
        s_min_scan[wave] = min_scan;
        s_e2[wave] = e2;
        s_x2[wave] = x2max;
    }
    __syncthreads();

    // bitonic sort, descending by key
    for (int size = 2; size <= kp2; size <<= 1) {
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            for (int t = tid; t < kp2 / 2; t += RS_THREADS) {
                const int lo = 2 * t - (t & (stride - 1));
                const int hi = lo + stride;
                const bool desc = (lo & size) == 0;
                const u64 a = keys[lo], b = keys[hi];
                if ((a < b) == desc) {
                    keys[lo] = b;
                    keys[hi] = a;
                }
            }
            __syncthreads();
        }
    }

    for (int r = tid; r < k; r += RS_THREADS) {
        const u64 key = keys[r];
        const bool have = r < n;
        out_ids[q * k + r] = have ? key_id(key) : -1;
        out_scores[q * k + r] = have ? key_score(key) : -__builtin_inff();
    }
    if (stats && tid == 0) {
        u64 ms = s_min_scan[0];
        double se2 = s_e2[0], x2m = s_x2[0];
        for (int w = 1; w < RS_WAVES; ++w) {
            ms = s_min_scan[w] < ms ? s_min_scan[w] : ms;
            se2 += s_e2[w];
            x2m = s_x2[w] > x2m ? s_x2[w] : x2m;
        }
        // margin: exact score at rank k minus the scan's score of the worst kept candidate.  A row
        // that was not kept has a scan score at most the latter, so it can belong in the top k only
        // if the scan mis-scored it by at least the margin.
        float margin;
        if (n < k)
            margin = __builtin_nanf("");
        else if (n < k_prime)
            margin = __builtin_inff();   // every row of the datastore was re-scored
        else
            margin = key_score(keys[k - 1]) - (key_score(ms) - q_sq);
        if (out_margin) out_margin[q] = margin;
        if (cert.flags) {
            // what the scan's rounding can do to a score: the deterministic bound (every rounding
            // error aligned; rows outside the candidates are taken to be no longer than the longest
            // candidate), and the spread actually seen on this query's candidates
            const double qn = sqrt(q2), xn = sqrt(x2m);
            const double uq = cert.u_query, ux = cert.u_rows;
            double hard = (uq + ux + uq * ux) * qn * xn + (double)d * 5.9604644775390625e-08 * qn * xn;
            if (L2) hard = 2.0 * hard + (ux * ux + (double)d * 5.9604644775390625e-08) * x2m;
            const double soft = n > 0 ? 8.0 * sqrt(se2 / (double)n) : 0.0;
            const bool truncated = cert.lost && cert.lost[q] != 0;
            const bool all_rows = n < k_prime && !truncated;
            const double m = (double)margin;
            const bool soft_ok = all_rows || (!truncated && n >= k && (m > soft || (soft == 0.0 && m >= 0.0)));
            if (soft_ok) {
                atomicAdd(cert.flags + FLAG_SOFT_CERTIFIED, 1);
                if (all_rows || m > hard) atomicAdd(cert.flags + FLAG_HARD_CERTIFIED, 1);
            } else if (n >= k) {
                // answered again by the exact pass: every row whose exact key reaches the exact
                // rank-k key found here (a lower bound of the true one) is collected in the list
                const int at = atomicAdd(cert.flags + FLAG_FALLBACKS, 1);
                cert.fb_list[at] = (int32_t)q;
                cert.tau_exact[q] = keys[k - 1];
                cert.cnt_rw[q] = 0u;
            }
        }
    }
}

// ---- exact pass for the queries whose scan result could not be trusted -------------------------
// All rows of the exact copy are scored exactly against up to QG of those queries at a time and
// every row whose exact key reaches the query's bound is appended to the query's list.  The
// arithmetic is that of the re-score (same order of the sums), so a row gets the same number.
constexpr int XS_THREADS = 256, XS_WAVES = XS_THREADS / 64, XS_QG = 8;

template <int EX, bool L2>
__global__ __launch_bounds__(XS_THREADS) void exact_scan_kernel(const float *__restrict__ queries,
                                                                const void *__restrict__ exact, int64_t ld,
                                                                int64_t N, int d, int qgroup,
                                                                const int32_t *__restrict__ fb_list,
                                                                const int32_t *__restrict__ flags,
                                                                const u64 *__restrict__ tau_exact,
                                                                u64 *__restrict__ cand, uint32_t *__restrict__ cnt,
                                                                uint32_t cap)
{
    extern __shared__ __align__(16) unsigned char smem[];
    float *qs = reinterpret_cast<float *>(smem);     // [qgroup][d]
    __shared__ u64 s_tau[XS_QG];
    __shared__ float s_tsc[XS_QG];                   // score part of the bound: a cheap first test
    __shared__ int32_t s_q[XS_QG];

    const int F = flags[FLAG_FALLBACKS];
    if (F <= 0) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t wave0 = (int64_t)blockIdx.x * XS_WAVES + wave, n_waves = (int64_t)gridDim.x * XS_WAVES;

    for (int g0 = 0; g0 < F; g0 += qgroup) {
        const int nq = F - g0 < qgroup ? F - g0 : qgroup;
        __syncthreads();
        if (tid < nq) {
            const int32_t q = fb_list[g0 + tid];
            s_q[tid] = q;
            s_tau[tid] = tau_exact[q];
            s_tsc[tid] = key_score(tau_exact[q]);
        }
        __syncthreads();
        for (int qi = 0; qi < nq; ++qi) {
            const float *src = queries + (int64_t)s_q[qi] * d;
            for (int j = tid * 4; j < d; j += XS_THREADS * 4)
                *reinterpret_cast<float4 *>(qs + (size_t)qi * d + j) = *reinterpret_cast<const float4 *>(src + j);
        }
        __syncthreads();

        for (int64_t row = wave0; row < N; row += n_waves) {
            const int64_t row_off = row * ld;
            double sum[XS_QG];
#pragma unroll
            for (int qi = 0; qi < XS_QG; ++qi) sum[qi] = 0.0;
            for (int j = lane * 4; j < d; j += 256) {
                const float4 x = exact_load4<EX>(exact, row_off, j);
#pragma unroll
                for (int qi = 0; qi < XS_QG; ++qi) {
                    if (qi < nq) {   // wave-uniform
                        const float4 y = *reinterpret_cast<const float4 *>(qs + (size_t)qi * d + j);
                        exact_accum4<L2>(sum[qi], x, y);
                    }
                }
            }
#pragma unroll
            for (int qi = 0; qi < XS_QG; ++qi) {
                if (qi < nq) {
                    const double t = wave_sum(sum[qi]);
                    const float sc = L2 ? (float)(-t) : (float)t;
                    if (lane == 0 && sc >= s_tsc[qi]) {   // a key that reaches the bound has a score that does
                        const u64 key = make_key(sc, (int32_t)row);
                        if (key >= s_tau[qi]) {
                            const int32_t q = s_q[qi];
                            const uint32_t at = atomicAdd(cnt + q, 1u);
                            if (at < cap) cand[(int64_t)q * cap + at] = key;
                        }
                    }
                }
            }
        }
    }
}

// The exact pass on the fp64 matrix cores (inner product, rows that are whole 256-byte steps).
// v_mfma_f64_16x16x4: operand A of lane l is element (i = l%16, k = l/16), operand B element
// (k = l/16, j = l%16), and the lane receives D(i = 4v + l/16, j = l%16) in its v-th result,
// v = 0..3.  i runs over 16 consecutive rows, j over up to 16 queued queries, so one pass over the
// exact copy serves 16 queries at the cost of one, with sums in double and no reduction across
// lanes.  A lane holds elements 4*CH*u + CH*(l/16) .. + CH-1 of its row (CH elements per 16-byte
// load); the queries sit in LDS as floats in the order the instructions consume them.  The sums
// are formed in another order than the re-score forms them, so a row's score may differ from the
// re-score's in the last place of the fp32 result (rarely: both are double sums rounded once);
// rows are therefore collected from one fp32 step BELOW the bound's score on, which keeps the k
// rows that defined the bound in the list whatever the order, and the final ranking uses this
// kernel's scores only.
constexpr int XM_NW = 8, XM_QG = 16;

template <int EX, int SEG>
__global__ __launch_bounds__(XM_NW * 64) void exact_scan_mfma_kernel(const float *__restrict__ queries,
                                                                      const void *__restrict__ exact, int64_t ld,
                                                                      int64_t N, int d,
                                                                      const int32_t *__restrict__ fb_list,
                                                                      const int32_t *__restrict__ flags,
                                                                      const u64 *__restrict__ tau_exact,
                                                                      u64 *__restrict__ cand, uint32_t *__restrict__ cnt,
                                                                      uint32_t cap)
{
    constexpr int CH = EX == DT_F32 ? 4 : 8;   // elements per 16-byte piece
    constexpr int ES = EX == DT_F32 ? 4 : 2;
    typedef double d4 __attribute__((ext_vector_type(4)));
    extern __shared__ __align__(16) unsigned char smem[];
    float *qf = reinterpret_cast<float *>(smem);   // [d / 4 instructions][4 k][16 j]
    __shared__ float s_tsc[XM_QG];
    __shared__ int32_t s_q[XM_QG];

    const int F = flags[FLAG_FALLBACKS];
    if (F <= 0) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r16 = lane & 15, kq = lane >> 4;
    const int NC = d / (4 * CH), nsegs = NC / SEG;
    const int64_t nblk = (N + 15) / 16;
    const int64_t blk0 = (int64_t)blockIdx.x * XM_NW + wave, blk_step = (int64_t)gridDim.x * XM_NW;
    const unsigned char *base = static_cast<const unsigned char *>(exact) + kq * 16;

    for (int g0 = 0; g0 < F; g0 += XM_QG) {
        const int nq = F - g0 < XM_QG ? F - g0 : XM_QG;
        __syncthreads();
        if (tid < XM_QG) {
            int32_t q = -1;
            float tsc = __builtin_inff();
            if (tid < nq) {
                q = fb_list[g0 + tid];
                const uint32_t b = (uint32_t)(tau_exact[q] >> 32);
                tsc = bits_score(b ? b - 1u : 0u);   // one fp32 step below the bound's score
            }
            s_q[tid] = q;
            s_tsc[tid] = tsc;
        }
        __syncthreads();
        for (int i = tid; i < XM_QG * d; i += XM_NW * 64) {
            const int qi = i / d, e = i - qi * d;
            const float v = qi < nq ? queries[(int64_t)s_q[qi] * d + e] : 0.f;
            const int t = CH * (e / (4 * CH)) + e % CH, k = (e / CH) & 3;
            qf[(size_t)t * 64 + k * 16 + qi] = v;
        }
        __syncthreads();
        const float my_tsc = s_tsc[r16];
        const int64_t my_q = s_q[r16];

        int64_t blk = blk0;
        if (blk >= nblk) continue;
        auto row_of = [&](int64_t b) {
            int64_t row = b * 16 + r16;
            row = row < N ? row : N - 1;   // rows past the end re-read the last one; their results are dropped
            return base + row * ld * ES;
        };
        const unsigned char *row = row_of(blk);
        int seg = 0;
        d4 acc = {0.0, 0.0, 0.0, 0.0};
        uint4 buf0[SEG], buf1[SEG];
        auto load = [&](uint4(&buf)[SEG], const unsigned char *rw, int sg) __attribute__((always_inline)) {
#pragma unroll
            for (int c = 0; c < SEG; ++c) buf[c] = *reinterpret_cast<const uint4 *>(rw + (size_t)(sg * SEG + c) * 64);
        };
        auto item = [&](uint4(&cur)[SEG], uint4(&nxt)[SEG]) __attribute__((always_inline)) -> bool {
            const bool last_seg = seg + 1 == nsegs;
            const int64_t blk_n = last_seg ? blk + blk_step : blk;
            const bool more = blk_n < nblk;
            const unsigned char *row_n = last_seg ? row_of(more ? blk_n : blk) : row;
            if (more) load(nxt, row_n, last_seg ? 0 : seg + 1);
            const float *ql = qf + (size_t)seg * (SEG * CH * 64) + lane;
#pragma unroll
            for (int c = 0; c < SEG; ++c) {
                double a[CH];
                if constexpr (EX == DT_F32) {
                    a[0] = (double)__uint_as_float(cur[c].x);
                    a[1] = (double)__uint_as_float(cur[c].y);
                    a[2] = (double)__uint_as_float(cur[c].z);
                    a[3] = (double)__uint_as_float(cur[c].w);
                } else {
                    a[0] = (double)f16_bits_to_f32(cur[c].x & 0xffffu);
                    a[1] = (double)f16_bits_to_f32(cur[c].x >> 16);
                    a[2] = (double)f16_bits_to_f32(cur[c].y & 0xffffu);
                    a[3] = (double)f16_bits_to_f32(cur[c].y >> 16);
                    a[4] = (double)f16_bits_to_f32(cur[c].z & 0xffffu);
                    a[5] = (double)f16_bits_to_f32(cur[c].z >> 16);
                    a[6] = (double)f16_bits_to_f32(cur[c].w & 0xffffu);
                    a[7] = (double)f16_bits_to_f32(cur[c].w >> 16);
                }
#pragma unroll
                for (int e = 0; e < CH; ++e)
                    acc = __builtin_amdgcn_mfma_f64_16x16x4f64(a[e], (double)ql[(size_t)(c * CH + e) * 64], acc, 0, 0, 0);
            }
            if (last_seg) {
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int64_t rw = blk * 16 + 4 * v + kq;
                    const float sc = (float)acc[v];
                    if (rw < N && sc >= my_tsc) {
                        const uint32_t at = atomicAdd(cnt + my_q, 1u);
                        if (at < cap) cand[my_q * cap + at] = make_key(sc, (int32_t)rw);
                    }
                }
                acc = d4{0.0, 0.0, 0.0, 0.0};
                blk = blk_n;
                seg = 0;
                row = row_n;
            } else {
                ++seg;
            }
            return !more;
        };
        load(buf0, row, 0);
        for (;;) {
            if (item(buf0, buf1)) break;
            if (item(buf1, buf0)) break;
        }
    }
}

// Final ranking of an exact-pass query: the k best keys of its list, sorted, written out.
__global__ __launch_bounds__(SEL_THREADS) void exact_finish_kernel(const u64 *__restrict__ cand,
                                                                   const uint32_t *__restrict__ cnt, uint32_t cap,
                                                                   int k, int kp2, const int32_t *__restrict__ fb_list,
                                                                   int32_t *__restrict__ flags,
                                                                   int32_t *__restrict__ out_ids,
                                                                   float *__restrict__ out_scores)
{
    extern __shared__ __align__(16) unsigned char smem[];
    u64 *keys = reinterpret_cast<u64 *>(smem);   // [kp2]
    __shared__ RadixShared sh;
    __shared__ uint32_t s_out;

    const int F = flags[FLAG_FALLBACKS];
    const int tid = threadIdx.x;
    for (int i = blockIdx.x; i < F; i += gridDim.x) {
        const int64_t q = fb_list[i];
        const uint32_t n = cnt[q];
        const u64 *c = cand + q * (int64_t)cap;
        __syncthreads();
        if (n > cap || n < (uint32_t)k) {
            // more rows reach the bound than a list holds (n < k cannot happen: the k rows that
            // defined the bound reach it): this query stays unanswered and is counted
            for (int r = tid; r < k; r += SEL_THREADS) {
                out_ids[q * k + r] = -1;
                out_scores[q * k + r] = __builtin_nanf("");
            }
            if (tid == 0) atomicAdd(flags + FLAG_UNANSWERED, 1);
            continue;
        }
        const u64 kth = radix_kth(c, n, (uint32_t)k, sh);
        if (tid == 0) s_out = 0;
        for (int r = tid; r < kp2; r += SEL_THREADS) keys[r] = 0ull;
        __syncthreads();
        for (uint32_t e = tid; e < n; e += SEL_THREADS) {
            const u64 key = c[e];
            if (key >= kth) {
                const uint32_t at = atomicAdd(&s_out, 1u);
                if (at < (uint32_t)kp2) keys[at] = key;
            }
        }
        __syncthreads();
        for (int size = 2; size <= kp2; size <<= 1) {
            for (int stride = size >> 1; stride > 0; stride >>= 1) {
                for (int t = tid; t < kp2 / 2; t += SEL_THREADS) {
                    const int lo = 2 * t - (t & (stride - 1));
                    const int hi = lo + stride;
                    const bool desc = (lo & size) == 0;
                    const u64 a = keys[lo], b = keys[hi];
                    if ((a < b) == desc) {
                        keys[lo] = b;
                        keys[hi] = a;
                    }
                }
                __syncthreads();
            }
        }
        for (int r = tid; r < k; r += SEL_THREADS) {
            out_ids[q * k + r] = key_id(keys[r]);
            out_scores[q * k + r] = key_score(keys[r]);
        }
    }
}

}  // namespace

hipError_t launch_select(u64 *cand, uint32_t *cnt, uint32_t cap, int32_t k_prime, int64_t Q, u64 *tau, u64 *tmp,
                         uint32_t *lost, int32_t *flags, int32_t stage, hipStream_t stream)
{
    if (Q <= 0) return hipSuccess;
    hipLaunchKernelGGL(select_kernel, dim3((unsigned)Q), dim3(SEL_THREADS), 0, stream, cand, cnt, cap, k_prime, tau, tmp,
                       lost, flags, stage);
    return hipGetLastError();
}

hipError_t launch_rescore(const u64 *cand, const uint32_t *cnt, uint32_t cap, int32_t k_prime, const float *queries,
                          int64_t Q, const void *exact, int32_t exact_dtype, int64_t ld, int32_t d, int32_t metric,
                          int32_t k, int32_t *out_ids, float *out_scores, float *out_margin,
                          const CertifyParams &cert, hipStream_t stream)
{
    if (Q <= 0) return hipSuccess;
    int kp2 = 2;
    while (kp2 < k_prime) kp2 <<= 1;
    const size_t smem = (size_t)kp2 * sizeof(u64);
#define RALM_RS(EXV, L2V)                                                                                    \
    hipLaunchKernelGGL((rescore_kernel<EXV, L2V>), dim3((unsigned)Q), dim3(RS_THREADS), smem, stream, cand, cnt, \
                       cap, k_prime, kp2, queries, exact, ld, d, k, out_ids, out_scores, out_margin, cert)
    if (exact_dtype == DT_F16) {
        if (metric == METRIC_L2) RALM_RS(DT_F16, true);
        else RALM_RS(DT_F16, false);
    } else {
        if (metric == METRIC_L2) RALM_RS(DT_F32, true);
        else RALM_RS(DT_F32, false);
    }
#undef RALM_RS
    return hipGetLastError();
}

hipError_t launch_exact_pass(const float *queries, int64_t Q, const void *exact, int32_t exact_dtype, int64_t ld,
                             int64_t N, int32_t d, int32_t metric, int32_t k, const int32_t *fb_list, int32_t *flags,
                             const u64 *tau_exact, u64 *cand, uint32_t *cnt, uint32_t cap, int32_t *out_ids,
                             float *out_scores, int n_cu, hipStream_t stream)
{
    if (Q <= 0) return hipSuccess;
    // as many of the queries at a time as fit 64 KB of LDS in fp32, at most XS_QG
    int qgroup = (64 * 1024) / (d * 4);
    if (qgroup > XS_QG) qgroup = XS_QG;
    if (qgroup < 1) return hipErrorInvalidValue;   // d <= 16384 is checked by the caller
    const size_t smem = (size_t)qgroup * d * 4;
    // both kernels return at once when no query needs them; their grids do not depend on that count,
    // which only the device knows
    int64_t rows_per_pass = (int64_t)n_cu * 4 * XS_WAVES;
    int64_t grid = N < rows_per_pass ? (N + XS_WAVES - 1) / XS_WAVES : (int64_t)n_cu * 4;
#define RALM_XS(EXV, L2V)                                                                                       \
    do {                                                                                                        \
        auto kern = exact_scan_kernel<EXV, L2V>;                                                                \
        static std::atomic<bool> attr_done{false};                                                              \
        if (!attr_done.load(std::memory_order_acquire)) {                                                       \
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),                            \
                                               hipFuncAttributeMaxDynamicSharedMemorySize, 64 * 1024);          \
            if (e != hipSuccess) return e;                                                                      \
            attr_done.store(true, std::memory_order_release);                                                   \
        }                                                                                                       \
        hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(XS_THREADS), smem, stream, queries, exact, ld, N, d, \
                           qgroup, fb_list, flags, tau_exact, cand, cnt, cap);                                  \
    } while (0)
    // matrix-core form: inner product, rows of a multiple of 4 sixteen-byte pieces per lane, queries of
    // a group within 128 KB of LDS
    const int nc = d / (exact_dtype == DT_F32 ? 16 : 32);
    const bool mfma = metric == METRIC_IP && d % (exact_dtype == DT_F32 ? 64 : 128) == 0 && d <= 2048;
#define RALM_XM(EXV, SEGV)                                                                                      \
    do {                                                                                                        \
        auto kern = exact_scan_mfma_kernel<EXV, SEGV>;                                                          \
        static std::atomic<bool> attr_done{false};                                                              \
        if (!attr_done.load(std::memory_order_acquire)) {                                                       \
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),                            \
                                               hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024);         \
            if (e != hipSuccess) return e;                                                                      \
            attr_done.store(true, std::memory_order_release);                                                   \
        }                                                                                                       \
        const int64_t nblk = (N + 15) / 16, wgs = (int64_t)n_cu * ((size_t)d * 64 * 2 <= 150 * 1024 ? 2 : 1);   \
        const int64_t g = nblk < wgs * XM_NW ? (nblk + XM_NW - 1) / XM_NW : wgs;                                \
        hipLaunchKernelGGL(kern, dim3((unsigned)g), dim3(XM_NW * 64), (size_t)d * 64, stream, queries, exact, ld, N, \
                           d, fb_list, flags, tau_exact, cand, cnt, cap);                                       \
    } while (0)
#define RALM_XM_SEG(EXV)                  \
    do {                                  \
        if (nc % 8 == 0) RALM_XM(EXV, 8); \
        else if (nc % 6 == 0) RALM_XM(EXV, 6); \
        else RALM_XM(EXV, 4);             \
    } while (0)
    if (exact_dtype == DT_F16) {
        if (metric == METRIC_L2) RALM_XS(DT_F16, true);
        else if (mfma) RALM_XM_SEG(DT_F16);
        else RALM_XS(DT_F16, false);
    } else {
        if (metric == METRIC_L2) RALM_XS(DT_F32, true);
        else if (mfma) RALM_XM_SEG(DT_F32);
        else RALM_XS(DT_F32, false);
    }
#undef RALM_XM_SEG
#undef RALM_XM
#undef RALM_XS
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    int kp2 = 2;
    while (kp2 < k) kp2 <<= 1;
    const int64_t fgrid = Q < 256 ? Q : 256;
    hipLaunchKernelGGL(exact_finish_kernel, dim3((unsigned)fgrid), dim3(SEL_THREADS), (size_t)kp2 * sizeof(u64), stream,
                       cand, cnt, cap, k, kp2, fb_list, flags, out_ids, out_scores);
    return hipGetLastError();
}

}  // namespace ralm
