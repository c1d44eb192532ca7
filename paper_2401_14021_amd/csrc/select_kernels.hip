// Per-query selection and exact re-scoring (gfx950).
//
//  select_kernel   exact k'-th best of a query's candidate keys by an 8-bit radix descent
//                  over the 64-bit ranking key; writes it as the admission key for the next
//                  scan stage and cuts the list down to its k' best keys in place.
//  rescore_kernel  for the k' rows kept by the scan: inner product with the fp32 query from
//                  the EXACT datastore copy, products and sum in double, one rounding to
//                  fp32; final ranking (score descending, id ascending); first k written.
//                  This is what makes the result that of the paper's exact dense retriever
//                  (Section 5.1) although the scan ran in bf16/fp16.
#include "ralm_common.h"
#include "ralm_kernels.h"

namespace ralm {

namespace {

constexpr int SEL_THREADS = 1024;

// Exact k'-th best key of a list by a radix descent, 8 bits of the key per pass, from the top.
// A pass histograms the digit of the keys that match the prefix found so far; wave 0 walks the
// 256 bins from the best digit down to the one that holds the k'-th key.  As soon as that bin
// holds a single key the descent stops and one more pass over the list fetches that key
// (scores are mostly distinct, so this usually happens before the id bits are reached).
__global__ __launch_bounds__(SEL_THREADS) void select_kernel(u64 *__restrict__ cand, uint32_t *__restrict__ cnt,
                                                             uint32_t cap, int k_prime, u64 *__restrict__ tau,
                                                             u64 *__restrict__ tmp,
                                                             int32_t *__restrict__ overflow_count)
{
    __shared__ uint32_t hist[256];
    __shared__ uint32_t s_digit, s_remaining, s_bin, s_out;
    __shared__ u64 s_kth;

    const int64_t q = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63;
    const uint32_t n = cnt[q];
    u64 *c = cand + q * (int64_t)cap;

    if (n == 0xffffffffu) return;   // flagged by an earlier stage
    if (n > cap) {                  // list overflowed: this query cannot be answered from it
        if (tid == 0) {
            tau[q] = ~0ull;         // admits nothing from now on
            cnt[q] = 0xffffffffu;
            atomicAdd(overflow_count, 1);
        }
        return;
    }
    if (n < (uint32_t)k_prime) {    // fewer than k' candidates exist so far: keep admitting everything
        if (tid == 0) tau[q] = 0ull;
        return;
    }

    u64 prefix = 0, mask = 0;
    uint32_t remaining = (uint32_t)k_prime;
    bool single = false;
    for (int shift = 56; shift >= 0; shift -= 8) {
        if (tid < 256) hist[tid] = 0;
        __syncthreads();
        for (uint32_t i = tid; i < n; i += SEL_THREADS) {
            const u64 key = c[i];
            if ((key & mask) == prefix) atomicAdd(&hist[(uint32_t)(key >> shift) & 255u], 1u);
        }
        __syncthreads();
        if (tid < 64) {
            // lane l owns digits 255-4l .. 252-4l, best first
            uint32_t h[4], tot = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                h[j] = hist[255 - 4 * lane - j];
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
                    s_digit = 255 - 4 * lane - j;
                    s_remaining = remaining - run;
                    s_bin = h[j];
                }
                run += h[j];
            }
        }
        __syncthreads();
        prefix |= (u64)s_digit << shift;
        mask |= 0xffull << shift;
        remaining = s_remaining;
        if (s_bin == 1) {
            single = shift > 0;
            break;
        }
    }
    u64 kth = prefix;
    if (single) {   // the only key under the prefix is the k'-th
        for (uint32_t i = tid; i < n; i += SEL_THREADS) {
            const u64 key = c[i];
            if ((key & mask) == prefix) s_kth = key;
        }
        __syncthreads();
        kth = s_kth;
    }
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

__device__ __forceinline__ double wave_sum(double x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
    return x;
}

constexpr int RS_THREADS = 1024, RS_WAVES = RS_THREADS / 64;

// EX: DT_F32 or DT_F16 exact rows.  L2: the score is minus the squared distance; the scan's
// score of a row is then 2<q, x> - |x|^2, so |q|^2 is subtracted from it for the margin.
template <int EX, bool L2>
__global__ __launch_bounds__(RS_THREADS) void rescore_kernel(const u64 *__restrict__ cand,
                                                      const uint32_t *__restrict__ cnt, uint32_t cap,
                                                      int k_prime, int kp2, const float *__restrict__ queries,
                                                      const void *__restrict__ exact, int64_t ld, int d,
                                                      int k, int32_t *__restrict__ out_ids,
                                                      float *__restrict__ out_scores,
                                                      float *__restrict__ out_margin)
{
    extern __shared__ __align__(16) unsigned char smem[];
    u64 *keys = reinterpret_cast<u64 *>(smem);   // [kp2]
    __shared__ u64 s_min_scan[RS_WAVES];

    const int64_t q = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t n_raw = cnt[q];
    const bool overflow = n_raw == 0xffffffffu;
    const int n = overflow ? 0 : (int)(n_raw < (uint32_t)k_prime ? n_raw : (uint32_t)k_prime);
    const u64 *mine = cand + q * (int64_t)cap;
    const float *qv = queries + q * (int64_t)d;

    u64 min_scan = ~0ull;
    for (int c = wave; c < n; c += RS_WAVES) {
        const u64 skey = mine[c];
        min_scan = skey < min_scan ? skey : min_scan;
        const int32_t id = key_id(skey);
        double sum = 0.0;
        if constexpr (EX == DT_F32) {
            const float *row = static_cast<const float *>(exact) + (int64_t)id * ld;
            for (int j = lane * 4; j < d; j += 256) {
                const float4 x = *reinterpret_cast<const float4 *>(row + j);
                const float4 y = *reinterpret_cast<const float4 *>(qv + j);
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
        } else {
            const uint16_t *row = static_cast<const uint16_t *>(exact) + (int64_t)id * ld;
            for (int j = lane * 8; j < d; j += 512) {
                const uint4 x = *reinterpret_cast<const uint4 *>(row + j);
                const float4 y0 = *reinterpret_cast<const float4 *>(qv + j);
                const float4 y1 = *reinterpret_cast<const float4 *>(qv + j + 4);
                const double xs[8] = {(double)f16_bits_to_f32(x.x & 0xffffu), (double)f16_bits_to_f32(x.x >> 16),
                                      (double)f16_bits_to_f32(x.y & 0xffffu), (double)f16_bits_to_f32(x.y >> 16),
                                      (double)f16_bits_to_f32(x.z & 0xffffu), (double)f16_bits_to_f32(x.z >> 16),
                                      (double)f16_bits_to_f32(x.w & 0xffffu), (double)f16_bits_to_f32(x.w >> 16)};
                const double ys[8] = {(double)y0.x, (double)y0.y, (double)y0.z, (double)y0.w,
                                      (double)y1.x, (double)y1.y, (double)y1.z, (double)y1.w};
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    if constexpr (L2) {
                        const double df = ys[u] - xs[u];
                        sum += df * df;
                    } else {
                        sum += xs[u] * ys[u];
                    }
                }
            }
        }
        sum = wave_sum(sum);
        if (lane == 0) keys[c] = make_key(L2 ? (float)(-sum) : (float)sum, id);
    }
    for (int c = n + tid; c < kp2; c += RS_THREADS) keys[c] = 0ull;
    if (lane == 0) s_min_scan[wave] = min_scan;
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
        out_scores[q * k + r] = have ? key_score(key) : (overflow ? __builtin_nanf("") : -__builtin_inff());
    }
    if (out_margin && tid == 0) {
        float q_sq = 0.f;
        if constexpr (L2) {
            double t = 0.0;
            for (int j = 0; j < d; ++j) t += (double)qv[j] * (double)qv[j];
            q_sq = (float)t;
        }
        u64 ms = s_min_scan[0];
        for (int w = 1; w < RS_WAVES; ++w) ms = s_min_scan[w] < ms ? s_min_scan[w] : ms;
        float margin;
        if (overflow || n < k)
            margin = __builtin_nanf("");
        else if (n < k_prime)
            margin = __builtin_inff();   // every row of the datastore was re-scored
        else
            margin = key_score(keys[k - 1]) - (key_score(ms) - q_sq);
        out_margin[q] = margin;
    }
}

}  // namespace

hipError_t launch_select(u64 *cand, uint32_t *cnt, uint32_t cap, int32_t k_prime, int64_t Q, u64 *tau, u64 *tmp,
                         int32_t *overflow_count, hipStream_t stream)
{
    if (Q <= 0) return hipSuccess;
    hipLaunchKernelGGL(select_kernel, dim3((unsigned)Q), dim3(SEL_THREADS), 0, stream, cand, cnt, cap, k_prime, tau, tmp,
                       overflow_count);
    return hipGetLastError();
}

hipError_t launch_rescore(const u64 *cand, const uint32_t *cnt, uint32_t cap, int32_t k_prime, const float *queries,
                          int64_t Q, const void *exact, int32_t exact_dtype, int64_t ld, int32_t d, int32_t metric,
                          int32_t k, int32_t *out_ids, float *out_scores, float *out_margin, hipStream_t stream)
{
    if (Q <= 0) return hipSuccess;
    int kp2 = 2;
    while (kp2 < k_prime) kp2 <<= 1;
    const size_t smem = (size_t)kp2 * sizeof(u64);
#define RALM_RS(EXV, L2V)                                                                                    \
    hipLaunchKernelGGL((rescore_kernel<EXV, L2V>), dim3((unsigned)Q), dim3(RS_THREADS), smem, stream, cand, cnt, \
                       cap, k_prime, kp2, queries, exact, ld, d, k, out_ids, out_scores, out_margin)
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

}  // namespace ralm
