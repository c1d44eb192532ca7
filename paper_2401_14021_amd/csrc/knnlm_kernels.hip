// KNN-LM neighbour distribution (Section 5.3): from the k retrieved entries of a query to
// weights over their target tokens.
//
//  knnlm_probs_kernel  weight_i = exp(s_i / T) / sum_j exp(s_j / T) over the query's retrieved
//                      entries (s = retrieval score: larger is closer), token_i = values[id_i];
//                      the probability of a token is the sum of the weights of the entries that
//                      carry it; the most probable token (smallest id on ties) is reported.
//                      All of it in double, rounded once to fp32 on output.
#include "ralm_common.h"
#include "ralm_kernels.h"

namespace ralm {

namespace {

constexpr int KP_THREADS = 256, KP_WAVES = KP_THREADS / 64;

__device__ __forceinline__ double block_sum(double x, double *red /*[KP_WAVES]*/)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = x;
    __syncthreads();
    double t = 0.0;
    for (int w = 0; w < KP_WAVES; ++w) t += red[w];
    return t;
}
__device__ __forceinline__ double block_max(double x, double *red)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const double y = __shfl_xor(x, o, 64);
        x = y > x ? y : x;
    }
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = x;
    __syncthreads();
    double t = red[0];
    for (int w = 1; w < KP_WAVES; ++w) t = red[w] > t ? red[w] : t;
    return t;
}

// one workgroup per query
__global__ __launch_bounds__(KP_THREADS) void knnlm_probs_kernel(
    const int32_t *__restrict__ ids, const float *__restrict__ scores, int k, int kp2,
    const int32_t *__restrict__ values, int64_t N, double T, int32_t *__restrict__ tokens,
    float *__restrict__ weights, int32_t *__restrict__ top_token, float *__restrict__ top_prob)
{
    extern __shared__ __align__(16) unsigned char smem[];
    double *e = reinterpret_cast<double *>(smem);     // [kp2] weight of the entry at each rank
    u64 *keys = reinterpret_cast<u64 *>(e + kp2);      // [kp2] (token, rank), sorted by token then rank
    __shared__ double red[KP_WAVES];
    __shared__ double s_p[KP_THREADS];
    __shared__ int32_t s_tok[KP_THREADS];

    const int64_t q = blockIdx.x;
    const int tid = threadIdx.x;
    const int32_t *id = ids + q * k;
    const float *sc = scores + q * k;

    double best = -__builtin_inf();
    for (int i = tid; i < k; i += KP_THREADS) {
        const int32_t j = id[i];
        if (j >= 0 && (int64_t)j < N) {
            const double s = (double)sc[i];
            best = s > best ? s : best;
        }
    }
    best = block_max(best, red);

    double part = 0.0;
    for (int i = tid; i < kp2; i += KP_THREADS) {
        double x = 0.0;
        u64 key = ~0ull;
        if (i < k) {
            const int32_t j = id[i];
            const bool ok = j >= 0 && (int64_t)j < N;
            int32_t tok = -1;
            if (ok) {
                x = exp(((double)sc[i] - best) / T);
                tok = values[j];
                key = ((u64)((uint32_t)tok ^ 0x80000000u) << 32) | (uint32_t)i;
            }
            tokens[q * k + i] = tok;
        }
        e[i] = x;
        keys[i] = key;
        part += x;
    }
    const double Z = block_sum(part, red);
    for (int i = tid; i < k; i += KP_THREADS) {
        const double w = Z > 0.0 ? e[i] / Z : 0.0;
        e[i] = w;
        weights[q * k + i] = (float)w;
    }
    if (!top_token && !top_prob) return;
    __syncthreads();

    // entries grouped by token, ranks ascending inside a group
    for (int size = 2; size <= kp2; size <<= 1) {
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            for (int t = tid; t < kp2 / 2; t += KP_THREADS) {
                const int lo = 2 * t - (t & (stride - 1));
                const int hi = lo + stride;
                const bool asc = (lo & size) == 0;
                const u64 a = keys[lo], b = keys[hi];
                if ((a > b) == asc) {
                    keys[lo] = b;
                    keys[hi] = a;
                }
            }
            __syncthreads();
        }
    }
    // the thread at the start of a group adds the group's weights in rank order
    double my_p = -1.0;
    int32_t my_tok = -1;
    for (int i = tid; i < kp2; i += KP_THREADS) {
        const u64 key = keys[i];
        if (key == ~0ull) continue;
        const uint32_t t32 = (uint32_t)(key >> 32);
        if (i > 0 && (uint32_t)(keys[i - 1] >> 32) == t32) continue;
        double p = 0.0;
        for (int j = i; j < kp2 && (uint32_t)(keys[j] >> 32) == t32 && keys[j] != ~0ull; ++j)
            p += e[(uint32_t)keys[j]];
        const int32_t tok = (int32_t)(t32 ^ 0x80000000u);
        if (p > my_p || (p == my_p && tok < my_tok)) {
            my_p = p;
            my_tok = tok;
        }
    }
    s_p[tid] = my_p;
    s_tok[tid] = my_tok;
    __syncthreads();
    for (int o = KP_THREADS / 2; o > 0; o >>= 1) {
        if (tid < o) {
            const double p2 = s_p[tid + o];
            const int32_t t2 = s_tok[tid + o];
            if (p2 > s_p[tid] || (p2 == s_p[tid] && p2 >= 0.0 && t2 < s_tok[tid])) {
                s_p[tid] = p2;
                s_tok[tid] = t2;
            }
        }
        __syncthreads();
    }
    if (tid == 0) {
        const bool any = s_p[0] >= 0.0;
        if (top_token) top_token[q] = any ? s_tok[0] : -1;
        if (top_prob) top_prob[q] = any ? (float)s_p[0] : 0.f;
    }
}

}  // namespace

hipError_t launch_knnlm_probs(const int32_t *ids, const float *scores, int64_t Q, int32_t k, const int32_t *values,
                              int64_t N, double T, int32_t *tokens, float *weights, int32_t *top_token,
                              float *top_prob, hipStream_t stream)
{
    if (Q <= 0) return hipSuccess;
    int kp2 = 2;
    while (kp2 < k) kp2 <<= 1;
    const size_t smem = (size_t)kp2 * 16;
    hipLaunchKernelGGL(knnlm_probs_kernel, dim3((unsigned)Q), dim3(KP_THREADS), smem, stream, ids, scores, k, kp2,
                       values, N, T, tokens, weights, top_token, top_prob);
    return hipGetLastError();
}

}  // namespace ralm
