// Speculative retrieval from the per-request caches, the verification compare, and the
// small elementwise helpers (gfx950).
//
//  cache_lookup_kernel  Q.retrieve(q_i) of Alg. 1: rank the request's cached rows with the
//                       retriever's own metric (Section 3 "Speculative retrieval", Fig. 2)
//                       and return the top one.  Scores are formed exactly as the final
//                       scores of the knowledge-base retrieval (double products and sum,
//                       one rounding to fp32; only the order of the double additions
//                       differs), so a cached entry gets the same number from both and
//                       "top-1 of the knowledge base is cached => it is the cache's top-1"
//                       holds.
//  cache_lookup_mfma_kernel  the same lookup with the sums formed on the fp64 matrix cores
//                       (inner product, rows that are whole 256-byte steps).
//  verify_kernel        m = argmin_i (d^_i != d_i) of Alg. 1, per request.
//  cache_insert_kernel  Q.insert(C.retrieve(..)) of Alg. 1: the ids a verification step
//                       retrieved go into the request's cache (Section 3 "Batched
//                       verification": top-1 or top-k update; Section 5.3: the next n rows
//                       after a retrieved one), skipping ids already cached, first in first
//                       out once the cache is full.
#include <atomic>
#include <type_traits>

#include "ralm_common.h"
#include "ralm_kernels.h"

namespace ralm {

namespace {

constexpr int CL_GS = 16;          // lanes that share one cached row
constexpr int CL_ROWS = 64 / CL_GS;   // rows per wave step
constexpr int CL_LDS_BYTES = 100 * 1024;   // queries of a request, widened to double

__device__ __forceinline__ void clamp_range(const int64_t *off, int64_t r, int64_t Qt, int64_t &lo, int64_t &hi)
{
    lo = off[r];
    hi = off[r + 1];
    lo = lo < 0 ? 0 : (lo > Qt ? Qt : lo);
    hi = hi < lo ? lo : (hi > Qt ? Qt : hi);
}

// elements (c*CL_GS + sub)*4 .. +4 of a cached row, c = 0 .. NCH-1, widened exactly to fp32 (zeros
// for a missing row and past d)
template <int EX, int NCH>
__device__ __forceinline__ void cl_load_row(float4 (&x)[NCH], const void *__restrict__ exact, int64_t ld, int32_t id,
                                            bool ok, int sub, int d)
{
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int j = (c * CL_GS + sub) * 4;
        x[c] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (ok && j < d) {
            if constexpr (EX == DT_F32) {
                x[c] = *reinterpret_cast<const float4 *>(static_cast<const float *>(exact) + (int64_t)id * ld + j);
            } else {
                const uint2 h = *reinterpret_cast<const uint2 *>(static_cast<const uint16_t *>(exact) + (int64_t)id * ld + j);
                x[c] = make_float4(f16_bits_to_f32(h.x & 0xffffu), f16_bits_to_f32(h.x >> 16),
                                   f16_bits_to_f32(h.y & 0xffffu), f16_bits_to_f32(h.y >> 16));
            }
        }
    }
}

constexpr int CL_QB = 4;    // queries scored together (independent sums hide the latency of the adds)
static_assert(CL_QB == 4, "the block dispatch in cache_lookup_kernel is written out for blocks of 4");

// NCH = float4 chunks of a row held by one lane (row element (c*CL_GS + sub)*4 .. +4).
// One block of NW waves per request.  A wave step scores CL_ROWS cached rows against all of the
// request's queries: the rows are gathered from the exact copy (while the previous rows are
// being scored: the loads of the next step are issued first), widened to double ONCE, and every
// query, kept in LDS as doubles, costs one fused multiply-add per element on top of that;
// CL_QB queries are scored together, whose independent sums hide the latency of the adds, and
// the 16 lane sums of a row meet through DPP.
// L2: the score is minus the squared distance (KNN-LM datastores) instead of the inner product.
// MAXQ (8 or 16): queries of a request held in LDS at a time (more are served in groups); their
// bests sit in registers, which is why wide rows take 8.
template <int EX, int NCH, int NW, bool L2, int MAXQ>
__global__ __launch_bounds__(NW * 64) void cache_lookup_kernel(
    const int32_t *__restrict__ cache_ids, const int32_t *__restrict__ cache_len, int C,
    const float *__restrict__ queries, int64_t Qt, const int64_t *__restrict__ q_offsets,
    const void *__restrict__ exact, int64_t ld, int64_t N, int d, int qgroup,
    int32_t *__restrict__ spec_ids, float *__restrict__ spec_scores, u64 *__restrict__ partial)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int dq = (d + 63) & ~63;                                  // a query's doubles in LDS
    double *qs = reinterpret_cast<double *>(smem);                  // [qgroup][dq], see below
    u64 *best = reinterpret_cast<u64 *>(qs + (size_t)qgroup * dq);  // [NW waves][CL_ROWS][qgroup]

    // gridDim.y workgroups share a request (few requests: spread each over many CUs); they then
    // merge their best keys with a 64-bit atomic max in `partial`, decoded by a second kernel
    const int64_t r = blockIdx.x;
    const int part = blockIdx.y, parts = gridDim.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int sub = lane % CL_GS, slot = lane / CL_GS;
    int64_t q_lo, q_hi;
    clamp_range(q_offsets, r, Qt, q_lo, q_hi);
    int len = cache_len[r];
    len = len < 0 ? 0 : (len > C ? C : len);
    const int32_t *ids = cache_ids + r * (int64_t)C;
    const int e_step = parts * NW * CL_ROWS;

    for (int64_t g0 = q_lo; g0 < q_hi; g0 += qgroup) {
        const int nq = (int)((q_hi - g0) < qgroup ? (q_hi - g0) : qgroup);
        __syncthreads();
        // A lane scores elements (c*16 + sub)*4 .. +3 of a row.  The query's elements are laid
        // out so that, for one c, the first two of the 16 lanes' four are contiguous (256 bytes),
        // then the last two: the two 16-byte reads of a lane are then free of bank conflicts.
        for (int i = tid * 4; i < nq * d; i += NW * 256) {
            const int qi = i / d, j = i - qi * d;
            const float4 y = *reinterpret_cast<const float4 *>(queries + g0 * d + i);
            double *dst = qs + (size_t)qi * dq + ((j >> 6) * 64) + ((j >> 2) & 15) * 2;
            dst[0] = (double)y.x;
            dst[1] = (double)y.y;
            dst[32] = (double)y.z;
            dst[33] = (double)y.w;
        }
        for (int i = tid; i < NW * CL_ROWS * qgroup; i += NW * 64) best[i] = 0ull;
        __syncthreads();
        u64 *my_best = best + (wave * CL_ROWS + slot) * qgroup;
        // best (score, id) per query so far, in registers of the row's first lane: the comparison
        // is two float compares, and a key is formed only once, at the end
        float best_sc[MAXQ];
        int32_t best_id[MAXQ];
#pragma unroll
        for (int i = 0; i < MAXQ; ++i) {
            best_sc[i] = -__builtin_inff();
            best_id[i] = -1;
        }

        int e0 = (part * NW + wave) * CL_ROWS;
        float4 xn[NCH];   // the next step's rows, in flight while this step's are scored
        int32_t id_n = e0 + slot < len ? ids[e0 + slot] : -1;
        bool ok_n = id_n >= 0 && (int64_t)id_n < N;
        cl_load_row<EX, NCH>(xn, exact, ld, id_n, ok_n, sub, d);
        for (; e0 < len; e0 += e_step) {
            const int32_t id = id_n;
            const bool ok = ok_n;
            double x[NCH][4];
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                x[c][0] = (double)xn[c].x;
                x[c][1] = (double)xn[c].y;
                x[c][2] = (double)xn[c].z;
                x[c][3] = (double)xn[c].w;
            }
            const int e_n = e0 + e_step + slot;
            id_n = e_n < len ? ids[e_n] : -1;
            ok_n = id_n >= 0 && (int64_t)id_n < N;
            cl_load_row<EX, NCH>(xn, exact, ld, id_n, ok_n, sub, d);

            // U queries q0 .. q0+U-1 against this step's rows
            auto score = [&](auto u_tag, auto q0_tag) __attribute__((always_inline)) {
                constexpr int U = decltype(u_tag)::value, q0 = decltype(q0_tag)::value;
                const double *qv[U];
                double sum[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    qv[u] = qs + (size_t)(q0 + u) * dq + sub * 2;
                    sum[u] = 0.0;
                }
#pragma unroll
                for (int c = 0; c < NCH; ++c) {
                    if ((c * CL_GS + sub) * 4 < d) {
#pragma unroll
                        for (int u = 0; u < U; ++u) {
                            const double2 y01 = *reinterpret_cast<const double2 *>(qv[u] + c * 64);
                            const double2 y23 = *reinterpret_cast<const double2 *>(qv[u] + c * 64 + 32);
                            if constexpr (L2) {
                                const double d0 = y01.x - x[c][0], d1 = y01.y - x[c][1];
                                const double d2 = y23.x - x[c][2], d3 = y23.y - x[c][3];
                                sum[u] += d0 * d0;
                                sum[u] += d1 * d1;
                                sum[u] += d2 * d2;
                                sum[u] += d3 * d3;
                            } else {
                                sum[u] += x[c][0] * y01.x;
                                sum[u] += x[c][1] * y01.y;
                                sum[u] += x[c][2] * y23.x;
                                sum[u] += x[c][3] * y23.y;
                            }
                        }
                    }
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const double t = row16_sum(sum[u]);
                    const float sc = (L2 ? (float)(-t) : (float)t) + 0.0f;   // -0 counts as +0, as in a key
                    // higher score, then lower id (ids of missing rows are -1 and never win)
                    const bool better = ok && (sc > best_sc[q0 + u] || (sc == best_sc[q0 + u] && id < best_id[q0 + u]));
                    best_sc[q0 + u] = better ? sc : best_sc[q0 + u];
                    best_id[q0 + u] = better ? id : best_id[q0 + u];
                }
            };
            // query blocks of CL_QB, the last one with as many sums as there are queries left
            // (block starts are compile-time constants: the bests are indexed statically)
            auto block = [&](auto q0_tag) __attribute__((always_inline)) {
                constexpr int q0 = decltype(q0_tag)::value;
                const int left = nq - q0;
                if (left >= 4) score(std::integral_constant<int, 4>{}, q0_tag);
                else if (left == 3) score(std::integral_constant<int, 3>{}, q0_tag);
                else if (left == 2) score(std::integral_constant<int, 2>{}, q0_tag);
                else if (left == 1) score(std::integral_constant<int, 1>{}, q0_tag);
            };
            block(std::integral_constant<int, 0>{});
            if (nq > 4) block(std::integral_constant<int, 4>{});
            if constexpr (MAXQ > 8) {
                if (nq > 8) block(std::integral_constant<int, 8>{});
                if (nq > 12) block(std::integral_constant<int, 12>{});
            }
        }
        if (sub == 0) {
#pragma unroll
            for (int i = 0; i < MAXQ; ++i)
                if (i < nq && best_id[i] >= 0) my_best[i] = make_key(best_sc[i], best_id[i]);
        }
        __syncthreads();
        for (int qi = tid; qi < nq; qi += NW * 64) {
            u64 b = 0ull;
            for (int w = 0; w < NW * CL_ROWS; ++w) {
                const u64 v = best[w * qgroup + qi];
                b = v > b ? v : b;
            }
            if (partial) {
                if (b) atomicMax(reinterpret_cast<unsigned long long *>(partial + g0 + qi), b);
            } else {
                spec_ids[g0 + qi] = b ? key_id(b) : -1;
                spec_scores[g0 + qi] = b ? key_score(b) : -__builtin_inff();
            }
        }
    }
}

// ---- the same lookup on the fp64 matrix cores (inner-product metric) ---------------------------
// v_mfma_f64_4x4x4 multiplies four independent 4x4x4 blocks: operand A of lane l is element
// (i = l%4, k = l/16) of block (l/4)%4, operand B element (k = l/16, j = l%4) of that block, and
// the lane receives D(i = l/16, j = l%4).  Block b takes cached rows 4b .. 4b+3 of a step of 16
// rows and all blocks take the same 4 queries, so lane l feeds row l%16 and gets the score of row
// 4*((l/4)%4) + l/16 against query l%4: a step of 16 rows x 4 queries x 4 elements per
// instruction, sums in double, and no reduction across lanes.  A lane holds elements
// 4*CH*u + CH*(l/16) .. + CH-1 of its row (CH elements per 16-byte load: whole 64-byte pieces of
// a row per load instruction); the queries sit in LDS as doubles in the order the instructions
// consume them ([group of 4][instruction][k][j]: a wave reads 128 contiguous bytes, no bank
// conflicts).  More than 4 queries: one more instruction per group and element, same row operand.
constexpr int CM_NW = 8;
constexpr int CM_MAX_GROUPS = 4;     // groups of 4 queries whose doubles are in LDS at a time

// SEG = 16-byte pieces of a row that a lane has in flight per buffer; it divides the number of
// pieces per lane and row, d / (4 * CH).
template <int EX, int SEG>
__global__ __launch_bounds__(CM_NW * 64) void cache_lookup_mfma_kernel(
    const int32_t *__restrict__ cache_ids, const int32_t *__restrict__ cache_len, int C,
    const float *__restrict__ queries, int64_t Qt, const int64_t *__restrict__ q_offsets,
    const void *__restrict__ exact, int64_t ld, int64_t N, int d, int ng_max,
    int32_t *__restrict__ spec_ids, float *__restrict__ spec_scores, u64 *__restrict__ partial)
{
    constexpr int CH = EX == DT_F32 ? 4 : 8;        // elements per 16-byte piece
    constexpr int ES = EX == DT_F32 ? 4 : 2;
    extern __shared__ __align__(16) unsigned char smem[];
    const int T = d / 4;                             // instructions per step and query group
    double *bq = reinterpret_cast<double *>(smem);   // [ng_max][T][4 k][4 j]
    u64 *best = reinterpret_cast<u64 *>(bq + (size_t)ng_max * T * 16);   // [4 * ng_max]

    const int64_t r = blockIdx.x;
    const int part = blockIdx.y, parts = gridDim.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r16 = lane & 15, kq = lane >> 4;            // row of the step and k index this lane feeds
    const int ro = ((lane >> 2) & 3) * 4 + (lane >> 4);   // row of the step whose score this lane receives
    const int jq = lane & 3;                              // ... against this query of a group
    int64_t q_lo, q_hi;
    clamp_range(q_offsets, r, Qt, q_lo, q_hi);
    int len = cache_len[r];
    len = len < 0 ? 0 : (len > C ? C : len);
    const int32_t *ids = cache_ids + r * (int64_t)C;
    const int NC = d / (4 * CH);                          // pieces per lane and row
    const int nsegs = NC / SEG;
    const int nblk = (len + 15) / 16;
    const int blk_step = parts * CM_NW;
    const unsigned char *base = static_cast<const unsigned char *>(exact) + kq * 16;

    for (int64_t g0 = q_lo; g0 < q_hi; g0 += 4 * ng_max) {
        const int nq = (int)((q_hi - g0) < 4 * ng_max ? (q_hi - g0) : 4 * ng_max);
        const int n_groups = (nq + 3) >> 2;
        __syncthreads();
        for (int i = tid; i < n_groups * 4 * d; i += CM_NW * 64) {
            const int qi = i / d, e = i - qi * d;
            const double v = qi < nq ? (double)queries[(g0 + qi) * d + e] : 0.0;
            const int t = CH * (e / (4 * CH)) + e % CH, k = (e / CH) & 3;
            bq[((size_t)(qi >> 2) * T + t) * 16 + k * 4 + (qi & 3)] = v;
        }
        for (int i = tid; i < 4 * ng_max; i += CM_NW * 64) best[i] = 0ull;
        __syncthreads();

        auto run = [&](auto ng_tag) __attribute__((always_inline)) {
            constexpr int NG = decltype(ng_tag)::value;
            float best_sc[NG];
            int32_t best_id[NG];
            double acc[NG];
#pragma unroll
            for (int g = 0; g < NG; ++g) {
                best_sc[g] = -__builtin_inff();
                best_id[g] = -1;
                acc[g] = 0.0;
            }
            int blk = part * CM_NW + wave;
            if (blk >= nblk) return;
            // ids of the rows this lane feeds and receives, for this step and (ahead) the next
            auto id_at = [&](int e) { return e < len ? ids[e] : -1; };
            auto row_of = [&](int32_t id) {
                const bool ok = id >= 0 && (int64_t)id < N;
                return base + (int64_t)(ok ? id : 0) * ld * ES;
            };
            int32_t id_out = id_at(blk * 16 + ro);
            const unsigned char *row = row_of(id_at(blk * 16 + r16));
            int32_t id_feed_n = id_at((blk + blk_step) * 16 + r16), id_out_n = id_at((blk + blk_step) * 16 + ro);
            int seg = 0;
            uint4 buf0[SEG], buf1[SEG];
            auto load = [&](uint4(&buf)[SEG], const unsigned char *rw, int sg) __attribute__((always_inline)) {
#pragma unroll
                for (int c = 0; c < SEG; ++c) buf[c] = *reinterpret_cast<const uint4 *>(rw + (size_t)(sg * SEG + c) * 64);
            };
            // one (step, segment) item: issue the next item's loads, multiply this one's pieces
            auto item = [&](uint4(&cur)[SEG], uint4(&nxt)[SEG]) __attribute__((always_inline)) -> bool {
                const bool last_seg = seg + 1 == nsegs;
                const int blk_n = last_seg ? blk + blk_step : blk;
                const bool more = blk_n < nblk;
                const unsigned char *row_n = last_seg ? row_of(id_feed_n) : row;
                if (more) load(nxt, row_n, last_seg ? 0 : seg + 1);
                const double *bl = bq + (size_t)seg * (SEG * CH * 16) + kq * 4 + jq;
#pragma unroll
                for (int c = 0; c < SEG; ++c) {
                    {
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
                        for (int e = 0; e < CH; ++e) {
#pragma unroll
                            for (int g = 0; g < NG; ++g)
                                acc[g] = __builtin_amdgcn_mfma_f64_4x4x4f64(a[e], bl[((size_t)g * T + c * CH + e) * 16], acc[g], 0, 0, 0);
                        }
                    }
                }
                if (last_seg) {
                    const bool ok = id_out >= 0 && (int64_t)id_out < N;
#pragma unroll
                    for (int g = 0; g < NG; ++g) {
                        const float sc = (float)acc[g] + 0.0f;   // -0 counts as +0, as in a key
                        // higher score, then lower id
                        const bool better = ok && g * 4 + jq < nq &&
                                            (sc > best_sc[g] || (sc == best_sc[g] && id_out < best_id[g]));
                        best_sc[g] = better ? sc : best_sc[g];
                        best_id[g] = better ? id_out : best_id[g];
                        acc[g] = 0.0;
                    }
                    blk = blk_n;
                    seg = 0;
                    row = row_n;
                    id_out = id_out_n;
                    if (more) {
                        id_feed_n = id_at((blk + blk_step) * 16 + r16);
                        id_out_n = id_at((blk + blk_step) * 16 + ro);
                    }
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
#pragma unroll
            for (int g = 0; g < NG; ++g)
                if (best_id[g] >= 0)
                    atomicMax(reinterpret_cast<unsigned long long *>(best + g * 4 + jq), make_key(best_sc[g], best_id[g]));
        };
        if (n_groups == 1) run(std::integral_constant<int, 1>{});
        else if (n_groups == 2) run(std::integral_constant<int, 2>{});
        else if (n_groups == 3) run(std::integral_constant<int, 3>{});
        else run(std::integral_constant<int, 4>{});
        __syncthreads();
        for (int qi = tid; qi < nq; qi += CM_NW * 64) {
            const u64 b = best[qi];
            if (partial) {
                if (b) atomicMax(reinterpret_cast<unsigned long long *>(partial + g0 + qi), b);
            } else {
                spec_ids[g0 + qi] = b ? key_id(b) : -1;
                spec_scores[g0 + qi] = b ? key_score(b) : -__builtin_inff();
            }
        }
    }
}

// decodes the merged keys of the split lookup; one wave per request
__global__ __launch_bounds__(256) void cache_lookup_finish_kernel(const u64 *__restrict__ partial, int64_t Qt,
                                                                  const int64_t *__restrict__ q_offsets, int64_t R,
                                                                  int32_t *__restrict__ spec_ids,
                                                                  float *__restrict__ spec_scores)
{
    const int lane = threadIdx.x & 63;
    const int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= R) return;
    int64_t lo, hi;
    clamp_range(q_offsets, r, Qt, lo, hi);
    for (int64_t q = lo + lane; q < hi; q += 64) {
        const u64 b = partial[q];
        spec_ids[q] = b ? key_id(b) : -1;
        spec_scores[q] = b ? key_score(b) : -__builtin_inff();
    }
}

__global__ __launch_bounds__(256) void verify_kernel(const int32_t *__restrict__ spec,
                                                     const int32_t *__restrict__ truth,
                                                     int64_t true_stride, int64_t Qt,
                                                     const int64_t *__restrict__ q_offsets, int64_t R,
                                                     int32_t *__restrict__ first_mismatch)
{
    // one wave per request; lanes look at 64 consecutive steps at a time
    const int lane = threadIdx.x & 63;
    const int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= R) return;
    int64_t lo, hi;
    clamp_range(q_offsets, r, Qt, lo, hi);
    const int64_t s = hi - lo;
    int64_t m = s;
    for (int64_t base = 0; base < s; base += 64) {
        const int64_t i = base + lane;
        const bool differ = i < s && spec[lo + i] != truth[(lo + i) * true_stride];
        const unsigned long long mask = __ballot(differ);
        if (mask) {
            m = base + __ffsll((long long)mask) - 1;
            break;
        }
    }
    if (lane == 0) first_mismatch[r] = (int32_t)m;
}

// One wave per request; the request's cache row sits in LDS while it is updated.  Candidates
// are taken one at a time in the defined order (the outcome depends on it once the cache is
// full); the membership test of a candidate is spread over the 64 lanes, 4 ids per LDS read.
__global__ __launch_bounds__(64) void cache_insert_kernel(
    int32_t *__restrict__ cache_ids, int32_t *__restrict__ cache_len, int32_t *__restrict__ cache_head, int C,
    const int32_t *__restrict__ truth, int64_t true_stride, int64_t Qt, const int64_t *__restrict__ q_offsets,
    const int32_t *__restrict__ first_mismatch, int p, int n_next, int64_t N)
{
    extern __shared__ __align__(16) int32_t cs[];   // [C rounded up to 256]; slots >= len hold -1
    const int64_t r = blockIdx.x;
    const int lane = threadIdx.x;
    int64_t q_lo, q_hi;
    clamp_range(q_offsets, r, Qt, q_lo, q_hi);
    int64_t n = q_hi - q_lo;
    if (first_mismatch) {
        int64_t fm = first_mismatch[r];
        fm = fm < 0 ? 0 : fm;
        if (fm + 1 < n) n = fm + 1;        // steps up to and including the first mis-speculated one
    }
    if (n <= 0) return;
    int len = cache_len[r];
    len = len < 0 ? 0 : (len > C ? C : len);
    int head = cache_head[r];
    head = head < 0 || head >= C ? 0 : head;
    int32_t *ids = cache_ids + r * (int64_t)C;
    const int cpad = (C + 255) & ~255;
    for (int x = lane; x < cpad; x += 64) cs[x] = x < len ? ids[x] : -1;
    __syncthreads();

    const int first = n_next > 0 ? 1 : 0, last = n_next > 0 ? n_next : 0;
    for (int64_t i = 0; i < n; ++i) {
        for (int j = 0; j < p; ++j) {
            const int64_t t = truth[(q_lo + i) * true_stride + j];
            if (t < 0) continue;
            for (int o = first; o <= last; ++o) {
                const int64_t e64 = t + o;
                if (e64 >= N) break;
                const int32_t e = (int32_t)e64;
                bool found = false;
                for (int x = lane * 4; x < len; x += 256) {
                    const int4 v = *reinterpret_cast<const int4 *>(cs + x);
                    found |= v.x == e || v.y == e || v.z == e || v.w == e;
                }
                if (__any(found)) continue;
                int slot;
                if (len < C) {
                    slot = len++;
                } else {
                    slot = head;
                    head = head + 1 == C ? 0 : head + 1;
                }
                if (lane == 0) cs[slot] = e;
                __syncthreads();   // one wave: orders the LDS write before the next candidate's reads
            }
        }
    }
    for (int x = lane; x < len; x += 64) ids[x] = cs[x];
    if (lane == 0) {
        cache_len[r] = len;
        cache_head[r] = head;
    }
}

// Candidate lists for the k-entry cache retrieval: every query of a request gets the request's
// valid cached ids as ranking keys (score part 0), in any order; one workgroup per request.
__global__ __launch_bounds__(256) void cache_keys_kernel(const int32_t *__restrict__ cache_ids,
                                                         const int32_t *__restrict__ cache_len, int C, int64_t Qt,
                                                         const int64_t *__restrict__ q_offsets, int64_t N,
                                                         u64 *__restrict__ keys, uint32_t *__restrict__ cnt)
{
    __shared__ uint32_t s_n;
    const int64_t r = blockIdx.x;
    int64_t q_lo, q_hi;
    clamp_range(q_offsets, r, Qt, q_lo, q_hi);
    if (q_hi <= q_lo) return;
    int len = cache_len[r];
    len = len < 0 ? 0 : (len > C ? C : len);
    if (threadIdx.x == 0) s_n = 0;
    __syncthreads();
    for (int x = threadIdx.x; x < len; x += 256) {
        const int32_t id = cache_ids[r * (int64_t)C + x];
        if (id >= 0 && (int64_t)id < N) {
            const uint32_t at = atomicAdd(&s_n, 1u);
            const u64 key = make_key(0.f, id);
            for (int64_t q = q_lo; q < q_hi; ++q) keys[q * C + at] = key;
        }
    }
    __syncthreads();
    for (int64_t q = q_lo + threadIdx.x; q < q_hi; q += 256) cnt[q] = s_n;
}

__global__ void fill_u32_kernel(uint32_t *p, uint32_t v, int64_t n)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
        p[i] = v;
}
__global__ void fill_u64_kernel(u64 *p, u64 v, int64_t n)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
        p[i] = v;
}

// query preparation: queries rounded to the scan dtype, zero padded to [Qpad, dpad]
// L2: the scan scores a row as 2<q, x> - |x|^2, its squared norm being stored behind the row as the
// sum of two scan-dtype numbers (columns d and d+1): the query is doubled and gets -1 in both.
// The same launch clears two ranges of 32-bit words (the call's counters and list lengths), which
// saves three tiny launches per retrieval call.
template <int DT, bool L2>
__global__ void query_prep_kernel(const float *__restrict__ q, int64_t Q, int d, uint16_t *__restrict__ out,
                                  int64_t Qpad, int dpad, uint32_t *__restrict__ z0, int64_t n0,
                                  uint32_t *__restrict__ z1, int64_t n1)
{
    const int64_t n = Qpad * dpad;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n0; i += (int64_t)gridDim.x * blockDim.x) z0[i] = 0u;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n1; i += (int64_t)gridDim.x * blockDim.x) z1[i] = 0u;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t row = i / dpad;
        const int col = (int)(i % dpad);
        uint32_t bits = 0;
        if (row < Q && col < d) bits = f32_to_scan_bits<DT>(L2 ? 2.f * q[row * d + col] : q[row * d + col]);
        if (L2 && row < Q && (col == d || col == d + 1)) bits = f32_to_scan_bits<DT>(-1.f);
        out[i] = (uint16_t)bits;
    }
}

template <int DT>
__global__ void convert_rows_kernel(const float *__restrict__ src, int64_t src_ld, uint16_t *__restrict__ dst,
                                    int64_t dst_ld, int64_t N, int d8)
{
    // one 8-element chunk per thread step
    const int64_t n = N * d8;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t row = i / d8;
        const int c = (int)(i % d8) * 8;
        const float4 a = *reinterpret_cast<const float4 *>(src + row * src_ld + c);
        const float4 b = *reinterpret_cast<const float4 *>(src + row * src_ld + c + 4);
        *reinterpret_cast<uint4 *>(dst + row * dst_ld + c) = pack8<DT>(a, b);
    }
}

// Scan copy for the squared-distance metric: one wave per row.  dst row = the d elements rounded
// to the scan dtype (skipped when dst is src: fp16 keys that are their own scan copy), then the
// row's squared norm (summed in double from the source) as hi + lo in the scan dtype, then six
// zeros: 8 extra columns, 16 bytes.
template <int SRC, int DT>
__global__ __launch_bounds__(256) void l2_scan_copy_kernel(const void *src, int64_t src_ld,
                                                            uint16_t *dst, int64_t dst_ld, int64_t N, int d,
                                                            int in_place)
{
    const int lane = threadIdx.x & 63;
    // rows are strided over a bounded grid: one block per four rows would exceed the 2^32 work-items
    // of a launch from 67M rows on
    for (int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6); row < N; row += (int64_t)gridDim.x * 4) {
        double sum = 0.0;
        for (int c = lane * 8; c < d; c += 512) {
            float4 a, b;
            if constexpr (SRC == DT_F32) {
                const float *s = static_cast<const float *>(src) + row * src_ld + c;
                a = *reinterpret_cast<const float4 *>(s);
                b = *reinterpret_cast<const float4 *>(s + 4);
            } else {
                const uint4 h = *reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(src) + row * src_ld + c);
                a = make_float4(f16_bits_to_f32(h.x & 0xffffu), f16_bits_to_f32(h.x >> 16),
                                f16_bits_to_f32(h.y & 0xffffu), f16_bits_to_f32(h.y >> 16));
                b = make_float4(f16_bits_to_f32(h.z & 0xffffu), f16_bits_to_f32(h.z >> 16),
                                f16_bits_to_f32(h.w & 0xffffu), f16_bits_to_f32(h.w >> 16));
            }
            sum += (double)a.x * (double)a.x + (double)a.y * (double)a.y + (double)a.z * (double)a.z +
                   (double)a.w * (double)a.w + (double)b.x * (double)b.x + (double)b.y * (double)b.y +
                   (double)b.z * (double)b.z + (double)b.w * (double)b.w;
            if (!in_place) *reinterpret_cast<uint4 *>(dst + row * dst_ld + c) = pack8<DT>(a, b);
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o, 64);
        if (lane == 0) {
            const uint32_t hi = f32_to_scan_bits<DT>((float)sum);
            const float hi_f = DT == DT_F16 ? f16_bits_to_f32(hi) : __uint_as_float(hi << 16);
            const uint32_t lo = f32_to_scan_bits<DT>((float)(sum - (double)hi_f));
            *reinterpret_cast<uint4 *>(dst + row * dst_ld + d) = make_uint4(hi | (lo << 16), 0u, 0u, 0u);
        }
    }
}

int grid_for(int64_t n, int block)
{
    int64_t g = (n + block - 1) / block;
    if (g > 256 * 32) g = 256 * 32;
    if (g < 1) g = 1;
    return (int)g;
}

template <int EX, bool L2>
hipError_t launch_cache_ex(const int32_t *cache_ids, const int32_t *cache_len, int32_t C, int64_t R,
                           const float *queries, int64_t Qt, const int64_t *q_offsets, const void *exact,
                           int64_t ld, int64_t N, int32_t d, int32_t *spec_ids, float *spec_scores,
                           u64 *partial, int parts, hipStream_t stream)
{
    int qgroup = CL_LDS_BYTES / (((d + 63) & ~63) * 8);
    const int nch = (d + CL_GS * 4 - 1) / (CL_GS * 4);
    const int maxq = nch <= 12 ? 16 : 8;
    if (qgroup > maxq) qgroup = maxq;
    if (qgroup < 1) return hipErrorInvalidValue;
    // a lane keeps its NCH chunks in registers (as doubles, and the next rows' as floats), which
    // bounds the waves a block can hold
#define RALM_CL(NCHV, NWV, MAXQV)                                                                           \
    do {                                                                                                    \
        auto kern = cache_lookup_kernel<EX, NCHV, NWV, L2, MAXQV>;                                          \
        static std::atomic<bool> attr_done{false};                                                          \
        if (!attr_done.load(std::memory_order_acquire)) {                                                   \
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),                        \
                                               hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024);     \
            if (e != hipSuccess) return e;                                                                  \
            attr_done.store(true, std::memory_order_release);                                               \
        }                                                                                                   \
        hipLaunchKernelGGL(kern, dim3((unsigned)R, (unsigned)parts), dim3(NWV * 64),                        \
                           (size_t)qgroup * ((d + 63) & ~63) * 8 + (size_t)NWV * CL_ROWS * qgroup * sizeof(u64),   \
                           stream,                                                                          \
                           cache_ids, cache_len, C, queries, Qt, q_offsets, exact, ld, N, d, qgroup, spec_ids, \
                           spec_scores, partial);                                                           \
    } while (0)
    if (nch <= 4) RALM_CL(4, 8, 16);
    else if (nch <= 8) RALM_CL(8, 8, 16);
    else if (nch <= 12) RALM_CL(12, 8, 16);
    else if (nch <= 16) RALM_CL(16, 4, 8);
    else if (nch <= 32) RALM_CL(32, 4, 8);
    else return hipErrorInvalidValue;
#undef RALM_CL
    return hipGetLastError();
}

// The matrix-core form of the lookup, for the shapes it is written for: inner product, rows of a
// multiple of 16 sixteen-byte pieces (d % 64 == 0 for fp32 rows, d % 128 == 0 for fp16 rows).
template <int EX>
bool cache_mfma_fits(int32_t d)
{
    const int nc = d / (EX == DT_F32 ? 16 : 32);
    return d % (EX == DT_F32 ? 64 : 128) == 0 && nc >= 4 && (size_t)d * 32 <= 64 * 1024;
}

template <int EX>
hipError_t launch_cache_mfma(const int32_t *cache_ids, const int32_t *cache_len, int32_t C, int64_t R,
                             const float *queries, int64_t Qt, const int64_t *q_offsets, const void *exact,
                             int64_t ld, int64_t N, int32_t d, int32_t *spec_ids, float *spec_scores,
                             u64 *partial, int parts, hipStream_t stream)
{
    const int nc = d / (EX == DT_F32 ? 16 : 32);
    // a group of 4 queries takes d * 32 bytes of LDS; up to 64 KB, so that two requests share a CU
    int ng = (int)((64 * 1024) / ((size_t)d * 32));
    ng = ng > CM_MAX_GROUPS ? CM_MAX_GROUPS : ng;
    const size_t smem = (size_t)ng * d * 32 + (size_t)4 * ng * sizeof(u64);
#define RALM_CM(SEGV)                                                                                       \
    do {                                                                                                    \
        auto kern = cache_lookup_mfma_kernel<EX, SEGV>;                                                     \
        static std::atomic<bool> attr_done{false};                                                          \
        if (!attr_done.load(std::memory_order_acquire)) {                                                   \
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),                        \
                                               hipFuncAttributeMaxDynamicSharedMemorySize, 80 * 1024);      \
            if (e != hipSuccess) return e;                                                                  \
            attr_done.store(true, std::memory_order_release);                                               \
        }                                                                                                   \
        hipLaunchKernelGGL(kern, dim3((unsigned)R, (unsigned)parts), dim3(CM_NW * 64), smem, stream, cache_ids, \
                           cache_len, C, queries, Qt, q_offsets, exact, ld, N, d, ng, spec_ids, spec_scores,   \
                           partial);                                                                        \
    } while (0)
    if (nc % 8 == 0) RALM_CM(8);
    else if (nc % 6 == 0) RALM_CM(6);
    else RALM_CM(4);
#undef RALM_CM
    return hipGetLastError();
}

}  // namespace

hipError_t launch_cache_lookup(const int32_t *cache_ids, const int32_t *cache_len, int32_t C, int64_t R,
                               const float *queries, int64_t Qt, const int64_t *q_offsets,
                               const void *exact, int32_t exact_dtype, int64_t ld, int64_t N, int32_t d,
                               int32_t metric, int32_t *spec_ids, float *spec_scores, u64 *partial,
                               hipStream_t stream)
{
    if (R <= 0) return hipSuccess;
    // With few requests one workgroup per request leaves most of the chip idle: split every
    // request's cache over `parts` workgroups (at least 64 cached rows each), if the caller
    // gave scratch for the merge.
    int parts = 1;
    if (partial && R < 128) {
        const int64_t want = (256 + R - 1) / R, most = (C + 63) / 64;
        parts = (int)(want < most ? want : most);
        if (parts < 1) parts = 1;
    }
    if (parts == 1) partial = nullptr;
    hipError_t e = hipSuccess;
    if (partial) {
        e = launch_fill_u64(partial, 0ull, Qt, stream);
        if (e != hipSuccess) return e;
    }
#define RALM_CACHE(EXV, L2V)                                                                           \
    e = launch_cache_ex<EXV, L2V>(cache_ids, cache_len, C, R, queries, Qt, q_offsets, exact, ld, N, d, \
                                  spec_ids, spec_scores, partial, parts, stream)
#define RALM_CACHE_MFMA(EXV)                                                                             \
    e = launch_cache_mfma<EXV>(cache_ids, cache_len, C, R, queries, Qt, q_offsets, exact, ld, N, d, spec_ids, \
                               spec_scores, partial, parts, stream)
    if (exact_dtype == DT_F16) {
        if (metric == METRIC_L2) RALM_CACHE(DT_F16, true);
        else if (cache_mfma_fits<DT_F16>(d)) RALM_CACHE_MFMA(DT_F16);
        else RALM_CACHE(DT_F16, false);
    } else {
        if (metric == METRIC_L2) RALM_CACHE(DT_F32, true);
        else if (cache_mfma_fits<DT_F32>(d)) RALM_CACHE_MFMA(DT_F32);
        else RALM_CACHE(DT_F32, false);
    }
#undef RALM_CACHE_MFMA
#undef RALM_CACHE
    if (e != hipSuccess || !partial) return e;
    hipLaunchKernelGGL(cache_lookup_finish_kernel, dim3((unsigned)((R + 3) / 4)), dim3(256), 0, stream, partial, Qt,
                       q_offsets, R, spec_ids, spec_scores);
    return hipGetLastError();
}

hipError_t launch_verify(const int32_t *spec, const int32_t *truth, int64_t true_stride, int64_t Qt,
                         const int64_t *q_offsets, int64_t R, int32_t *first_mismatch, hipStream_t stream)
{
    if (R <= 0) return hipSuccess;
    hipLaunchKernelGGL(verify_kernel, dim3((unsigned)((R + 3) / 4)), dim3(256), 0, stream, spec, truth,
                       true_stride, Qt, q_offsets, R, first_mismatch);
    return hipGetLastError();
}

hipError_t launch_cache_insert(int32_t *cache_ids, int32_t *cache_len, int32_t *cache_head, int32_t C, int64_t R,
                               const int32_t *truth, int64_t true_stride, int64_t Qt, const int64_t *q_offsets,
                               const int32_t *first_mismatch, int32_t p, int32_t n_next, int64_t N,
                               hipStream_t stream)
{
    if (R <= 0) return hipSuccess;
    const size_t smem = (size_t)((C + 255) & ~255) * sizeof(int32_t);
    static std::atomic<bool> attr_done{false};   // per instantiation; setting it twice is harmless
    if (!attr_done.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(cache_insert_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, CACHE_INSERT_MAX_C * 4);
        if (e != hipSuccess) return e;
        attr_done.store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL(cache_insert_kernel, dim3((unsigned)R), dim3(64), smem, stream, cache_ids, cache_len,
                       cache_head, C, truth, true_stride, Qt, q_offsets, first_mismatch, p, n_next, N);
    return hipGetLastError();
}

hipError_t launch_cache_keys(const int32_t *cache_ids, const int32_t *cache_len, int32_t C, int64_t R, int64_t Qt,
                             const int64_t *q_offsets, int64_t N, u64 *keys, uint32_t *cnt, hipStream_t stream)
{
    hipError_t e = launch_fill_u32(cnt, 0u, Qt, stream);
    if (e != hipSuccess || R <= 0) return e;
    hipLaunchKernelGGL(cache_keys_kernel, dim3((unsigned)R), dim3(256), 0, stream, cache_ids, cache_len, C, Qt,
                       q_offsets, N, keys, cnt);
    return hipGetLastError();
}

hipError_t launch_fill_u32(uint32_t *p, uint32_t v, int64_t n, hipStream_t stream)
{
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(fill_u32_kernel, dim3(grid_for(n, 256)), dim3(256), 0, stream, p, v, n);
    return hipGetLastError();
}
hipError_t launch_fill_u64(u64 *p, u64 v, int64_t n, hipStream_t stream)
{
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(fill_u64_kernel, dim3(grid_for(n, 256)), dim3(256), 0, stream, p, v, n);
    return hipGetLastError();
}

hipError_t launch_l2_scan_copy(const void *src, int32_t src_dtype, int64_t src_ld, void *dst, int32_t dst_dtype,
                               int64_t dst_ld, int64_t N, int32_t d, hipStream_t stream)
{
    if (N <= 0) return hipSuccess;
    const int in_place = src == dst ? 1 : 0;
    const int64_t blocks = (N + 3) / 4;
    const dim3 grid((unsigned)(blocks < (1 << 20) ? blocks : (1 << 20))), block(256);
    uint16_t *out = static_cast<uint16_t *>(dst);
    if (src_dtype == DT_F16) {
        if (dst_dtype == DT_F16)
            hipLaunchKernelGGL((l2_scan_copy_kernel<DT_F16, DT_F16>), grid, block, 0, stream, src, src_ld, out, dst_ld, N, d, in_place);
        else
            hipLaunchKernelGGL((l2_scan_copy_kernel<DT_F16, DT_BF16>), grid, block, 0, stream, src, src_ld, out, dst_ld, N, d, in_place);
    } else {
        if (dst_dtype == DT_F16)
            hipLaunchKernelGGL((l2_scan_copy_kernel<DT_F32, DT_F16>), grid, block, 0, stream, src, src_ld, out, dst_ld, N, d, in_place);
        else
            hipLaunchKernelGGL((l2_scan_copy_kernel<DT_F32, DT_BF16>), grid, block, 0, stream, src, src_ld, out, dst_ld, N, d, in_place);
    }
    return hipGetLastError();
}

hipError_t launch_query_prep(const float *q, int64_t Q, int32_t d, uint16_t *out, int64_t Qpad, int32_t dpad,
                             int32_t scan_dtype, int32_t metric, uint32_t *z0, int64_t n0, uint32_t *z1, int64_t n1,
                             hipStream_t stream)
{
    const int64_t n = Qpad * dpad;
    if (n <= 0) return hipSuccess;
    const dim3 grid(grid_for(n, 256)), block(256);
    if (scan_dtype == DT_F16) {
        if (metric == METRIC_L2)
            hipLaunchKernelGGL((query_prep_kernel<DT_F16, true>), grid, block, 0, stream, q, Q, d, out, Qpad, dpad, z0, n0, z1, n1);
        else
            hipLaunchKernelGGL((query_prep_kernel<DT_F16, false>), grid, block, 0, stream, q, Q, d, out, Qpad, dpad, z0, n0, z1, n1);
    } else {
        if (metric == METRIC_L2)
            hipLaunchKernelGGL((query_prep_kernel<DT_BF16, true>), grid, block, 0, stream, q, Q, d, out, Qpad, dpad, z0, n0, z1, n1);
        else
            hipLaunchKernelGGL((query_prep_kernel<DT_BF16, false>), grid, block, 0, stream, q, Q, d, out, Qpad, dpad, z0, n0, z1, n1);
    }
    return hipGetLastError();
}

hipError_t launch_convert_rows(const float *src, int64_t src_ld, void *dst, int32_t dst_dtype, int64_t dst_ld,
                               int64_t N, int32_t d, hipStream_t stream)
{
    const int64_t n = N * (d / 8);
    if (n <= 0) return hipSuccess;
    if (dst_dtype == DT_F16)
        hipLaunchKernelGGL(convert_rows_kernel<DT_F16>, dim3(grid_for(n, 256)), dim3(256), 0, stream, src,
                           src_ld, static_cast<uint16_t *>(dst), dst_ld, N, d / 8);
    else
        hipLaunchKernelGGL(convert_rows_kernel<DT_BF16>, dim3(grid_for(n, 256)), dim3(256), 0, stream, src,
                           src_ld, static_cast<uint16_t *>(dst), dst_ld, N, d / 8);
    return hipGetLastError();
}

}  // namespace ralm
