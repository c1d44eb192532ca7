// Fused scoring + threshold selection scan over the datastore (gfx950).
//
// This is the knowledge-base retrieval C.retrieve(q_1..q_s) of Alg. 1 (the batched
// verification step) for the exact dense retriever of Section 5.1: every datastore row is
// scored against every query of the batch by inner product.  The [N, Q] score matrix is
// never written: scores come out of the matrix cores (bf16 or fp16 inputs, fp32
// accumulation) and each one is compared at once with its query's admission key; the few
// that pass are appended to that query's candidate list.
//
// Tiling: a workgroup of 4 waves owns a 256-row x BN-query tile; the reduction dimension is
// walked in steps of 64 elements staged through LDS (double buffered, global loads for step
// t+1 in flight while step t is multiplied).  Datastore rows are the A operand of
// v_mfma_f32_32x32x16, queries the B operand, so every accumulator register of a lane
// belongs to ONE query (column = lane % 32) and the lane can hold that query's threshold in
// a register.
//
// Work items (row tile, query tile) are dealt to a persistent grid so that workgroups that
// run at the same time on one XCD (workgroup b lands on XCD b % 8) hold consecutive items:
// all query tiles of a row tile, then the next row tile.  The row tile's second to last
// readers therefore hit that XCD's L2.
#include "ralm_common.h"
#include "ralm_kernels.h"

namespace ralm {

namespace {

template <int IN>
struct RawChunk {
    uint4 v;
};
template <>
struct RawChunk<DT_F32> {
    float4 lo, hi;
};

template <int IN>
__device__ __forceinline__ void load_chunk(RawChunk<IN> &r, const void *X, int64_t elem_off, bool ok)
{
    if constexpr (IN == DT_F32) {
        if (ok) {
            const float4 *p = reinterpret_cast<const float4 *>(static_cast<const float *>(X) + elem_off);
            r.lo = p[0];
            r.hi = p[1];
        } else {
            r.lo = make_float4(0.f, 0.f, 0.f, 0.f);
            r.hi = r.lo;
        }
    } else {
        if (ok)
            r.v = *reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(X) + elem_off);
        else
            r.v = make_uint4(0u, 0u, 0u, 0u);
    }
}

template <int IN>
__device__ __forceinline__ uint4 chunk_bits(const RawChunk<IN> &r)
{
    if constexpr (IN == DT_F32)
        return pack8<DT_BF16>(r.lo, r.hi);
    else
        return r.v;
}

template <bool F16>
__device__ __forceinline__ f32x16 mfma32(const uint4 &a, const uint4 &b, const f32x16 &c)
{
    if constexpr (F16)
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a),
                                                      __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                       __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// IN: dtype of the datastore copy being scanned.  WM x WN waves, each TM x TN MFMA blocks.
template <int IN, int WM, int WN, int TM, int TN>
__global__ __launch_bounds__(256) void scan_kernel(const ScanParams p, const int nqt)
{
    constexpr int BM = WM * TM * 32, BN = WN * TN * 32, BK = SCAN_BK, LDA = BK + 8;
    constexpr int PA = BM / 32, PB = BN / 32;
    constexpr bool F16 = (IN == DT_F16);
    static_assert(WM * WN == 4 && BM == SCAN_BM, "4 waves, 256-row tiles");

    extern __shared__ __align__(16) unsigned char smem[];
    uint16_t *As = reinterpret_cast<uint16_t *>(smem);      // [2][BM][LDA]
    uint16_t *Bs = As + 2 * BM * LDA;                        // [2][BN][LDA]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int ld_c = tid & 7, ld_r = tid >> 3;   // staging: 8 lanes cover 64 elements of a row
    const int fr = lane & 31, fk = (lane >> 5) * 8;

    const int64_t G = gridDim.x;
    const int64_t vb = (int64_t)(blockIdx.x % 8) * (G / 8) + blockIdx.x / 8;
    const int64_t total = p.n_row_tiles * nqt;
    const int KT = p.dpad / BK;

    for (int64_t item = vb; item < total; item += G) {
        const int64_t rt = item / nqt;
        const int qt = (int)(item % nqt);
        const int64_t row0 = rt * p.tile_stride * BM;
        const int q0 = qt * BN;

        f32x16 acc[TM][TN];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

        RawChunk<IN> ra[PA];
        uint4 rb[PB];

        auto load_stage = [&](int kt) {
            const int kc = kt * BK + ld_c * 8;
            const bool kok = kc < p.d;
#pragma unroll
            for (int pa = 0; pa < PA; ++pa) {
                const int64_t g = row0 + pa * 32 + ld_r;
                load_chunk<IN>(ra[pa], p.X, g * p.ldx + kc, kok && g < p.N);
            }
#pragma unroll
            for (int pb = 0; pb < PB; ++pb) {
                const int64_t qrow = q0 + pb * 32 + ld_r;
                rb[pb] = *reinterpret_cast<const uint4 *>(p.Qs + qrow * p.dpad + kc);
            }
        };
        auto store_stage = [&](int buf) {
            uint16_t *a = As + buf * BM * LDA;
            uint16_t *b = Bs + buf * BN * LDA;
#pragma unroll
            for (int pa = 0; pa < PA; ++pa)
                *reinterpret_cast<uint4 *>(a + (pa * 32 + ld_r) * LDA + ld_c * 8) = chunk_bits<IN>(ra[pa]);
#pragma unroll
            for (int pb = 0; pb < PB; ++pb)
                *reinterpret_cast<uint4 *>(b + (pb * 32 + ld_r) * LDA + ld_c * 8) = rb[pb];
        };

        load_stage(0);
        store_stage(0);
        __syncthreads();

        for (int kt = 0; kt < KT; ++kt) {
            const int buf = kt & 1;
            if (kt + 1 < KT) load_stage(kt + 1);
            const uint16_t *a = As + buf * BM * LDA + (wm * TM * 32 + fr) * LDA + fk;
            const uint16_t *b = Bs + buf * BN * LDA + (wn * TN * 32 + fr) * LDA + fk;
#pragma unroll
            for (int kk = 0; kk < BK / 16; ++kk) {
                uint4 fa[TM], fb[TN];
#pragma unroll
                for (int i = 0; i < TM; ++i)
                    fa[i] = *reinterpret_cast<const uint4 *>(a + i * 32 * LDA + kk * 16);
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    fb[j] = *reinterpret_cast<const uint4 *>(b + j * 32 * LDA + kk * 16);
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) acc[i][j] = mfma32<F16>(fa[i], fb[j], acc[i][j]);
            }
            if (kt + 1 < KT) store_stage(buf ^ 1);
            __syncthreads();
        }

        // ---- selection epilogue: one query per lane and MFMA block column ----
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int q = q0 + (wn * TN + j) * 32 + fr;
            const bool qok = q < p.Q;
            const u64 tkey = qok ? p.tau[q] : ~0ull;
            const float tsc = qok ? key_score(tkey) : __builtin_inff();
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                float m = acc[i][j][0];
#pragma unroll
                for (int v = 1; v < 16; ++v) m = fmaxf(m, acc[i][j][v]);
                // tkey == 0 admits everything (its score bits decode to NaN: compare separately)
                if (qok && (tkey == 0ull || m >= tsc)) {
                    const int64_t rbase = row0 + (wm * TM + i) * 32 + (lane >> 5) * 4;
                    uint32_t pass = 0;
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int64_t g = rbase + (v >> 2) * 8 + (v & 3);
                        if (g < p.N && make_key(acc[i][j][v], (int32_t)g) >= tkey) pass |= 1u << v;
                    }
                    if (pass) {
                        const uint32_t n = __popc(pass);
                        uint32_t at = atomicAdd(p.cnt + q, n);
                        u64 *dst = p.cand + (int64_t)q * p.cap;
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            if (pass & (1u << v)) {
                                const int64_t g = rbase + (v >> 2) * 8 + (v & 3);
                                if (at < p.cap) dst[at] = make_key(acc[i][j][v], (int32_t)g);
                                ++at;
                            }
                        }
                    }
                }
            }
        }
    }
}

template <int IN, int WM, int WN, int TM, int TN>
hipError_t launch_variant(const ScanParams &p, int n_cu, hipStream_t stream)
{
    constexpr int BM = WM * TM * 32, BN = WN * TN * 32, LDA = SCAN_BK + 8;
    constexpr size_t smem = (size_t)2 * (BM + BN) * LDA * sizeof(uint16_t);
    auto kern = scan_kernel<IN, WM, WN, TM, TN>;
    static bool attr_done = false;   // per instantiation
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    const int nqt = (int)((p.Q + BN - 1) / BN);
    const int64_t total = p.n_row_tiles * nqt;
    if (total <= 0) return hipSuccess;
    const int per_cu = smem * 2 <= 160 * 1024 ? 2 : 1;
    int64_t grid = (int64_t)n_cu * per_cu;
    if (total < grid) grid = total;
    grid = (grid + 7) / 8 * 8;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(256), smem, stream, p, nqt);
    return hipGetLastError();
}

template <int IN>
hipError_t launch_in(const ScanParams &p, int n_cu, hipStream_t stream)
{
    const int bn = scan_bn_for(p.Q);
    switch (bn) {
        case 32: return launch_variant<IN, 4, 1, 2, 1>(p, n_cu, stream);
        case 64: return launch_variant<IN, 4, 1, 2, 2>(p, n_cu, stream);
        case 128: return launch_variant<IN, 2, 2, 4, 2>(p, n_cu, stream);
        default: return launch_variant<IN, 2, 2, 4, 4>(p, n_cu, stream);
    }
}

}  // namespace

int scan_bn_for(int64_t Q)
{
    if (Q <= 32) return 32;
    if (Q <= 64) return 64;
    if (Q <= 128) return 128;
    return 256;
}

hipError_t launch_scan(const ScanParams &p, int n_cu, hipStream_t stream)
{
    switch (p.in_dtype) {
        case DT_F32: return launch_in<DT_F32>(p, n_cu, stream);
        case DT_F16: return launch_in<DT_F16>(p, n_cu, stream);
        default: return launch_in<DT_BF16>(p, n_cu, stream);
    }
}

}  // namespace ralm
