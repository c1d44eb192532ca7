// Fused scoring + threshold selection scan over the datastore (gfx950).
//
// This is the knowledge-base retrieval C.retrieve(q_1..q_s) of Alg. 1 (the batched
// verification step) for the exact dense retriever of Section 5.1: every datastore row is
// scored against every query of the batch by inner product.  The [N, Q] score matrix is
// never written: scores come out of the matrix cores (bf16 or fp16 inputs, fp32
// accumulation) and each one is compared at once with its query's admission key; the few
// that pass are appended to that query's candidate list.
//
// Tiling: a workgroup of 4 or 8 waves owns a 256-row x BN-query tile (BN = 32 on 4 waves; 64,
// 128 and 256 on 8 waves, two per SIMD); the reduction dimension is walked in strips of BK
// elements.  Datastore rows are the A operand of v_mfma_f32_32x32x16, queries the B operand, so
// every accumulator register of a lane belongs to ONE query (column = lane % 32) and the lane
// can hold that query's threshold in a register.
//
// Two kernels share that tiling and the epilogue:
//   scan_dma_kernel     bf16 / fp16 datastore copies, and fp32 rows as they are (rounded to
//                       bf16 between the operand read and the multiply).  Strips go from global memory straight
//                       into LDS (global_load_lds_dwordx4, no VGPR staging) through a ring of
//                       S stages that runs ahead of the multiply and keeps running across tile
//                       boundaries; the 16-byte chunks of a row are XOR-swizzled on the way in
//                       (by choosing which global chunk each lane fetches) so that the MFMA
//                       operand reads (32 rows, same chunk) are free of bank conflicts.
//   scan_staged_kernel  global -> registers -> LDS, double buffered: launches that keep every
//                       score: the first, small stage of a ladder with a partial last tile,
//                       and the blocks of the sequential ladder.  Otherwise
//                       the first stage runs in scan_dma_kernel<.., ALL>, which writes each
//                       score to the list slot that its row's place in the launch determines.
//
// Work items (row tile, query tile) are dealt to a persistent grid so that workgroups that
// run at the same time on one XCD (workgroup b lands on XCD b % 8) hold consecutive items:
// all query tiles of a row tile, then the next row tile.  The row tile's second to last
// readers therefore hit that XCD's L2.
#include <type_traits>

#include <atomic>

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

#define RALM_LDS __attribute__((address_space(3)))

// datastore tile of the t-th tile a launch visits (see ScanParams)
__device__ __forceinline__ int64_t visited_tile(const ScanParams &p, int64_t t)
{
    if (p.tile_skip) {
        // tile counts fit 32 bits (N < 2^31 rows): a 32-bit division, not an emulated 64-bit one
        const uint32_t g1 = (uint32_t)p.tile_skip - 1u, t32 = (uint32_t)t;
        const uint32_t q = t32 / g1;
        t = (int64_t)q * p.tile_skip + (t32 - q * g1) + 1;
    }
    return (p.tile_begin + t) * p.tile_stride;
}

// acc[i][j][v] of a wave is the score of datastore row
//     row0 + (wm*TM + i)*32 + (v/4)*8 + (lane/32)*4 + v%4
// against query  q0 + (wn*TN + j)*32 + lane%32.  A score is admitted (appended to its query's
// candidate list) iff its ranking key is >= the query's admission key.

// Direct epilogue (staged kernel): admitted scores go straight to the global candidate lists,
// one atomic per lane and 32x32 block.
template <int WM, int WN, int TM, int TN>
__device__ __forceinline__ void select_epilogue_direct(const ScanParams &p, f32x16 (&acc)[TM][TN], int32_t row0,
                                                       int q0, int wm, int wn, int lane)
{
    const int fr = lane & 31;
    const int32_t n_rows = (int32_t)p.N;
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
                const int32_t rbase = row0 + (wm * TM + i) * 32 + (lane >> 5) * 4;
                uint32_t pass = 0;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int32_t g = rbase + (v >> 2) * 8 + (v & 3);
                    if (g < n_rows && make_key(acc[i][j][v], g) >= tkey) pass |= 1u << v;
                }
                if (pass) {
                    uint32_t at = atomicAdd(p.cnt + q, (uint32_t)__popc(pass));
                    u64 *dst = p.cand + (int64_t)q * p.cap;
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        if (pass & (1u << v)) {
                            if (at < p.cap) dst[at] = make_key(acc[i][j][v], rbase + (v >> 2) * 8 + (v & 3));
                            ++at;
                        }
                    }
                }
            }
        }
    }
}

// Parked epilogue (pipelined kernel).  Admitted scores are first parked in a small LDS list
// (an LDS atomic is ~20x quicker than a global atomic round trip, which a lone wave per SIMD
// cannot hide) and moved to the global lists in batches by flush_parked().  An entry that
// finds the list full goes to its global list directly, so nothing is ever lost.
struct PushList {
    RALM_LDS uint32_t *count;   // entries appended so far (may exceed cap; the excess went to global)
    RALM_LDS u64 *keys;         // [cap]
    RALM_LDS uint32_t *qs;      // [cap]
    uint32_t cap;
};

__device__ __forceinline__ void push_global(const ScanParams &p, int q, u64 key)
{
    const uint32_t at = atomicAdd(p.cnt + q, 1u);
    if (at < p.cap) p.cand[(int64_t)q * p.cap + at] = key;
}

// all threads of the workgroup, after a barrier that follows the last append: moves the first n parked
// entries to the global lists and empties the LDS list
__device__ __forceinline__ void flush_parked(const ScanParams &p, const PushList pl, uint32_t n)
{
    for (uint32_t e = threadIdx.x; e < n; e += blockDim.x) push_global(p, (int)pl.qs[e], pl.keys[e]);
    __syncthreads();
    if (threadIdx.x == 0) *pl.count = 0;
    __syncthreads();
}

// one 32x32 block of one wave: out[v] for row rbase + (v/4)*8 + v%4 and query q.
//
// The common case (no lane of the wave holds an admitted score) must be a handful of
// instructions: the pipelined kernel's last stage contains 16 copies of this function, and
// anything bulky here pushes that stage out of the instruction cache.  So the rare case does
// not unroll over the 16 values: a lane that may hold an admitted score writes its 16 values
// to a 64-byte LDS slot and walks them in a rolled loop (registers cannot be indexed
// dynamically, LDS can).  Slots are handed out by rank among the candidate lanes, 8 per round.
constexpr int SLOW_SLOTS = 8;   // 64-byte slots per wave
__device__ __forceinline__ void select_block_parked(const ScanParams &p, const PushList pl,
                                                    RALM_LDS float *wave_slots, const f32x16 &out,
                                                    int32_t rbase, int32_t n_rows, int q, bool qok, u64 tkey,
                                                    float tsc)
{
    float m = out[0];
#pragma unroll
    for (int v = 1; v < 16; ++v) m = fmaxf(m, out[v]);
    // tsc is -inf where the key admits everything and +inf for padding columns: one compare
    bool cand = m >= tsc;
    unsigned long long mask = __builtin_amdgcn_ballot_w64(cand);
    while (mask) {   // wave-uniform
        const uint32_t rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                                        __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
        const bool mine = cand && rank < (uint32_t)SLOW_SLOTS;
        if (mine) {
            RALM_LDS float *slot = wave_slots + rank * 16;
            typedef float f32x4v __attribute__((ext_vector_type(4)));
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                f32x4v t = {out[c * 4], out[c * 4 + 1], out[c * 4 + 2], out[c * 4 + 3]};
                *(RALM_LDS f32x4v *)(slot + c * 4) = t;
            }
            // which of the 16 values reach the threshold score (cheap, in registers) ...
            uint32_t pm = 0;
#pragma unroll
            for (int v = 0; v < 16; ++v) pm |= out[v] >= tsc ? (1u << v) : 0u;
            // ... and only those are fetched back and tested exactly (usually one or two)
#pragma unroll 1
            while (pm) {
                const int v = __builtin_ctz(pm);
                pm &= pm - 1;
                const int32_t g = rbase + (v >> 2) * 8 + (v & 3);
                const u64 key = make_key(slot[v], g);
                if (g < n_rows && key >= tkey) {
                    const uint32_t at =
                        __hip_atomic_fetch_add(pl.count, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                    if (at < pl.cap) {
                        pl.keys[at] = key;
                        pl.qs[at] = (uint32_t)q;
                    } else {
                        push_global(p, q, key);
                    }
                }
            }
        }
        cand = cand && !mine;
        mask = __builtin_amdgcn_ballot_w64(cand);
    }
}

// Epilogue of a launch that keeps every score into empty lists (the first stage of a ladder): the
// score of the launch's r-th row goes to slot r of its query's list, no atomics.  A lane's 16
// values are 4 runs of 4 consecutive rows: 8 stores of two keys each.
__device__ __forceinline__ void store_block_all(const ScanParams &p, const f32x16 &out, int32_t row_id0, int64_t pos0,
                                                int q, bool qok)
{
    if (!qok) return;
    u64 *dst = p.cand + (int64_t)q * p.cap + pos0;
    typedef unsigned long long u64x2 __attribute__((ext_vector_type(2)));
#pragma unroll
    for (int c = 0; c < 4; ++c) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int v = c * 4 + h * 2;
            const u64x2 two = {make_key(out[v], row_id0 + c * 8 + h * 2), make_key(out[v + 1], row_id0 + c * 8 + h * 2 + 1)};
            *reinterpret_cast<u64x2 *>(dst + c * 8 + h * 2) = two;
        }
    }
}

// IN: dtype of the datastore copy being scanned.  WM x WN waves, each TM x TN MFMA blocks.
template <int IN, int WM, int WN, int TM, int TN>
__global__ __launch_bounds__(256) void scan_staged_kernel(const ScanParams p, const int nqt)
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
        const int64_t row0 = visited_tile(p, rt) * BM;
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

        select_epilogue_direct<WM, WN, TM, TN>(p, acc, (int32_t)row0, q0, wm, wn, lane);
    }
}


// ---- direct-to-LDS pipelined kernel ----------------------------------------------------------
// LDS chunk swizzle: row r of a strip stores its global 16-byte chunk c at chunk slot c ^ swz(r).
// Chosen so that 8 or 16 consecutive rows reading the same global chunk touch distinct
// 16-byte bank groups, for both 128 B and 256 B of LDS banking.
// CPR = 16-byte chunks per strip row: 4 (64-byte rows), 8 (128-byte rows) or 16 (256-byte rows).
template <int CPR>
__device__ __forceinline__ int swz(int r)
{
    static_assert(CPR == 4 || CPR == 8 || CPR == 16, "strip row of 64, 128 or 256 bytes");
    if constexpr (CPR == 16)
        return r & 15;
    else if constexpr (CPR == 8)
        return (r ^ (r >> 3)) & 7;
    else
        return ((r >> 2) & 1) | ((((r >> 1) ^ (r >> 3)) & 1) << 1);
}

// eight fp32 values (two 16-byte chunks) -> eight bf16, round to nearest even, as an MFMA operand
__device__ __forceinline__ uint4 round8_bf16(const uint4 &lo, const uint4 &hi)
{
    typedef float f32x8 __attribute__((ext_vector_type(8)));
    const f32x8 f = {__uint_as_float(lo.x), __uint_as_float(lo.y), __uint_as_float(lo.z), __uint_as_float(lo.w),
                     __uint_as_float(hi.x), __uint_as_float(hi.y), __uint_as_float(hi.z), __uint_as_float(hi.w)};
    return __builtin_bit_cast(uint4, __builtin_convertvector(f, bf16x8));
}

// 64 lanes x 16 bytes, from  base + per-lane byte offset,  to 1 KB of LDS starting at lds_base
// (base and lds_base are wave-uniform).  Written as inline asm so that the compiler does not
// track it: completion is awaited by hand with s_waitcnt vmcnt(n) (loads complete in order).
//
// NT: the load is marked non-temporal.  Datastore rows that no other workgroup will read (the
// batch fits one query tile) are streamed that way: they do not displace the query tile in L2,
// and a pure read stream reaches a higher HBM rate with it.  Rows that several query tiles share
// through L2, and the queries themselves, are loaded with the default policy.
template <bool NT>
__device__ __forceinline__ void dma_1kb(const unsigned char *base, uint32_t voff, uint32_t lds_base)
{
    if constexpr (NT)
        asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2 nt" ::"s"(lds_base), "v"(voff), "s"(base)
                     : "memory");
    else
        asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_base), "v"(voff), "s"(base)
                     : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

constexpr int TAU_LDS_MAX_Q = 2560;   // admission keys of up to this many queries are kept in LDS
// ... by the widest query tile; the narrower tiles serve only batches of at most one tile
constexpr int tau_lds_q(int BN) { return BN <= 128 ? BN : TAU_LDS_MAX_Q; }
constexpr int PARK_CAP = 672;         // parked admitted scores per workgroup (12 bytes each)

#define RALM_SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)

// The instruction stream of a stage is laid out by hand (one wave per SIMD: nothing else fills
// the issue slots between MFMAs).  After each MFMA exactly one "side" instruction follows: an
// LDS operand read for the next k-step, or one 1 KB global->LDS load of the strip that is S-1
// stages ahead.  sched_barrier keeps the compiler from regrouping them.  In a tile's last
// k-step the MFMA results are written to VGPRs and each block's selection test runs two MFMAs
// behind its last multiply, so the selection costs no separate pass over the accumulators.
//
// The ring has S slots and the issue cursor runs D stages ahead of the multiply.  D = S - 1 (the
// loads issued during stage t refill the slot of stage t - 1) or D = S (they refill the slot of
// stage t itself, once every wave has read the operands of the stage's last k-step out of it: a
// ring of two 64-element strips then does the work of four 32-element strips, with half the
// rendezvous per multiply and whole 128-byte lines per request).  The rendezvous of a stage
// sits in k-step RK, behind that k-step's operand reads; the query part of the new strip is
// requested after it in the same k-step, the datastore part in the next k-step.  RK = KS - 2 is
// the k-step whose reads are the stage's last, which D = S needs.
//
// A32: the datastore rows are fp32 (a datastore scanned as it is).  They travel to LDS as they
// are, twice the bytes per strip row, and are rounded to bf16 between the operand read and the
// multiply (two 16-byte reads and four conversions per operand instead of one read).
// ALL: a launch into empty lists that keeps every score (see store_block_all); no thresholds.
template <bool F16, int WM, int WN, int TM, int TN, int BK, int S, bool NTA, int D = S - 1, int RK = 0,
          bool A32 = false, bool ALL = false>
__global__ __launch_bounds__(WM *WN * 64) void scan_dma_kernel(const ScanParams p, const int nqt, const int tau_in_lds)
{
    constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
    constexpr int ESA = A32 ? 4 : 2;                       // bytes of a datastore element
    constexpr int ROWB_A = BK * ESA, ROWB_B = BK * 2;      // bytes of one strip row (datastore, queries)
    constexpr int CPR_A = ROWB_A / 16, CPR_B = ROWB_B / 16;   // 16-byte chunks per strip row
    constexpr int RPI_A = 64 / CPR_A, RPI_B = 64 / CPR_B;  // rows covered by one wave load
    constexpr int NW = WM * WN, NT = NW * 64;     // waves (4: one per SIMD, 8: two per SIMD), threads
    constexpr int NA = BM / RPI_A / NW, NB = BN / RPI_B / NW;   // wave loads per wave and stage
    constexpr int LPS = NA + NB;
    constexpr int A_BYTES = BM * ROWB_A, B_BYTES = BN * ROWB_B, STAGE = A_BYTES + B_BYTES;
    static_assert(!(A32 && F16), "fp32 rows are rounded to bf16");
    constexpr int KS = BK / 16;
    constexpr int NM = TM * TN, NR = TM + TN;
    constexpr int LAG = NM > 2 ? 2 : NM - 1;     // selection runs this many MFMAs behind
    constexpr int RV = NR - 1;                   // slot of k-step RK after which the stage rendezvous sits
    // a workgroup tile covers the whole 256-row tile of the ladder, or half of it
    constexpr int PARTS = SCAN_BM / BM;
    static_assert((NW == 4 || NW == 8) && (BM == SCAN_BM || BM * 2 == SCAN_BM) && NA >= 1 && NB >= 1, "tile shape");
    static_assert(S >= 2 && (D == S - 1 || D == S) && D >= 2 && KS % 2 == 0, "ring depth / k-steps per stage");
    static_assert(RK >= 0 && RK + 1 < KS && (D < S || RK == KS - 2), "rendezvous position");
    static_assert(LPS * (D - 1) < 64, "vmcnt range");

    extern __shared__ __align__(16) unsigned char smem[];
    const uint32_t lds0 = (uint32_t)(size_t)(RALM_LDS unsigned char *)smem;
    RALM_LDS u64 *tau_lds = (RALM_LDS u64 *)(smem + S * STAGE);
    PushList pl;
    pl.keys = tau_lds + tau_lds_q(BN);
    pl.qs = (RALM_LDS uint32_t *)(pl.keys + PARK_CAP);
    pl.count = pl.qs + PARK_CAP;
    pl.cap = PARK_CAP;
    RALM_LDS float *wave_slots = (RALM_LDS float *)(pl.count + 4) + (threadIdx.x >> 6) * (SLOW_SLOTS * 16);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int fr = lane & 31;
    const int la_r = lane / CPR_A, la_c = lane % CPR_A;   // row and chunk of this lane in a wave load
    const int lb_r = lane / CPR_B, lb_c = lane % CPR_B;

    // item indices fit 32 bits: at most 2^23 row tiles times a few query tiles (host checks)
    const int G = (int)gridDim.x;
    const int vb = (int)(blockIdx.x % 8) * (G / 8) + (int)(blockIdx.x / 8);
    const int n_tiles = (int)p.n_row_tiles * PARTS;      // workgroup tiles of this launch
    const int total = n_tiles * nqt;
    // first datastore row of the rt-th workgroup tile
    auto tile_row0 = [&](int rt) __attribute__((always_inline)) -> int64_t {
        if constexpr (PARTS == 1) return visited_tile(p, rt) * SCAN_BM;
        else return visited_tile(p, rt / PARTS) * SCAN_BM + (rt % PARTS) * BM;
    };
    const int KT = p.dpad / BK;
    const int n_mine = vb < total ? (total - vb + G - 1) / G : 0;
    if constexpr (ALL) {
        // every list ends up with one entry per row of the launch (all of its tiles are full: host check)
        if (blockIdx.x == 0)
            for (int q = tid; q < p.Q; q += NT) p.cnt[q] = (uint32_t)n_tiles * BM;
    }
    if (n_mine == 0) return;
    const unsigned char *Xb = static_cast<const unsigned char *>(p.X);
    const unsigned char *Qb = reinterpret_cast<const unsigned char *>(p.Qs);
    const uint32_t ldx2 = (uint32_t)p.ldx * (uint32_t)ESA, dpad2 = (uint32_t)p.dpad * 2u;   // row pitches in bytes
    const int32_t n_rows = (int32_t)p.N;

    if (tid == 0) *pl.count = 0;
    if (tau_in_lds)
        for (int q = tid; q < p.Q; q += NT) tau_lds[q] = p.tau[q];

    // ---- issue cursor: runs S-1 stages ahead of the multiply, also across tile boundaries ----
    // per-lane constants of the loads: byte offset (tile row, swizzled chunk) of each wave load
    // inside a strip that lies fully inside the datastore; strips at its edges are clamped instead
    uint32_t a_voff[NA], b_voff[NB];
    auto a_tile_row = [&](int j) __attribute__((always_inline)) { return (uint32_t)((wave * NA + j) * RPI_A + la_r); };
    auto a_tile_chunk = [&](int j) __attribute__((always_inline)) {
        return (uint32_t)((la_c ^ swz<CPR_A>((int)a_tile_row(j) & 15)) << 4);
    };
#pragma unroll
    for (int j = 0; j < NA; ++j) a_voff[j] = __umul24(a_tile_row(j), ldx2) + a_tile_chunk(j);   // row < 2^8, ldx2 < 2^24
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        const int row = (wave * NB + j) * RPI_B + lb_r;
        b_voff[j] = (uint32_t)row * dpad2 + (uint32_t)((lb_c ^ swz<CPR_B>(row & 15)) << 4);
    }
    // (row tile, query tile) of an item advance by (G / nqt, G % nqt) from one item of this
    // workgroup to its next: no division in the loop
    const int step_rt = G / nqt;
    const int step_qt = G % nqt;
    int is_rt = vb / nqt;
    int is_qt = vb % nqt;
    int is_kt = 0, is_buf = 0;
    // wave-uniform state of the stage being issued
    const unsigned char *is_abase = nullptr, *is_bbase = nullptr, *is_aload = nullptr;
    uint32_t is_rowmax = 0, is_kmax = 0, is_lds = 0;
    bool is_inside = false;   // the strip needs no clamping
    auto issue_begin = [&]() __attribute__((always_inline)) {
        if (is_kt == 0) {
            // The cursor is never stopped: past this workgroup's last tile it fetches (valid)
            // strips that nobody multiplies, so the steady-state loop has no conditionals.
            const int rt = is_rt < n_tiles ? is_rt : 0;
            int64_t row0 = tile_row0(rt);
            int64_t left = p.N - 1 - row0;                  // rows past N re-read row N-1 ...
            if (left < 0) {                                 // ... also a half tile that starts past it
                row0 = p.N - 1;
                left = 0;
            }
            is_abase = Xb + row0 * p.ldx * ESA;
            is_bbase = Qb + (int64_t)is_qt * BN * p.dpad * 2;
            is_rowmax = (uint32_t)(left < BM - 1 ? left : BM - 1);
        }
        // chunks past d re-read the row's last valid one (the query side is zero there): inside a
        // strip by clamping the chunk offset, for a strip that lies past d entirely by stepping
        // the strip's base back to that chunk
        const int kleft = (p.d - 16 / ESA - is_kt * BK) * ESA;   // the row's last chunk, from the strip's start
        is_kmax = (uint32_t)(kleft < 0 ? 0 : (kleft < ROWB_A - 16 ? kleft : ROWB_A - 16));
        is_aload = is_abase + (kleft < 0 ? kleft : 0);
        is_inside = is_rowmax == (uint32_t)(BM - 1) && kleft >= ROWB_A - 16;
        is_lds = lds0 + is_buf * STAGE + wave * (NA * 1024);
    };
    auto issue_part = [&](int idx) __attribute__((always_inline)) {
        if (idx < NA) {
            uint32_t voff = a_voff[idx];
            if (!is_inside) {   // wave-uniform, rare: the datastore's last rows or last columns
                const uint32_t row = a_tile_row(idx), chunk = a_tile_chunk(idx);
                const uint32_t r = row < is_rowmax ? row : is_rowmax;
                const uint32_t c = chunk < is_kmax ? chunk : is_kmax;
                voff = __umul24(r, ldx2) + c;
            }
            dma_1kb<NTA>(is_aload, voff, is_lds + idx * 1024);
        } else {
            const int j = idx - NA;
            dma_1kb<false>(is_bbase, b_voff[j], lds0 + is_buf * STAGE + A_BYTES + (wave * NB + j) * 1024);
        }
    };
    auto issue_end = [&]() __attribute__((always_inline)) {
        is_abase += ROWB_A;
        is_bbase += ROWB_B;
        is_buf = is_buf + 1 == S ? 0 : is_buf + 1;
        if (++is_kt == KT) {
            is_kt = 0;
            is_rt += step_rt;
            is_qt += step_qt;
            if (is_qt >= nqt) {
                is_qt -= nqt;
                ++is_rt;
            }
        }
    };

    for (int st = 0; st < D; ++st) {
        issue_begin();
#pragma unroll
        for (int idx = 0; idx < LPS; ++idx) issue_part(idx);
        issue_end();
    }

    // Operand read offsets of this lane inside a stage (bytes) for k-step 0.  A lane multiplies the
    // 8 elements 16 kk + 8 (lane / 32) .. of its row in k-step kk: one 16-byte chunk of 2-byte
    // elements, chunk slot (2 kk + lane / 32) ^ swz, or the two chunks 4 kk + 2 (lane / 32), + 1 of
    // fp32 rows.  Either way the k-step's offset is the k-step 0 offset with (16 kk elements, in
    // bytes) XOR-ed in: the row part is a multiple of the row size and lies above those bits.
    const int hi = lane >> 5;
    const int a_off0 = (wm * TM * 32 + fr) * ROWB_A + (((A32 ? 2 * hi : hi) ^ swz<CPR_A>(fr & 15)) << 4);
    const int b_off0 = A_BYTES + (wn * TN * 32 + fr) * ROWB_B + ((hi ^ swz<CPR_B>(fr & 15)) << 4);
    static_assert((KS - 1) * 16 * ESA < ROWB_A && (KS - 1) * 32 < ROWB_B && A_BYTES % ROWB_B == 0,
                  "k-step offset stays inside the row");
    uint4 fa[2][TM], fb[2][TN];
    auto read_frag = [&](int slot, const unsigned char *sbase, int kk, int idx) __attribute__((always_inline)) {
        // in the order the MFMAs need them: A0, all of B, then A1..
        if (idx == 0 || idx > TN) {
            const int i = idx == 0 ? 0 : idx - TN;
            const unsigned char *at = sbase + (a_off0 ^ (kk * 16 * ESA)) + i * 32 * ROWB_A;
            if constexpr (A32)
                fa[slot][i] = round8_bf16(*reinterpret_cast<const uint4 *>(at),
                                          *reinterpret_cast<const uint4 *>(sbase + ((a_off0 ^ (kk * 16 * ESA)) ^ 16) +
                                                                           i * 32 * ROWB_A));
            else
                fa[slot][i] = *reinterpret_cast<const uint4 *>(at);
        } else {
            const int j = idx - 1;
            fb[slot][j] = *reinterpret_cast<const uint4 *>(sbase + (b_off0 ^ (kk << 5)) + j * 32 * ROWB_B);
        }
    };

    // stage 0 must be in LDS before the first operand read
    wait_vmcnt<LPS *(D - 1)>();
    __syncthreads();
#pragma unroll
    for (int idx = 0; idx < NR; ++idx) read_frag(0, smem, 0, idx);

    uint32_t parked = 0;   // entries in the LDS list (uniform; maintained at tile ends)
    int buf = 0;
    int cur_rt = vb / nqt;
    int cur_qt = vb % nqt;
    for (int it = 0; it < n_mine; ++it) {
        f32x16 acc[TM][TN];
        const int32_t row0 = (int32_t)tile_row0(cur_rt);
        const int q0 = cur_qt * BN;
        // admission keys of this lane's TN queries
        // tsc: the score a value must reach to be looked at more closely; -inf for a key of 0
        // (admit everything; its score bits decode to NaN), +inf for padding columns
        u64 tkey[TN];
        float tsc[TN];
        bool qok[TN];
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int q = q0 + (wn * TN + j) * 32 + fr;
            qok[j] = q < p.Q;
            tkey[j] = qok[j] ? (tau_in_lds ? tau_lds[q] : p.tau[q]) : ~0ull;
            tsc[j] = qok[j] ? (tkey[j] == 0ull ? -__builtin_inff() : key_score(tkey[j])) : __builtin_inff();
        }

        // one stage; FIRST: accumulators start from zero; LAST: selection fused into the last k-step
        auto stage = [&](auto first_tag, auto last_tag) __attribute__((always_inline)) {
            constexpr bool FIRST = decltype(first_tag)::value, LAST = decltype(last_tag)::value;
            const unsigned char *sb = smem + buf * STAGE;
            const int nbuf = buf + 1 == S ? 0 : buf + 1;
#pragma unroll
            for (int kk = 0; kk < KS; ++kk) {
                // Two waves share a SIMD (and its matrix core): the one further along its stage
                // issues first, so that they take turns in k-step-long runs instead of
                // interleaving instruction by instruction (measured: 2 % faster).
                if constexpr (NW == 8) {
                    if (kk >= 3) __builtin_amdgcn_s_setprio(3);
                    else if (kk == 2) __builtin_amdgcn_s_setprio(2);
                    else if (kk == 1) __builtin_amdgcn_s_setprio(1);
                    else __builtin_amdgcn_s_setprio(0);
                }
                const int cur = kk & 1;
                const bool last_kk = kk + 1 == KS;
                const unsigned char *nsb = last_kk ? smem + nbuf * STAGE : sb;
                const int nkk = last_kk ? 0 : kk + 1;
                // side instructions of this k-step: the operand reads of the next k-step (for the
                // last k-step: of the next stage), then the global->LDS loads (the rendezvous sits
                // inside k-step RK; the query part of the strip is requested after it in that
                // k-step, the datastore part in the next)
                const int nd = kk == RK + 1 ? NA : (kk == RK ? NB : 0);
                const int d0 = kk == RK + 1 ? 0 : NA;
                f32x16 outs[LAG + 1];
                RALM_SCHED_FENCE();
#pragma unroll
                for (int m = 0; m < (NM > LPS + NR ? NM : LPS + NR) + LAG; ++m) {
                    if (m < NM) {
                        const int i = m / TN, j = m % TN;
                        if constexpr (FIRST) {
                            if (kk == 0) {
                                f32x16 zero;
#pragma unroll
                                for (int v = 0; v < 16; ++v) zero[v] = 0.f;
                                acc[i][j] = mfma32<F16>(fa[cur][i], fb[cur][j], zero);
                            } else if (LAST && last_kk) {
                                outs[m % (LAG + 1)] = mfma32<F16>(fa[cur][i], fb[cur][j], acc[i][j]);
                            } else {
                                acc[i][j] = mfma32<F16>(fa[cur][i], fb[cur][j], acc[i][j]);
                            }
                        } else {
                            if (LAST && last_kk)
                                outs[m % (LAG + 1)] = mfma32<F16>(fa[cur][i], fb[cur][j], acc[i][j]);
                            else
                                acc[i][j] = mfma32<F16>(fa[cur][i], fb[cur][j], acc[i][j]);
                        }
                    }
                    if (m < NR)
                        read_frag(cur ^ 1, nsb, nkk, m);
                    else if (m - NR < nd)
                        issue_part(d0 + m - NR);
                    if (kk == RK && m == RV) {
                        // Rendezvous.  After it: the next stage is complete in LDS for every
                        // wave, and every wave has finished reading the slot that the loads
                        // issued from here on refill: the previous stage's (D = S - 1), or this
                        // stage's own (D = S; its last operand reads were issued just above
                        // and are awaited first).  No LDS data is written by ds instructions
                        // that another wave reads without a later full barrier, so no LDS fence
                        // is needed; the asm statements keep the compiler from moving memory
                        // operations across the barrier.
                        wait_vmcnt<LPS *(D - 2)>();
                        if constexpr (D == S) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                        asm volatile("" ::: "memory");
                        __builtin_amdgcn_s_barrier();
                        asm volatile("" ::: "memory");
                        issue_begin();
                    }
                    if (LAST && last_kk && m >= LAG && m - LAG < NM) {
                        const int mm = m - LAG, i = mm / TN, j = mm % TN;
                        if constexpr (ALL)
                            store_block_all(p, outs[mm % (LAG + 1)], row0 + (wm * TM + i) * 32 + (lane >> 5) * 4,
                                            (int64_t)cur_rt * BM + (wm * TM + i) * 32 + (lane >> 5) * 4,
                                            q0 + (wn * TN + j) * 32 + fr, qok[j]);
                        else
                            select_block_parked(p, pl, wave_slots, outs[mm % (LAG + 1)],
                                                row0 + (wm * TM + i) * 32 + (lane >> 5) * 4, n_rows,
                                                q0 + (wn * TN + j) * 32 + fr, qok[j], tkey[j], tsc[j]);
                    }
                    RALM_SCHED_FENCE();
                }
                if (kk == RK + 1) issue_end();
                RALM_SCHED_FENCE();
            }
            buf = nbuf;
        };

        // A wave whose query columns are all padding (the batch's last query tile is ragged) has
        // nothing to multiply or select: it only keeps its part of the load ring and the
        // rendezvous going, and reads the operands of the next tile's first k-step at the end.
        auto stage_idle = [&]() __attribute__((always_inline)) {
            const int nbuf = buf + 1 == S ? 0 : buf + 1;
            RALM_SCHED_FENCE();
            wait_vmcnt<LPS *(D - 2)>();
            if constexpr (D == S) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // its last reads of the slot
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            issue_begin();
#pragma unroll
            for (int idx = NA; idx < LPS; ++idx) issue_part(idx);   // query part, as in k-step RK
#pragma unroll
            for (int idx = 0; idx < NA; ++idx) issue_part(idx);     // datastore part, as in k-step RK + 1
            issue_end();
#pragma unroll
            for (int idx = 0; idx < NR; ++idx) read_frag(((KS - 1) & 1) ^ 1, smem + nbuf * STAGE, 0, idx);
            RALM_SCHED_FENCE();
            buf = nbuf;
        };
        const bool wave_idle = q0 + wn * TN * 32 >= p.Q;   // wave-uniform

        if (wave_idle) {
            for (int kt = 0; kt < KT; ++kt) stage_idle();
        } else if (KT == 1) {
            stage(std::true_type{}, std::true_type{});
        } else {
            stage(std::true_type{}, std::false_type{});
            for (int kt = 1; kt + 1 < KT; ++kt) stage(std::false_type{}, std::false_type{});
            stage(std::false_type{}, std::true_type{});
        }

        // tile end: every few tiles the parked entries move to the global lists
        const bool last_tile = it + 1 == n_mine;
        if ((it & 3) == 3 || last_tile) {
            __syncthreads();
            const uint32_t n = *pl.count;   // uniform: read after the barrier
            const uint32_t held = n < pl.cap ? n : pl.cap;
            if (held >= pl.cap / 4 || (last_tile && held > 0)) {
                flush_parked(p, pl, held);
                parked = 0;
            } else {
                parked = held;
            }
        }
        cur_rt += step_rt;
        cur_qt += step_qt;
        if (cur_qt >= nqt) {
            cur_qt -= nqt;
            ++cur_rt;
        }
    }
    (void)parked;
    wait_vmcnt<0>();   // the run-ahead loads must land before this workgroup's LDS is released
}

template <bool F16, int WM, int WN, int TM, int TN, int BK, int S, bool NTA, int D = S - 1, int RK = 0,
          bool A32 = false, bool ALL = false>
hipError_t launch_dma_variant(const ScanParams &p, int n_cu, hipStream_t stream)
{
    constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
    constexpr size_t ring = (size_t)S * (BM * (A32 ? 4 : 2) + BN * 2) * BK;
    constexpr size_t smem = ring + (size_t)tau_lds_q(BN) * 8 + (size_t)PARK_CAP * 12 + 16 + WM * WN * SLOW_SLOTS * 64;
    static_assert(smem <= 160 * 1024, "LDS budget");
    auto kern = scan_dma_kernel<F16, WM, WN, TM, TN, BK, S, NTA, D, RK, A32, ALL>;
    const int tau_in_lds = p.Q <= tau_lds_q(BN) ? 1 : 0;
    static std::atomic<bool> attr_done{false};   // per instantiation; setting it twice is harmless
    if (!attr_done.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        attr_done.store(true, std::memory_order_release);
    }
    const int nqt = (int)((p.Q + BN - 1) / BN);
    const int64_t total = p.n_row_tiles * (SCAN_BM / BM) * nqt;
    if (total <= 0) return hipSuccess;
    if (total > 0x7fffffffLL) return hipErrorInvalidValue;   // the kernel counts items in 32 bits
    const int per_cu = smem * 2 <= 160 * 1024 ? 2 : 1;
    int64_t grid = (int64_t)n_cu * per_cu;
    if (total < grid) grid = total;
    grid = (grid + 7) / 8 * 8;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(WM * WN * 64), smem, stream, p, nqt, tau_in_lds);
    return hipGetLastError();
}

template <bool F16>
hipError_t launch_dma(const ScanParams &p, int n_cu, hipStream_t stream)
{
    const int bn = scan_bn_for(p.Q);
    switch (bn) {
        // One query tile: nobody shares the rows through L2, they are streamed non-temporally
        // (strips of whole 128-byte lines; with 64-byte strips a line would be requested twice, a
        // stage apart, and would have to stay in L2 in between).
        case 32: return launch_dma_variant<F16, 4, 1, 2, 1, 64, 4, true>(p, n_cu, stream);
        // 64 and 128 queries: 8 waves (two per SIMD, wave tiles of 64 x 32 and 128 x 32), so that one wave's
        // waits are covered by the other's multiplies; with 4 waves of twice the width they were 5 % and 3 % slower
        case 64: return launch_dma_variant<F16, 4, 2, 2, 1, 64, 3, true, 3, 2>(p, n_cu, stream);
        case 128: return launch_dma_variant<F16, 2, 4, 4, 1, 64, 3, true, 3, 2>(p, n_cu, stream);
        default:
            // two slots of 64-element strips, refilled in place (D = S): same LDS as four 32-element
            // slots, half the rendezvous and half the L2 requests per multiply
            if (p.Q <= 256) return launch_dma_variant<F16, 2, 4, 4, 2, 64, 2, true, 2, 2>(p, n_cu, stream);
            return launch_dma_variant<F16, 2, 4, 4, 2, 64, 2, false, 2, 2>(p, n_cu, stream);
    }
}

template <int IN, int WM, int WN, int TM, int TN>
hipError_t launch_variant(const ScanParams &p, int n_cu, hipStream_t stream)
{
    constexpr int BM = WM * TM * 32, BN = WN * TN * 32, LDA = SCAN_BK + 8;
    constexpr size_t smem = (size_t)2 * (BM + BN) * LDA * sizeof(uint16_t);
    auto kern = scan_staged_kernel<IN, WM, WN, TM, TN>;
    static std::atomic<bool> attr_done{false};   // per instantiation; setting it twice is harmless
    if (!attr_done.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        attr_done.store(true, std::memory_order_release);
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
    // Launches whose thresholds admit everything (the first, tiny stage of the ladder) append
    // nearly every score: they take the staged kernel, whose epilogue writes to the global lists
    // with one atomic per lane and block.  fp32 rows always do (they are rounded on the way in).
    // a launch that keeps every score into empty lists, all of its tiles full: fixed list positions
    const int64_t last_tile = (p.tile_begin + p.n_row_tiles - 1) * p.tile_stride;
    const bool all_kept = !p.park_pushes && p.lists_empty && p.tile_skip == 0 && p.n_row_tiles > 0 &&
                          (last_tile + 1) * SCAN_BM <= p.N && p.n_row_tiles * SCAN_BM <= (int64_t)p.cap && p.cap % 2 == 0;
    if (p.in_dtype == DT_F32) {
        if (all_kept) {
            const int bn = scan_bn_for(p.Q);
            if (bn == 32) return launch_dma_variant<false, 4, 1, 1, 1, 64, 4, false, 3, 0, true, true>(p, n_cu, stream);
            if (bn == 64) return launch_dma_variant<false, 4, 1, 1, 2, 64, 3, false, 3, 2, true, true>(p, n_cu, stream);
            if (bn == 128) return launch_dma_variant<false, 2, 4, 4, 1, 32, 3, false, 3, 0, true, true>(p, n_cu, stream);
            return launch_dma_variant<false, 2, 4, 4, 2, 32, 2, false, 2, 0, true, true>(p, n_cu, stream);
        }
        // fp32 rows: batches of one query tile stream them as they are and round on the way to the
        // matrix cores (32-element strips for 128 and 256 queries: an fp32 strip row is 128 bytes)
        if (p.park_pushes && p.Q <= 32) return launch_dma_variant<false, 4, 1, 1, 1, 64, 4, true, 3, 0, true>(p, n_cu, stream);
        if (p.park_pushes && p.Q <= 64) return launch_dma_variant<false, 4, 1, 1, 2, 64, 3, true, 3, 2, true>(p, n_cu, stream);
        if (p.park_pushes && p.Q <= 128) return launch_dma_variant<false, 2, 4, 4, 1, 32, 3, true, 3, 0, true>(p, n_cu, stream);
        if (p.park_pushes && p.Q <= 256) return launch_dma_variant<false, 2, 4, 4, 2, 32, 2, true, 2, 0, true>(p, n_cu, stream);
        // several query tiles: the rows are shared through L2 (default cache policy); 11.5 ms per query tile at
        // 21M x 768 against 6.5 ms from a bf16 copy, so callers with many tiles are better off with a copy
        if (p.park_pushes) return launch_dma_variant<false, 2, 4, 4, 2, 32, 2, false, 2, 0, true>(p, n_cu, stream);
        return launch_in<DT_F32>(p, n_cu, stream);
    }
    if (!p.park_pushes) {
        // The first stage of a ladder (every score kept, lists empty): the
        // pipelined kernel with stores to fixed list positions; its tiles must all be full and fit
        // the lists.  (One 256 x 256 tile takes the staged kernel 125 us, mostly its epilogue's
        // atomics and its shallow pipeline.)
        if (all_kept) {
            const int bn = scan_bn_for(p.Q);
            if (p.in_dtype == DT_F16) {
                if (bn == 32) return launch_dma_variant<true, 4, 1, 2, 1, 64, 4, false, 3, 0, false, true>(p, n_cu, stream);
                if (bn == 64) return launch_dma_variant<true, 4, 2, 2, 1, 64, 3, false, 3, 2, false, true>(p, n_cu, stream);
                if (bn == 128) return launch_dma_variant<true, 2, 4, 4, 1, 64, 3, false, 3, 2, false, true>(p, n_cu, stream);
                return launch_dma_variant<true, 2, 4, 4, 2, 64, 2, false, 2, 2, false, true>(p, n_cu, stream);
            }
            if (bn == 32) return launch_dma_variant<false, 4, 1, 2, 1, 64, 4, false, 3, 0, false, true>(p, n_cu, stream);
            if (bn == 64) return launch_dma_variant<false, 4, 2, 2, 1, 64, 3, false, 3, 2, false, true>(p, n_cu, stream);
            if (bn == 128) return launch_dma_variant<false, 2, 4, 4, 1, 64, 3, false, 3, 2, false, true>(p, n_cu, stream);
            return launch_dma_variant<false, 2, 4, 4, 2, 64, 2, false, 2, 2, false, true>(p, n_cu, stream);
        }
        return p.in_dtype == DT_F16 ? launch_in<DT_F16>(p, n_cu, stream) : launch_in<DT_BF16>(p, n_cu, stream);
    }
    return p.in_dtype == DT_F16 ? launch_dma<true>(p, n_cu, stream) : launch_dma<false>(p, n_cu, stream);
}

}  // namespace ralm
