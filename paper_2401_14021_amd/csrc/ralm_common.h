// Shared device helpers of the retrieval library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ralm {

typedef unsigned long long u64;

enum { DT_F32 = 0, DT_BF16 = 1, DT_F16 = 2 };
enum { METRIC_IP = 0, METRIC_L2 = 1 };   // inner product; minus the squared Euclidean distance
constexpr int L2_EXTRA_COLS = 8;        // columns behind a scan-copy row that hold its squared norm

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// ---- ranking keys -----------------------------------------------------------------------
// A candidate (score, row id) is packed into one 64-bit key whose unsigned order is the
// library's ranking: larger key = better = (higher score, then lower id).  -0.0 is folded
// into +0.0 first so that equal floats always give equal score bits.
__device__ __forceinline__ uint32_t score_bits(float s)
{
    s += 0.0f;
    uint32_t u = __float_as_uint(s);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float bits_score(uint32_t b)
{
    uint32_t u = (b & 0x80000000u) ? (b & 0x7fffffffu) : ~b;
    return __uint_as_float(u);
}
__device__ __forceinline__ u64 make_key(float s, int32_t id)
{
    return ((u64)score_bits(s) << 32) | (uint32_t)(0x7fffffff - id);
}
__device__ __forceinline__ int32_t key_id(u64 key) { return 0x7fffffff - (int32_t)(uint32_t)key; }
__device__ __forceinline__ float key_score(u64 key) { return bits_score((uint32_t)(key >> 32)); }

// ---- element conversions ----------------------------------------------------------------
// fp32 -> bf16 bits, round to nearest even (finite inputs).
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}
__device__ __forceinline__ uint32_t f32_to_f16_bits(float f)
{
    _Float16 h = (_Float16)f;   // v_cvt_f16_f32, round to nearest even
    return (uint32_t)__builtin_bit_cast(unsigned short, h);
}
__device__ __forceinline__ float f16_bits_to_f32(uint32_t h)
{
    return (float)__builtin_bit_cast(_Float16, (unsigned short)h);
}
template <int DT>
__device__ __forceinline__ uint32_t f32_to_scan_bits(float f)
{
    return DT == DT_F16 ? f32_to_f16_bits(f) : f32_to_bf16_bits(f);
}
template <int DT>
__device__ __forceinline__ uint4 pack8(const float4 &a, const float4 &b)
{
    uint4 r;
    r.x = f32_to_scan_bits<DT>(a.x) | (f32_to_scan_bits<DT>(a.y) << 16);
    r.y = f32_to_scan_bits<DT>(a.z) | (f32_to_scan_bits<DT>(a.w) << 16);
    r.z = f32_to_scan_bits<DT>(b.x) | (f32_to_scan_bits<DT>(b.y) << 16);
    r.w = f32_to_scan_bits<DT>(b.z) | (f32_to_scan_bits<DT>(b.w) << 16);
    return r;
}

// ---- sums of doubles across lanes ------------------------------------------------------------
// Lane exchanges through DPP and readlane: a shuffle through LDS costs ~100 cycles of latency per
// level, and these sums sit at the end of every exact score.
template <int CTRL>
__device__ __forceinline__ double dpp_mov_f64(double v)
{
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), CTRL, 0xf, 0xf, false);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), CTRL, 0xf, 0xf, false);
    return __hiloint2double(hi, lo);
}
// sum over the 16 lanes of a row (lanes 16 r .. 16 r + 15); every lane gets its row's sum
__device__ __forceinline__ double row16_sum(double v)
{
    v += dpp_mov_f64<0xB1>(v);    // quad_perm [1,0,3,2]: lane ^ 1
    v += dpp_mov_f64<0x4E>(v);    // quad_perm [2,3,0,1]: lane ^ 2
    v += dpp_mov_f64<0x141>(v);   // row_half_mirror: the other quad of the 8 (quads are uniform by now)
    v += dpp_mov_f64<0x140>(v);   // row_mirror: the other half of the 16
    return v;
}
__device__ __forceinline__ double readlane_f64(double v, int lane)
{
    return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(v), lane),
                            __builtin_amdgcn_readlane(__double2loint(v), lane));
}
// sum over the 64 lanes of a wave, always in this order; every lane gets it
__device__ __forceinline__ double wave64_sum(double v)
{
    v = row16_sum(v);
    return (readlane_f64(v, 0) + readlane_f64(v, 16)) + (readlane_f64(v, 32) + readlane_f64(v, 48));
}

}  // namespace ralm
