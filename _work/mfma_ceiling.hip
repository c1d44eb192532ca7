// Stand-alone probe: what dense bf16 MFMA rate does one MI355X sustain when the operands are
// (a) constant and (b) random data?  No memory or LDS traffic, 16 independent 32x32x16
// accumulators per wave, one wave per SIMD.  The chip lowers its clock under the switching
// activity of real data, so (b) is the practical ceiling any bf16 kernel with real operands can
// approach, below the nominal 2.5 PFLOP/s that the roofline figures are quoted against.
//
//   hipcc --offload-arch=gfx950 -O3 -o mfma_ceiling paper_2401_14021_amd/csrc/mfma_ceiling.hip && ./mfma_ceiling
#include <hip/hip_runtime.h>
#include <stdio.h>
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
__device__ unsigned hash(unsigned x) { x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16; return x; }
template <int RANDOM>
__global__ __launch_bounds__(256) void k(float *out, int iters)
{
    f32x16 acc[16];
    for (int a = 0; a < 16; ++a) for (int v = 0; v < 16; ++v) acc[a][v] = 0.f;
    // 8 operand registers sets with (optionally) random bf16 values in [-1,1)-ish range
    u32x4 ops[8];
    for (int i = 0; i < 8; ++i) {
        for (int e = 0; e < 4; ++e) {
            unsigned h = hash(threadIdx.x * 977 + blockIdx.x * 31 + i * 13 + e);
            // two bf16 with exponent ~ 2^-4..2^0 and random sign/mantissa
            unsigned lo = ((h & 0x807f) | 0x3d00 | ((h >> 7) & 0x0180)), hi = (((h >> 16) & 0x807f) | 0x3d00 | ((h >> 23) & 0x0180));
            ops[i][e] = RANDOM ? (lo | (hi << 16)) : 0x3f803f80u;
        }
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int a = 0; a < 16; ++a)
            acc[a] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ops[a & 3]), __builtin_bit_cast(bf16x8, ops[4 + (a >> 2)]), acc[a], 0, 0, 0);
    }
    float s = 0;
    for (int a = 0; a < 16; ++a) for (int v = 0; v < 16; ++v) s += acc[a][v];
    out[blockIdx.x * 256 + threadIdx.x] = s;
}
template <int R> void run()
{
    float *out; (void)hipMalloc(&out, 256 * 256 * 4);
    const int iters = 400000;
    hipLaunchKernelGGL(k<R>, dim3(256), dim3(256), 0, 0, out, 1000);
    (void)hipDeviceSynchronize();
    hipEvent_t a, b; (void)hipEventCreate(&a); (void)hipEventCreate(&b);
    (void)hipEventRecord(a);
    hipLaunchKernelGGL(k<R>, dim3(256), dim3(256), 0, 0, out, iters);
    (void)hipEventRecord(b); (void)hipEventSynchronize(b);
    float ms; (void)hipEventElapsedTime(&ms, a, b);
    printf("random=%d: %.1f ms, %.0f TFLOP/s\n", R, ms, (double)iters * 16 * 32768.0 * 4 * 256 / ms / 1e9);
}
int main() { run<0>(); run<1>(); run<1>(); return 0; }
