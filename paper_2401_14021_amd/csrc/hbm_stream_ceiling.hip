// Stand-alone probe (not part of libralm.so): the HBM read rate one MI355X sustains when a
// 32 GB buffer is streamed exactly once, in the access patterns the scan kernel can use.
//
//   hipcc --offload-arch=gfx950 -O3 -o hbm_stream_ceiling hbm_stream_ceiling.hip && ./hbm_stream_ceiling
//
// Patterns (256 persistent workgroups of 4 waves, global->LDS loads of 1 KB per wave instruction,
// DEPTH groups of loads in flight per wave; rows are 1536 bytes as in a 768-dim bf16 datastore):
//   contiguous      each instruction reads 1 KB of consecutive bytes
//   128 B per row   each instruction reads 8 rows x 128 bytes (a 64-element strip of 8 rows)
//   64 B per row    each instruction reads 16 rows x 64 bytes (a 32-element strip of 16 rows);
//                   the other half of each 128-byte line is requested one strip later
// and, for comparison, plain 16-byte register loads from a large grid.
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <stdlib.h>

#define CHECK(x)                                                                  \
    do {                                                                          \
        hipError_t e_ = (x);                                                      \
        if (e_ != hipSuccess) {                                                   \
            printf("%s failed: %s\n", #x, hipGetErrorString(e_));                 \
            exit(1);                                                              \
        }                                                                         \
    } while (0)

constexpr int ROWB = 1536, TILE_ROWS = 256, TILE = TILE_ROWS * ROWB;

__device__ __forceinline__ void dma_1kb(const unsigned char *base, unsigned voff, unsigned lds_base)
{
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_base), "v"(voff), "s"(base)
                 : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// SEG = contiguous bytes per row and instruction (0: fully contiguous); every step of the loop
// issues PER instructions per wave (PER * 4 KB per workgroup) into a ring of DEPTH slots.
template <int SEG, int DEPTH>
__global__ __launch_bounds__(256) void stream_kernel(const unsigned char *src, long tiles, unsigned *sink)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char *)smem;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    constexpr int PER = SEG == 64 ? 4 : 8;               // instructions per wave and step
    constexpr int STEP_BYTES = PER * 4 * 1024;            // per workgroup
    constexpr int STEPS = TILE / STEP_BYTES;
    const int G = gridDim.x, b = blockIdx.x;
    const int vb = (b % 8) * (G / 8) + b / 8;             // neighbours in tile order share an XCD
    const long n_items = vb < tiles ? (tiles - vb + G - 1) / G : 0;
    const long total = n_items * STEPS;
    int slot = 0;
    for (long i = 0; i < total; ++i) {
        const long t = vb + (i / STEPS) * G;
        const int ks = (int)(i % STEPS);
        const unsigned char *base = src + t * TILE;
        const unsigned lds = lds0 + slot * STEP_BYTES + wave * (PER * 1024);
        if constexpr (SEG == 0) {
            base += ks * STEP_BYTES + wave * (PER * 1024);
#pragma unroll
            for (int j = 0; j < PER; ++j) dma_1kb(base + j * 1024, lane * 16, lds + j * 1024);
        } else {
            constexpr int LPR = SEG / 16, RPI = 64 / LPR;  // lanes per row, rows per instruction
            const unsigned voff = (lane / LPR) * ROWB + (lane % LPR) * 16;
#pragma unroll
            for (int j = 0; j < PER; ++j)
                dma_1kb(base + (long)(wave * 64 + j * RPI) * ROWB + ks * SEG, voff, lds + j * 1024);
        }
        slot = slot + 1 == DEPTH ? 0 : slot + 1;
        wait_vmcnt<PER *(DEPTH - 1)>();
    }
    wait_vmcnt<0>();
    __syncthreads();
    if (threadIdx.x == 0) sink[blockIdx.x] = smem[5];
}

__global__ __launch_bounds__(256) void plain_kernel(const uint4 *src, long n16, unsigned *sink)
{
    unsigned acc = 0;
    const long stride = (long)gridDim.x * 256;
    long i = (long)blockIdx.x * 256 + threadIdx.x;
    for (; i + 7 * stride < n16; i += 8 * stride) {
        uint4 r[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) r[u] = src[i + u * stride];
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += r[u].x ^ r[u].y ^ r[u].z ^ r[u].w;
    }
    if (acc == 0x12345678u) sink[0] = acc;
}

template <typename K>
void run(const char *name, K kern, const unsigned char *src, long tiles, int lds, unsigned *sink)
{
    hipEvent_t a, b;
    CHECK(hipEventCreate(&a));
    CHECK(hipEventCreate(&b));
    CHECK(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds));
    float best = 1e9f;
    for (int r = 0; r < 4; ++r) {
        CHECK(hipEventRecord(a));
        hipLaunchKernelGGL(kern, dim3(256), dim3(256), lds, 0, src, tiles, sink);
        CHECK(hipEventRecord(b));
        CHECK(hipEventSynchronize(b));
        float ms;
        CHECK(hipEventElapsedTime(&ms, a, b));
        if (r && ms < best) best = ms;
    }
    printf("%-32s %.3f ms  %.3f TB/s\n", name, best, (double)tiles * TILE / best / 1e9);
    fflush(stdout);
}

int main()
{
    const long tiles = 82032;   // 21 M rows of 1536 bytes
    const size_t bytes = (size_t)tiles * TILE;
    unsigned char *src;
    unsigned *sink;
    CHECK(hipMalloc(&src, bytes));
    CHECK(hipMemset(src, 1, bytes));
    CHECK(hipMalloc(&sink, 65536 * 4));
    CHECK(hipDeviceSynchronize());
    printf("streaming %.2f GB once per launch\n", bytes / 1e9);
    run("contiguous, depth 2", stream_kernel<0, 2>, src, tiles, 2 * 32768, sink);
    run("contiguous, depth 4", stream_kernel<0, 4>, src, tiles, 4 * 32768, sink);
    run("128 B per row, depth 2", stream_kernel<128, 2>, src, tiles, 2 * 32768, sink);
    run("128 B per row, depth 4", stream_kernel<128, 4>, src, tiles, 4 * 32768, sink);
    run("64 B per row, depth 4", stream_kernel<64, 4>, src, tiles, 4 * 16384, sink);
    run("64 B per row, depth 8", stream_kernel<64, 8>, src, tiles, 8 * 16384, sink);
    {
        hipEvent_t a, b;
        CHECK(hipEventCreate(&a));
        CHECK(hipEventCreate(&b));
        float best = 1e9f;
        for (int r = 0; r < 4; ++r) {
            CHECK(hipEventRecord(a));
            hipLaunchKernelGGL(plain_kernel, dim3(16384), dim3(256), 0, 0, (const uint4 *)src, (long)(bytes / 16), sink);
            CHECK(hipEventRecord(b));
            CHECK(hipEventSynchronize(b));
            float ms;
            CHECK(hipEventElapsedTime(&ms, a, b));
            if (r && ms < best) best = ms;
        }
        printf("%-32s %.3f ms  %.3f TB/s\n", "plain 16-byte loads, 16384 blocks", best, bytes / best / 1e9);
    }
    return 0;
}
