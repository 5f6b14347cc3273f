// Calibration, not part of the library: the rate at which this GPU sustains
// v_mfma_f32_32x32x16_bf16 when nothing else limits it (operands and accumulators stay in
// registers, no memory traffic), with all-zero and with random operands.  The matrix unit's
// clock under load depends on the data (power), so the random-operand rate, not the nominal
// 2.5 PFLOP/s, is what a GEMM on real data can approach.
//
// build and run:
//   hipcc --offload-arch=gfx950 -O3 -Xclang -target-feature -Xclang -packed-fp32-ops \
//       paper_2002_06015_amd/calib/mfma_bf16_peak.hip -o /tmp/mfma_bf16_peak && /tmp/mfma_bf16_peak
#include <hip/hip_runtime.h>

#include <cstdio>

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned short ushortx8 __attribute__((ext_vector_type(8)));

#define CHECK(call)                                                                          \
    do {                                                                                     \
        hipError_t e_ = (call);                                                              \
        if (e_ != hipSuccess) {                                                              \
            fprintf(stderr, "%s:%d: %s\n", __FILE__, __LINE__, hipGetErrorString(e_));       \
            return 1;                                                                        \
        }                                                                                    \
    } while (0)

// Four independent accumulator blocks per wavefront (the instruction's latency is covered),
// four wavefronts per workgroup.  pattern 0: every operand is zero; 1: bf16 values of magnitude
// 1..2 with random mantissas, a positive, b negative; 2: random sign, random mantissa and one of
// eight binary exponents (2^-7 .. 1), which is what the planes of real operands look like.  The
// sums stay finite in every case.
__global__ __launch_bounds__(256) void mfma_loop(float *out, long long *clocks, int iters, int pattern)
{
    constexpr int NACC = 4;
    floatx16 acc[NACC];
    for (int i = 0; i < NACC; ++i)
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    ushortx8 a[4], b[4];
    unsigned h = threadIdx.x * 2654435761u + blockIdx.x * 40503u;
    for (int i = 0; i < 4; ++i)
        for (int e = 0; e < 8; ++e) {
            h = h * 1664525u + 1013904223u;
            a[i][e] = pattern == 0 ? 0 : pattern == 1 ? (unsigned short)(0x3f80 + (h >> 25))
                                       : (unsigned short)(((h >> 16) & 0x8000) | ((120 + ((h >> 28) & 7)) << 7) | ((h >> 20) & 0x7f));
            h = h * 1664525u + 1013904223u;
            b[i][e] = pattern == 0 ? 0 : pattern == 1 ? (unsigned short)(0xbf80 + (h >> 25))
                                       : (unsigned short)(((h >> 16) & 0x8000) | ((120 + ((h >> 28) & 7)) << 7) | ((h >> 20) & 0x7f));
        }
    const long long c0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int i = 0; i < NACC; ++i)
                acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[(u + i) & 3]),
                                                                 __builtin_bit_cast(bf16x8, b[(u + 3 * i) & 3]), acc[i], 0, 0, 0);
    }
    const long long c1 = clock64(), w1 = wall_clock64();
    float s = 0.f;
    for (int i = 0; i < NACC; ++i)
        for (int v = 0; v < 16; ++v) s += acc[i][v];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        clocks[0] = c1 - c0;   // shader clock cycles
        clocks[1] = w1 - w0;   // constant-rate wall clock ticks
    }
}

int main()
{
    constexpr int kMaxBlocks = 2048;
    float *out = nullptr;
    long long *clocks = nullptr, host[2] = {0, 0};
    CHECK(hipMalloc((void **)&out, sizeof(float) * 256 * kMaxBlocks));
    CHECK(hipMalloc((void **)&clocks, sizeof(host)));
    int wall_khz = 0;
    CHECK(hipDeviceGetAttribute(&wall_khz, hipDeviceAttributeWallClockRate, 0));
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    const int grids[] = {256, 512, 2048};   // 1, 2 and 8 workgroups per compute unit
    const char *names[3] = {"zero operands", "random mantissas", "random sign / exponent / mantissa"};
    for (int pattern = 0; pattern < 3; ++pattern)
        for (int rep = 0; rep < 2; ++rep)   // the second pass of each is the sustained one
            for (int blocks : grids) {
                const int iters = 40000 * 256 / blocks;
                CHECK(hipEventRecord(e0, 0));
                mfma_loop<<<dim3(blocks), dim3(256), 0, 0>>>(out, clocks, iters, pattern);
                CHECK(hipGetLastError());
                CHECK(hipEventRecord(e1, 0));
                CHECK(hipDeviceSynchronize());
                float ms = 0.f;
                CHECK(hipEventElapsedTime(&ms, e0, e1));
                CHECK(hipMemcpy(host, clocks, sizeof(host), hipMemcpyDeviceToHost));
                // per workgroup: 4 wavefronts x iters x 16 instructions x (2 * 32 * 32 * 16) flops
                const double flops = (double)blocks * 4.0 * iters * 16.0 * 32768.0;
                const double seconds = (double)host[1] / (wall_khz * 1e3);
                printf("%-33s pass %d, %4d workgroups x %6d iterations: %8.3f ms  %7.1f TFLOP/s  shader clock %4.0f MHz\n",
                       names[pattern], rep, blocks, iters, ms, flops / ms / 1e9, (double)host[0] / seconds / 1e6);
            }
    CHECK(hipFree(out));
    CHECK(hipFree(clocks));
    return 0;
}
