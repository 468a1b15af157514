// Measurement aid: what the matrix cores of this part sustain on their own.  A loop of
// independent v_mfma_f32_32x32x16_bf16 (four accumulator chains per wave, two waves per SIMD,
// no memory traffic), timed with HIP events, with the shader clock read back from the cycle
// counter against the 100 MHz wall counter.  Operands are either small constants or
// pseudo-random bf16 values: the sustained clock, and with it the ceiling any kernel built on
// this instruction can reach, depends on how many bits toggle.
#include <hip/hip_runtime.h>

#include "../../include/dfa.h"
#include "../../include/dfa_bench.h"
#include "dfa_device.h"

namespace dfa {
namespace {

__global__ __launch_bounds__(256) void mfma_loop_kernel(int iters, int random_operands, float* sink, long long* clocks) {
    const long long c0 = clock64(), w0 = wall_clock64();
    bf16x8 a, b;
    unsigned s = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
    for (int t = 0; t < 8; ++t) {
        if (random_operands) {
            s = s * 1664525u + 1013904223u;
            a[t] = (__bf16)(((int)(s >> 8) % 2001 - 1000) * 0.001f);
            s = s * 1664525u + 1013904223u;
            b[t] = (__bf16)(((int)(s >> 8) % 2001 - 1000) * 0.001f);
        } else {
            a[t] = (__bf16)(float)(threadIdx.x % 3);
            b[t] = (__bf16)(float)(threadIdx.x % 5);
        }
    }
    floatx16 acc[4];
    for (int i = 0; i < 4; ++i)
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 16; ++i)
            asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc[i % 4]) : "v"(a), "v"(b));
    }
    float total = 0.f;
    for (int i = 0; i < 4; ++i)
        for (int v = 0; v < 16; ++v) total += acc[i][v];
    if (total == 12345.678f) sink[0] = total;              // keeps the loop alive, never true in practice
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        clocks[0] = clock64() - c0;
        clocks[1] = wall_clock64() - w0;
    }
}

}  // namespace
}  // namespace dfa

extern "C" int dfa_mfma_peak(int32_t random_operands, float* tflops, float* shader_mhz) {
    if (!tflops || !shader_mhz) return DFA_ERR_NULL;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
        return DFA_ERR_LAUNCH;
    float* sink = nullptr;
    long long* clocks = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    int rc = DFA_ERR_LAUNCH;
    const int iters = 60000, grid = 2 * cus;               // two 4-wave workgroups per CU: two waves per SIMD
    float ms = 0.f;
    long long h[2] = {0, 0};
    if (hipMalloc(&sink, sizeof(float)) == hipSuccess && hipMalloc(&clocks, 2 * sizeof(long long)) == hipSuccess &&
        hipEventCreate(&e0) == hipSuccess && hipEventCreate(&e1) == hipSuccess) {
        hipLaunchKernelGGL(dfa::mfma_loop_kernel, dim3(grid), dim3(256), 0, nullptr, 200, random_operands, sink, clocks);
        if (hipEventRecord(e0, nullptr) == hipSuccess) {
            hipLaunchKernelGGL(dfa::mfma_loop_kernel, dim3(grid), dim3(256), 0, nullptr, iters, random_operands, sink, clocks);
            if (hipGetLastError() == hipSuccess && hipEventRecord(e1, nullptr) == hipSuccess &&
                hipEventSynchronize(e1) == hipSuccess && hipEventElapsedTime(&ms, e0, e1) == hipSuccess &&
                hipMemcpy(h, clocks, sizeof(h), hipMemcpyDeviceToHost) == hipSuccess && ms > 0.f && h[1] > 0) {
                const double flop = (double)grid * 4 * iters * 16 * (2.0 * 32 * 32 * 16);
                *tflops = (float)(flop / (ms * 1e-3) / 1e12);
                *shader_mhz = (float)((double)h[0] / (double)h[1] * 100.0);
                rc = DFA_OK;
            }
        }
    }
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (sink) (void)hipFree(sink);
    if (clocks) (void)hipFree(clocks);
    return rc;
}
