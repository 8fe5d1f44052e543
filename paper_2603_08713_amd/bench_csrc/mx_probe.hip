// Yardstick for the GEMM numbers: the rate at which the device sustains back-to-back
// v_mfma_scale_f32_32x32x64_f8f6f4 (FP4) out of registers, with nothing else going on.  Under load the
// clock follows the power the operands' bit patterns draw, so the rate depends on the data: constant
// operands run close to the published peak, random ones far below it.
//
// This file is a measurement aid of the benchmark, built into libmx4_bench.so; it is not part of the product
// library (libmx4.so allocates nothing and holds no measurement code) and shares nothing with it.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mxb {
namespace {

constexpr int kWave = 64;

typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kProbeThreads = 512;  // two wavefronts per SIMD
constexpr int kProbeBlocks = 256;   // one workgroup per compute unit
constexpr int kProbeChain = 4;      // independent accumulators per wavefront
constexpr int kProbeWords = 4096;   // operand words the lanes pick from

__global__ __launch_bounds__(kProbeThreads) void mfma_probe_kernel(const v4i* operands, float* sink, int iters) {
    const int l = threadIdx.x;
    v4i a[kProbeChain], b[kProbeChain];
#pragma unroll
    for (int i = 0; i < kProbeChain; ++i) {
        a[i] = operands[(l * 7 + i * 64 + blockIdx.x) % (kProbeWords / 4)];
        b[i] = operands[(l * 13 + i * 97 + blockIdx.x * 3) % (kProbeWords / 4)];
    }
    const int sa = 120 + (a[0].x & 7), sb = 120 + (b[0].x & 7);  // E8M0 bytes near 1.0
    v16f acc[kProbeChain];
#pragma unroll
    for (int i = 0; i < kProbeChain; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < kProbeChain; ++i) {
            const v8i a8 = __builtin_shufflevector(a[i], a[i], 0, 1, 2, 3, -1, -1, -1, -1);
            const v8i b8 = __builtin_shufflevector(b[i], b[i], 0, 1, 2, 3, -1, -1, -1, -1);
            acc[i] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a8, b8, acc[i], 4, 4, 0, sa, 0, sb);
        }
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < kProbeChain; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) s += acc[i][e];
    sink[blockIdx.x * kProbeThreads + l] = s;
}

}  // namespace
}  // namespace mxb

// Runs `iters` rounds of four matrix instructions per wavefront on every SIMD of the device and returns the
// sustained rate in TFLOP/s through *tflops.  random_operands != 0 fills the operand registers with random
// bits (seeded), otherwise every nibble is the same code.  Allocates and frees its own small buffers.  Returns 0,
// or -1 on bad arguments or any HIP error.  The caller has made sure the device is gfx950.
extern "C" int mxb_mfma_rate(int random_operands, int iters, double* tflops) {
    using namespace mxb;
    if (!tflops || iters <= 0 || iters > (1 << 22)) return -1;
    v4i* operands = nullptr;
    float* sink = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    int status = -1;
    uint32_t* host = new uint32_t[kProbeWords];
    uint32_t x = 0x9E3779B9u;
    for (int i = 0; i < kProbeWords; ++i) {
        x ^= x << 13; x ^= x >> 17; x ^= x << 5;  // xorshift32
        host[i] = random_operands ? x : 0x22222222u;
    }
    float ms = 0.f;
    if (hipMalloc(&operands, kProbeWords * 4) == hipSuccess &&
        hipMalloc(&sink, (size_t)kProbeBlocks * kProbeThreads * 4) == hipSuccess &&
        hipMemcpy(operands, host, kProbeWords * 4, hipMemcpyHostToDevice) == hipSuccess &&
        hipEventCreate(&e0) == hipSuccess && hipEventCreate(&e1) == hipSuccess) {
        hipLaunchKernelGGL(mfma_probe_kernel, dim3(kProbeBlocks), dim3(kProbeThreads), 0, 0, operands, sink, 64);  // warm-up
        if (hipEventRecord(e0, 0) == hipSuccess) {
            hipLaunchKernelGGL(mfma_probe_kernel, dim3(kProbeBlocks), dim3(kProbeThreads), 0, 0, operands, sink, iters);
            if (hipEventRecord(e1, 0) == hipSuccess && hipEventSynchronize(e1) == hipSuccess &&
                hipEventElapsedTime(&ms, e0, e1) == hipSuccess && ms > 0.f) {
                const double flops = 2.0 * 32 * 32 * 64 * kProbeChain * (double)iters * (kProbeThreads / kWave) * kProbeBlocks;
                *tflops = flops / (ms * 1e-3) / 1e12;
                status = 0;
            }
        }
    }
    (void)hipGetLastError();
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (operands) (void)hipFree(operands);
    if (sink) (void)hipFree(sink);
    delete[] host;
    return status;
}
