// Matrix-core calibration for the benchmark: what a register-only loop of v_mfma_f32_32x32x16_bf16
// sustains on this device, and the shader clock it runs at meanwhile.  The published dense bf16 peak
// (2.5 PFLOP/s) assumes the 2.4 GHz peak engine clock; under sustained matrix load the clock settles
// lower, and this loop - no memory traffic, two wavefronts per SIMD, four independent accumulator
// chains each - is the ceiling any GEMM on the same chip can approach.  Plays the role for the
// "mfma" roofline that the plain copy kernel plays for the HBM counters.
#include <vector>

#include "free_internal.h"

namespace freemi {

namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int kCalibThreads = 512;       // 8 wavefronts: two per SIMD, as in the GEMM kernels
constexpr int kChains = 4;

__global__ __launch_bounds__(kCalibThreads) void mfma_ceiling_kernel(int32_t iters, float* __restrict__ sink,
                                                                     unsigned long long* __restrict__ clk) {
    const unsigned long long c0 = clock64(), w0 = wall_clock64();
    const int lane = threadIdx.x & 63;
    // a different pseudo-random operand pair per chain (values in [-1, 1)): consecutive MFMAs see different
    // bits on their inputs, as in a real product - constant or near-zero operands would draw less power and
    // let the clock settle higher than any GEMM can hold
    bf16x8_t a[kChains], b[kChains];
#pragma unroll
    for (int k = 0; k < kChains; ++k)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            uint32_t h = static_cast<uint32_t>(threadIdx.x * 64 + k * 16 + e) * 2654435761u;
            h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
            a[k][e] = static_cast<__bf16>(static_cast<float>(h & 0xffff) * (1.0f / 32768.0f) - 1.0f);
            b[k][e] = static_cast<__bf16>(static_cast<float>(h >> 16) * (1.0f / 32768.0f) - 1.0f);
        }
    f32x16_t acc[kChains];
#pragma unroll
    for (int k = 0; k < kChains; ++k)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[k][e] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int k = 0; k < kChains; ++k) acc[k] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[k], b[k], acc[k], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < kChains; ++k)
#pragma unroll
        for (int e = 0; e < 16; ++e) s += acc[k][e];
    // the comparison only keeps the loop alive
    if (s == 12345.678f) sink[blockIdx.x * kCalibThreads + threadIdx.x] = s;
    if (threadIdx.x == 0) {
        clk[2 * blockIdx.x] = clock64() - c0;
        clk[2 * blockIdx.x + 1] = wall_clock64() - w0;
    }
}

}  // namespace

int32_t run_mfma_ceiling(int32_t iters, double* tflops, double* mhz, hipStream_t s) {
    int dev = 0, cus = 0, wall_khz = 0;
    if (!hip_ok(hipGetDevice(&dev))) return FREE_ERR_HIP;
    if (!hip_ok(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev))) return FREE_ERR_HIP;
    if (!hip_ok(hipDeviceGetAttribute(&wall_khz, hipDeviceAttributeWallClockRate, dev))) return FREE_ERR_HIP;
    if (cus < 1 || wall_khz < 1) return FREE_ERR_HIP;
    float* sink = nullptr;
    unsigned long long* clk = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    std::vector<unsigned long long> h(2 * static_cast<size_t>(cus));
    int32_t rc = FREE_ERR_HIP;
    float ms = 0.f;
    do {
        if (!hip_ok(hipMalloc(&sink, sizeof(float) * kCalibThreads * cus))) break;
        if (!hip_ok(hipMalloc(&clk, sizeof(unsigned long long) * 2 * cus))) break;
        if (!hip_ok(hipEventCreate(&e0)) || !hip_ok(hipEventCreate(&e1))) break;
        // one untimed launch to bring the clocks to their loaded state, then the timed one
        hipLaunchKernelGGL(mfma_ceiling_kernel, dim3(cus), dim3(kCalibThreads), 0, s, iters, sink, clk);
        if (!launch_ok() || !hip_ok(hipEventRecord(e0, s))) break;
        hipLaunchKernelGGL(mfma_ceiling_kernel, dim3(cus), dim3(kCalibThreads), 0, s, iters, sink, clk);
        if (!launch_ok() || !hip_ok(hipEventRecord(e1, s))) break;
        if (!hip_ok(hipEventSynchronize(e1)) || !hip_ok(hipEventElapsedTime(&ms, e0, e1))) break;
        if (!hip_ok(hipMemcpy(h.data(), clk, sizeof(unsigned long long) * 2 * cus, hipMemcpyDeviceToHost))) break;
        rc = FREE_OK;
    } while (false);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (sink) (void)hipFree(sink);
    if (clk) (void)hipFree(clk);
    if (rc != FREE_OK) return rc;
    const double flops = static_cast<double>(cus) * (kCalibThreads / 64) * static_cast<double>(iters) * kChains *
                         (2.0 * 32 * 32 * 16);
    *tflops = flops / (static_cast<double>(ms) * 1e-3) / 1e12;
    double cyc = 0.0, wall = 0.0;
    for (int b = 0; b < cus; ++b) { cyc += static_cast<double>(h[2 * b]); wall += static_cast<double>(h[2 * b + 1]); }
    *mhz = wall > 0.0 ? cyc / wall * (static_cast<double>(wall_khz) * 1e-3) : 0.0;
    return FREE_OK;
}

}  // namespace freemi
