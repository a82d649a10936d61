// Matrix-pipe microbenchmark: what this device, in its present power state, delivers when every SIMD
// issues nothing but v_mfma_f32_32x32x16_bf16 on random operands.  The attention kernels' executed FLOP rate is quoted
// against the data-sheet peak (2.5 PFLOP/s dense bf16 at 2.4 GHz); this number says how much of that the
// device sustains when only the matrix pipeline is busy, and at which clock.
#include <hip/hip_runtime.h>

#include "clear_internal.h"

namespace clear {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kChains = 4;          // independent accumulators per wave
constexpr int kMfmaPerIter = 16;    // per wave and loop iteration
constexpr double kFlopPerMfma = 2.0 * 32 * 32 * 16;

// ticks[0]: shader-clock cycles, ticks[1]: 100 MHz reference ticks, both over the loop of workgroup 0.
__global__ void __launch_bounds__(512) mfma_peak_kernel(float* sink, unsigned long long* ticks, int iters)
{
    const int lane = threadIdx.x & 63;
    bf16x8 a, b;
    // operands with the statistics of the attention inputs (roughly uniform in [-2, 2), all mantissa bits
    // in use): the power the pipeline draws, and with it the clock the device holds, depends on the data
    unsigned h = (unsigned)(blockIdx.x * 1024 + threadIdx.x) * 2654435761u + 12345u;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        h = h * 1664525u + 1013904223u;
        a[j] = (__bf16)((float)(int)(h >> 8) * (4.0f / 16777216.0f) - 2.0f);
        h = h * 1664525u + 1013904223u;
        b[j] = (__bf16)((float)(int)(h >> 8) * (4.0f / 16777216.0f) - 2.0f);
    }
    f32x16 acc[kChains];
#pragma unroll
    for (int c = 0; c < kChains; ++c)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[c][r] = 0.f;
    const unsigned long long c0 = clock64(), w0 = wall_clock64();
#pragma unroll 1
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int k = 0; k < kMfmaPerIter; ++k) acc[k % kChains] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[k % kChains], 0, 0, 0);
    }
    const unsigned long long c1 = clock64(), w1 = wall_clock64();
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < kChains; ++c)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[c][r];
    if (s == 12345.678f) sink[0] = s;  // keeps the accumulators alive; never true for these operands
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        ticks[0] = c1 - c0;
        ticks[1] = w1 - w0;
    }
}

}  // namespace

hipError_t measure_mfma_peak(int num_cus, double seconds, double* tflops, double* shader_mhz)
{
    float* sink = nullptr;
    unsigned long long* ticks = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    hipError_t e = hipMalloc((void**)&sink, sizeof(float));
    if (e == hipSuccess) e = hipMalloc((void**)&ticks, 2 * sizeof(unsigned long long));
    if (e == hipSuccess) e = hipEventCreate(&e0);
    if (e == hipSuccess) e = hipEventCreate(&e1);
    const int nblk = num_cus, waves = 8;  // one workgroup of 8 waves per compute unit: 2 waves per SIMD
    const int iters = 20000;              // about 5 ms per launch
    double best = 0.0, mhz = 0.0, spent = 0.0;
    // repeated launches until `seconds` have been spent: the clock settles only under sustained load
    while (e == hipSuccess && spent < seconds) {
        e = hipEventRecord(e0, nullptr);
        if (e == hipSuccess) {
            hipLaunchKernelGGL(mfma_peak_kernel, dim3(nblk), dim3(waves * 64), 0, nullptr, sink, ticks, iters);
            e = hipGetLastError();
        }
        if (e == hipSuccess) e = hipEventRecord(e1, nullptr);
        if (e == hipSuccess) e = hipEventSynchronize(e1);
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
        unsigned long long h[2] = {0, 0};
        if (e == hipSuccess) e = hipMemcpy(h, ticks, sizeof(h), hipMemcpyDeviceToHost);
        if (e != hipSuccess) break;
        spent += ms * 1e-3;
        // the last launch counts: the one at the settled clock
        best = kFlopPerMfma * kMfmaPerIter * (double)iters * waves * nblk / (ms * 1e-3) / 1e12;
        mhz = h[1] ? (double)h[0] / ((double)h[1] * 0.01) : 0.0;
    }
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (sink) (void)hipFree(sink);
    if (ticks) (void)hipFree(ticks);
    if (e == hipSuccess) {
        *tflops = best;
        *shader_mhz = mhz;
    }
    return e;
}

}  // namespace clear
