// Measured ceiling of the 32-bit integer vector ALU: the figure the evaluators' lane-operation rates are
// set against is derived from the unit counts and the clock (256 compute units x 128 lanes per clock x
// 2.4 GHz, the rate behind the published fp32 vector peak); this kernel shows what a stream of independent
// v_xor_b32 instructions reaches on the device at hand (a wavefront's instruction every two to three cycles
// per SIMD, not every four).
#include <algorithm>

#include "p2_device.h"

namespace p2 {

namespace {

constexpr int kPeakChains = 8;       // independent accumulators per lane
constexpr int kPeakUnroll = 16;      // instructions per accumulator and loop trip

__global__ __launch_bounds__(256) void k_alu_peak(uint32_t* __restrict__ out, int trips, uint32_t key) {
    uint32_t a[kPeakChains];
#pragma unroll
    for (int c = 0; c < kPeakChains; ++c) a[c] = threadIdx.x * 2654435761u + (uint32_t)c;
    for (int t = 0; t < trips; ++t) {
#pragma unroll
        for (int u = 0; u < kPeakUnroll; ++u) {
#pragma unroll
            for (int c = 0; c < kPeakChains; ++c) asm volatile("v_xor_b32 %0, %0, %1" : "+v"(a[c]) : "v"(key));
        }
    }
    uint32_t r = 0;
#pragma unroll
    for (int c = 0; c < kPeakChains; ++c) r ^= a[c];
    if (r == 0x12345678u) out[0] = r;      // keeps the chains alive; practically never taken
}

}  // namespace

// Runs the kernel `reps` times on `stream` and returns the best rate in lane-operations per second.
hipError_t measure_alu_peak(int reps, double* lane_ops_per_s, hipStream_t stream) {
    uint32_t* out = nullptr;
    hipError_t e = hipMalloc(&out, 256);
    if (e != hipSuccess) return e;
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    e = hipEventCreate(&ev0);
    if (e == hipSuccess) e = hipEventCreate(&ev1);
    const int trips = 2048, blocks = 256 * 32;
    double best = 0.0;
    for (int r = 0; r < reps + 1 && e == hipSuccess; ++r) {
        e = hipEventRecord(ev0, stream);
        if (e != hipSuccess) break;
        hipLaunchKernelGGL(k_alu_peak, dim3(blocks), dim3(256), 0, stream, out, trips, 0x9e3779b9u + (uint32_t)r);
        e = hipGetLastError();
        if (e == hipSuccess) e = hipEventRecord(ev1, stream);
        if (e == hipSuccess) e = hipEventSynchronize(ev1);
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, ev0, ev1);
        if (e == hipSuccess && r > 0 && ms > 0.f) {      // the first run warms up
            const double ops = (double)blocks * 256.0 * (double)trips * kPeakUnroll * kPeakChains;
            best = std::max(best, ops / (ms * 1e-3));
        }
    }
    if (ev0) (void)hipEventDestroy(ev0);
    if (ev1) (void)hipEventDestroy(ev1);
    (void)hipFree(out);
    if (e == hipSuccess) *lane_ops_per_s = best;
    return e;
}

}  // namespace p2
