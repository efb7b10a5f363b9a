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

// Ceiling of the local data share: every lane reads 16 bytes per instruction from addresses that spread over all
// banks (consecutive lanes, consecutive quads), many reads in flight; the frontier kernels read their states
// from LDS in the same 128-bit accesses.
constexpr int kLdsQuads = 2048;      // 32 KB per block
constexpr int kLdsUnroll = 8;        // reads per batch, 4 KB apart
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void k_lds_peak(uint32_t* __restrict__ out, int trips, uint32_t key) {
    __shared__ uint4 buf[kLdsQuads];
    for (int i = threadIdx.x; i < kLdsQuads; i += 256) buf[i] = make_uint4(key + i, key ^ (uint32_t)i, key * 3u + i, key - i);
    __syncthreads();
    uint32_t acc = 0u;
    uint32_t at = threadIdx.x;
    for (int t = 0; t < trips; ++t) {
        // (written out: the compiler drops a plain loop of reads whose sum it does not need)
        const uint32_t addr = (uint32_t)(uintptr_t)buf + ((at & 255u) << 4);
        u32x4 v0, v1, v2, v3, v4, v5, v6, v7;
        asm volatile("ds_read_b128 %0, %8\n\tds_read_b128 %1, %8 offset:4096\n\tds_read_b128 %2, %8 offset:8192\n\t"
                     "ds_read_b128 %3, %8 offset:12288\n\tds_read_b128 %4, %8 offset:16384\n\tds_read_b128 %5, %8 offset:20480\n\t"
                     "ds_read_b128 %6, %8 offset:24576\n\tds_read_b128 %7, %8 offset:28672\n\ts_waitcnt lgkmcnt(0)"
                     : "=&v"(v0), "=&v"(v1), "=&v"(v2), "=&v"(v3), "=&v"(v4), "=&v"(v5), "=&v"(v6), "=&v"(v7)
                     : "v"(addr)
                     : "memory");
        acc ^= v0.x ^ v1.y ^ v2.z ^ v3.w ^ v4.x ^ v5.y ^ v6.z ^ v7.w;
        at += 64u;
    }
    if (acc == 0x12345678u) out[0] = acc;      // keeps the sums alive; practically never taken
}

template <typename Launch>
hipError_t best_rate(int reps, double work, double* rate, hipStream_t stream, Launch launch) {
    uint32_t* out = nullptr;
    hipError_t e = hipMalloc(&out, 256);
    if (e != hipSuccess) return e;
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    e = hipEventCreate(&ev0);
    if (e == hipSuccess) e = hipEventCreate(&ev1);
    double best = 0.0;
    for (int r = 0; r < reps + 1 && e == hipSuccess; ++r) {
        e = hipEventRecord(ev0, stream);
        if (e != hipSuccess) break;
        launch(out, r);
        e = hipGetLastError();
        if (e == hipSuccess) e = hipEventRecord(ev1, stream);
        if (e == hipSuccess) e = hipEventSynchronize(ev1);
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, ev0, ev1);
        if (e == hipSuccess && r > 0 && ms > 0.f) best = std::max(best, work / (ms * 1e-3));      // the first run warms up
    }
    if (ev0) (void)hipEventDestroy(ev0);
    if (ev1) (void)hipEventDestroy(ev1);
    (void)hipFree(out);
    if (e == hipSuccess) *rate = best;
    return e;
}

}  // namespace

// Runs the kernel `reps` times on `stream` and returns the best rate in bytes read from LDS per second.
hipError_t measure_lds_peak(int reps, double* bytes_per_s, hipStream_t stream) {
    const int trips = 2048, blocks = 256 * 16;
    const double bytes = (double)blocks * 256.0 * (double)trips * kLdsUnroll * 16.0;
    return best_rate(reps, bytes, bytes_per_s, stream, [&](uint32_t* out, int r) {
        hipLaunchKernelGGL(k_lds_peak, dim3(blocks), dim3(256), 0, stream, out, trips, 0x9e3779b9u + (uint32_t)r);
    });
}

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
