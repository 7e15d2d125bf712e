// Exclusive prefix sum of a uint32 array in device memory (total must stay
// below 2^32), in place, as three launches: per-chunk totals, scan of the
// totals by one block, per-chunk scan with the chunk's base added.
// Internal header; every translation unit that includes it gets its own copy
// of the kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace taser_scan {
namespace {

constexpr int kThreads = 256;
constexpr int kWave = 64;
constexpr int kWaves = kThreads / kWave;
constexpr int kScanItems = 16;
constexpr int kScanChunk = kThreads * kScanItems;

// Exclusive scan of one value per thread across the block; returns the prefix
// and leaves the block total in *total (valid for all threads).
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t x, uint32_t* total) {
    __shared__ uint32_t wave_sum[kWaves];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    uint32_t inc = x;
    for (int d = 1; d < kWave; d <<= 1) {
        const uint32_t y = __shfl_up(inc, d, kWave);
        if (lane >= d) inc += y;
    }
    __syncthreads();                      // wave_sum may still be read from a previous call
    if (lane == kWave - 1) wave_sum[wave] = inc;
    __syncthreads();
    uint32_t before = 0, all = 0;
    for (int w = 0; w < kWaves; ++w) {
        const uint32_t s = wave_sum[w];
        if (w < wave) before += s;
        all += s;
    }
    *total = all;
    return before + inc - x;
}

__global__ __launch_bounds__(kThreads) void scan_reduce_kernel(const uint32_t* __restrict__ a, int64_t n,
                                                               uint32_t* __restrict__ partial) {
    const int64_t base = (int64_t)blockIdx.x * kScanChunk + (int64_t)threadIdx.x * kScanItems;
    uint32_t s = 0;
    for (int j = 0; j < kScanItems; ++j)
        if (base + j < n) s += a[base + j];
    uint32_t total;
    block_exclusive_scan(s, &total);
    if (threadIdx.x == 0) partial[blockIdx.x] = total;
}

// One block: partial[] becomes its own exclusive scan.
__global__ __launch_bounds__(kThreads) void scan_partials_kernel(uint32_t* partial, int64_t count) {
    uint32_t carry = 0;
    for (int64_t base = 0; base < count; base += kThreads) {
        const int64_t i = base + threadIdx.x;
        const uint32_t x = i < count ? partial[i] : 0;
        uint32_t total;
        const uint32_t ex = block_exclusive_scan(x, &total);
        if (i < count) partial[i] = carry + ex;
        carry += total;
    }
}

__global__ __launch_bounds__(kThreads) void scan_apply_kernel(uint32_t* __restrict__ a, int64_t n,
                                                              const uint32_t* __restrict__ partial) {
    const int64_t base = (int64_t)blockIdx.x * kScanChunk + (int64_t)threadIdx.x * kScanItems;
    uint32_t v[kScanItems];
    uint32_t s = 0;
    for (int j = 0; j < kScanItems; ++j) {
        v[j] = base + j < n ? a[base + j] : 0;
        s += v[j];
    }
    uint32_t total;
    uint32_t run = partial[blockIdx.x] + block_exclusive_scan(s, &total);
    for (int j = 0; j < kScanItems; ++j) {
        if (base + j < n) a[base + j] = run;
        run += v[j];
    }
}

// Number of uint32 partial sums `exclusive_scan_u32` needs as scratch for n elements.
inline unsigned num_partials(int64_t n) { return (unsigned)((n + kScanChunk - 1) / kScanChunk); }

inline void exclusive_scan_u32(uint32_t* a, int64_t n, uint32_t* partial, hipStream_t stream) {
    if (n <= 0) return;
    const unsigned blocks = num_partials(n);
    hipLaunchKernelGGL(scan_reduce_kernel, dim3(blocks), dim3(kThreads), 0, stream, a, n, partial);
    hipLaunchKernelGGL(scan_partials_kernel, dim3(1), dim3(kThreads), 0, stream, partial, (int64_t)blocks);
    hipLaunchKernelGGL(scan_apply_kernel, dim3(blocks), dim3(kThreads), 0, stream, a, n, partial);
}

}  // namespace
}  // namespace taser_scan
