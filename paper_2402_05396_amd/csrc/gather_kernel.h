// Dense row gather: out row i <- the bytes of a source row chosen per i.
//
// The output is treated as one flat stream of V-wide elements (V = 16, 8, 4 or
// 2 bytes, the widest the row size, pitch and base addresses allow). Thread
// g of the launch produces output element g, so every wave instruction stores
// 64 consecutive elements (fully coalesced, whatever the row length) and loads
// runs of consecutive elements from at most a few source rows. Where a row
// comes from is a functor, so the same kernel serves a table in device memory
// and the cache's three-way choice (cache rows / staged rows / host memory).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace taser_gather {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

template <typename V> __device__ __forceinline__ V zero_of() { return V(0); }
template <> __device__ __forceinline__ u32x4 zero_of<u32x4>() { return u32x4{0, 0, 0, 0}; }
template <> __device__ __forceinline__ u32x2 zero_of<u32x2>() { return u32x2{0, 0}; }

constexpr int kThreads = 256;
constexpr int kUnroll = 4;
constexpr int kTile = kThreads * kUnroll;   // output elements per block

// Source::row(i) returns the address of the first byte of the row that output
// row i copies, or nullptr for a row of zeros.
template <typename V, typename Source>
__global__ __launch_bounds__(kThreads) void gather_kernel(Source source, uint32_t row_elems,
                                                          int64_t total_elems, V* __restrict__ out) {
    const int64_t tile = (int64_t)blockIdx.x * kTile;
    // first output row touched by this block and the column of its first element
    int64_t row0;
    if (tile < ((int64_t)1 << 32)) row0 = (uint32_t)tile / row_elems;
    else row0 = tile / (int64_t)row_elems;
    const uint32_t col0 = (uint32_t)(tile - row0 * row_elems);

    V vals[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
        const uint32_t e = col0 + threadIdx.x + u * kThreads;   // offset from the start of row0
        const uint32_t dr = e / row_elems;
        const uint32_t col = e - dr * row_elems;
        const int64_t g = tile + threadIdx.x + u * kThreads;
        vals[u] = zero_of<V>();
        if (g < total_elems) {
            const uint8_t* base = source.row(row0 + dr);
            if (base) vals[u] = reinterpret_cast<const V*>(base)[col];
        }
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
        const int64_t g = tile + threadIdx.x + u * kThreads;
        if (g < total_elems) __builtin_nontemporal_store(vals[u], out + g);
    }
}

// Largest power-of-two width (16, 8, 4, 2 or 1) dividing everything given.
inline int common_alignment(uint64_t bits) {
    if ((bits & 15) == 0) return 16;
    if ((bits & 7) == 0) return 8;
    if ((bits & 3) == 0) return 4;
    if ((bits & 1) == 0) return 2;
    return 1;
}

template <typename V, typename Source>
inline void launch_typed(const Source& source, int32_t row_bytes, int64_t n, void* out, hipStream_t stream) {
    const uint32_t row_elems = (uint32_t)(row_bytes / (int)sizeof(V));
    const int64_t total = n * (int64_t)row_elems;
    const int64_t blocks = (total + kTile - 1) / kTile;
    hipLaunchKernelGGL((gather_kernel<V, Source>), dim3((unsigned)blocks), dim3(kThreads), 0, stream, source,
                       row_elems, total, reinterpret_cast<V*>(out));
}

// Dispatch on the vector width `align` (from common_alignment). Returns false if
// the launch would need more blocks than a grid dimension holds.
template <typename Source>
inline bool launch(const Source& source, int align, int32_t row_bytes, int64_t n, void* out, hipStream_t stream) {
    if (n == 0) return true;
    const int64_t total = n * (int64_t)(row_bytes / align);
    if ((total + kTile - 1) / kTile > 0x7fffffffLL) return false;
    switch (align) {
        case 16: launch_typed<u32x4>(source, row_bytes, n, out, stream); break;
        case 8: launch_typed<u32x2>(source, row_bytes, n, out, stream); break;
        case 4: launch_typed<uint32_t>(source, row_bytes, n, out, stream); break;
        default: launch_typed<uint16_t>(source, row_bytes, n, out, stream); break;
    }
    return true;
}

}  // namespace taser_gather
