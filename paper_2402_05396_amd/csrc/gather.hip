// taser_gather_features: feature slicing from a table in device memory
// (TASER, arXiv 2402.05396, Sec. 3.4 / Alg. 3: serve the feature row of every
// requested id). A pure byte mover, bounded by HBM bandwidth.
#include "gather_kernel.h"
#include "taser_internal.h"

namespace {

struct TableSource {
    const uint8_t* table;
    int64_t pitch_bytes;
    const int32_t* ids;
    int64_t rows;
    __device__ __forceinline__ int32_t key(int64_t i) const { return ids[i]; }
    __device__ __forceinline__ const uint8_t* address(int32_t id, int64_t) const {
        const bool ok = id >= 0 && id < rows;
        const uint8_t* at = table + (int64_t)(ok ? id : 0) * pitch_bytes;   // computed either way: no branch
        return ok ? at : nullptr;
    }
};

}  // namespace

// 16 zero bytes in device memory. External linkage and "used": a device variable
// that no kernel names is otherwise dropped from the code object, and looking it
// up by symbol then fails inside the runtime.
__device__ __attribute__((used)) uint32_t taser_zero_chunk_storage[4] = {0u, 0u, 0u, 0u};

const uint8_t* taser_gather::zero_chunk() {
    // per device: every GPU holds its own copy of the symbol
    static const uint8_t* cached[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
    if (!cached[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(taser_zero_chunk_storage)) != hipSuccess) return nullptr;
        cached[dev] = static_cast<const uint8_t*>(p);
    }
    return cached[dev];
}

void taser_resolve_device_constants() { (void)taser_gather::zero_chunk(); }

int taser_launch_gather(const void* table, int64_t rows, int32_t row_bytes, int64_t pitch_bytes, const int32_t* ids,
                        int64_t n, void* out, hipStream_t stream) {
    taser_clear_stale_hip_error();
    const int align = taser_gather::common_alignment((uint64_t)row_bytes | (uint64_t)pitch_bytes |
                                                     (uint64_t)(uintptr_t)table);
    const TableSource source{static_cast<const uint8_t*>(table), pitch_bytes, ids, rows};
    TaserProfileSpan span(stream, "gather_rows");
    if (!taser_gather::launch(source, align, row_bytes, n, out, stream))
        return taser_fail(TASER_E_RANGE, "gather: %lld rows of %d bytes exceed one launch", (long long)n, row_bytes);
    TASER_HIP_TRY(hipGetLastError());
    return TASER_OK;
}

extern "C" int taser_gather_features(const void* table, int64_t rows, int32_t row_bytes,
                                     int64_t pitch_bytes, const int32_t* ids, int64_t n, void* out,
                                     void* hip_stream) {
    if (n < 0 || rows < 0) return taser_fail(TASER_E_ARG, "gather_features: negative size");
    if (row_bytes <= 0 || (row_bytes & 1)) return taser_fail(TASER_E_ARG, "gather_features: row_bytes = %d must be positive and even", row_bytes);
    if (pitch_bytes < row_bytes || (pitch_bytes & 1)) return taser_fail(TASER_E_ARG, "gather_features: pitch_bytes = %lld must be even and >= row_bytes", (long long)pitch_bytes);
    if (n == 0) return TASER_OK;
    if (!ids || !out) return taser_fail(TASER_E_ARG, "gather_features: null ids or out");
    if (!table && rows > 0) return taser_fail(TASER_E_ARG, "gather_features: null table");
    if (((uintptr_t)out & 1) || ((uintptr_t)table & 1)) return taser_fail(TASER_E_ARG, "gather_features: table and out must be 2-byte aligned");
    return taser_launch_gather(table, rows, row_bytes, pitch_bytes, ids, n, out, (hipStream_t)hip_stream);
}
