// Internal declarations shared by the HIP translation units of libtaser.
// Not part of the ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "taser.h"

// Records an error for taser_last_error() and returns `code`.
int taser_fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
int taser_fail_hip(hipError_t e, const char* what);

// hipGetLastError() reports the last error of ANY earlier HIP call of this
// thread, including other libraries' probes that were expected to fail. Entry
// points that check their kernel launches with it call this first.
inline void taser_clear_stale_hip_error() { (void)hipGetLastError(); }

#define TASER_HIP_TRY(expr)                                    \
    do {                                                       \
        hipError_t taser_e_ = (expr);                          \
        if (taser_e_ != hipSuccess) return taser_fail_hip(taser_e_, #expr); \
    } while (0)

// One T-CSR entry as the sampler reads it: a single 16-byte load per sample.
struct __attribute__((aligned(16))) TaserRec {
    int64_t ts;
    int32_t nbr;
    int32_t eid;
};

struct taser_tcsr {
    int64_t num_entries;
    int32_t num_nodes;
    int64_t* indptr;   // device int64[num_nodes + 1]
    TaserRec* rec;     // device TaserRec[num_entries], T-CSR order
};

static constexpr int kWave = 64;

// Host-side launcher of the dense row gather shared by taser_gather_features
// and the cache (defined in gather.hip). Pointers are device-visible.
int taser_launch_gather(const void* table, int64_t rows, int32_t row_bytes, int64_t pitch_bytes,
                        const int32_t* ids, int64_t n, void* out, hipStream_t stream);

// Brackets the kernel launches made during its lifetime with a pair of events
// on `stream` while a taser_profile_begin/_end session is active; otherwise
// it does nothing. `name` must have static storage.
class TaserProfileSpan {
public:
    TaserProfileSpan(hipStream_t stream, const char* name);
    ~TaserProfileSpan();
    TaserProfileSpan(const TaserProfileSpan&) = delete;
    TaserProfileSpan& operator=(const TaserProfileSpan&) = delete;

private:
    hipStream_t stream_;
    long index_;
};
