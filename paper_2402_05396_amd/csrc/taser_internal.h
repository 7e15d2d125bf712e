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

// Search index over the timestamps of the whole record array (all lists back to
// back): level l = 1..kTimeIndexLevels holds, for every run of 16^l consecutive
// records, the timestamp of the run's last record (of the array's last record for
// the final, partial run). A search for a query time inside one node's list reads
// one 128-byte line of 16 neighboring entries per level instead of 16 scattered
// records; the upper levels are small enough to stay in L2.
constexpr int kTimeIndexLevels = 7;   // 16^7 = 2^28: at the top a list of < 2^31 records spans < 16 entries
struct TaserTimeIndex {
    const int64_t* level[kTimeIndexLevels];   // level[l - 1]: device int64[len[l - 1]]
    int64_t len[kTimeIndexLevels];            // ceil(num_entries / 16^l)
    int64_t num_entries;
};

struct taser_tcsr {
    int64_t num_entries;
    int32_t num_nodes;
    int64_t* indptr;   // device int64[num_nodes + 1]
    TaserRec* rec;     // device TaserRec[num_entries], T-CSR order
    int64_t* time_index_storage;   // one device allocation behind time_index.level[*]
    TaserTimeIndex time_index;
    int64_t* ts_only;              // device int64[num_entries] or null: the timestamps alone, made on first use by
                                   // the one finder that reads whole lists (inverse timespan)
};

static constexpr int kWave = 64;

// Host-side launcher of the dense row gather shared by taser_gather_features
// and the cache (defined in gather.hip). Pointers are device-visible.
int taser_launch_gather(const void* table, int64_t rows, int32_t row_bytes, int64_t pitch_bytes,
                        const int32_t* ids, int64_t n, void* out, hipStream_t stream);

// Looks up, for the current device, the addresses of the library's device constants
// (a symbol lookup the first time; nothing afterwards). Handle-making entry points call
// it so that later gathers on the device only launch kernels.
void taser_resolve_device_constants();

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
