// Device cache of hot feature rows over a table in pinned host memory
// (TASER, arXiv 2402.05396, Sec. 3.4 and Alg. 3: a fixed budget of rows lives
// in device memory with a cache line of one row; other rows are read from host
// memory over the bus without an intermediate copy).
//
// Layout in device memory: `capacity` rows packed at a 4-byte-rounded pitch; an
// open-addressing hash table id -> slot (linear probing, power-of-two size
// >= 2 * capacity); and a per-call staging area so that a row which misses is
// pulled over PCIe once per call however many requests name it (with skewed
// access a hot non-resident row is otherwise re-read hundreds of times per
// batch over a bus 100x slower than HBM).
//
// A lookup is three kernels (1-2 = taser_cache_prefetch, 3 = taser_cache_gather;
// split so that a caller can run the bus-bound part beside other work):
//   1. classify: every request probes the resident hash; a miss claims a slot
//      of the miss table (compare-and-swap on the id) — the outcome per request
//      is written to `loc`;
//   2. stage: the claimed slots get consecutive rows of the staging area (so
//      that what a call staged is one dense block of memory), a wave per slot
//      copies that row host -> staging and empties the slot, so the miss table
//      is clear again for the next call; a third small kernel rewrites the
//      locations of the missed requests from table slot to staging row;
//   3. gather: the dense output is written from cache rows / staged rows /
//      zero rows, or straight from host memory for requests that found the
//      miss table or the staging area full.
// Which rows are resident only changes where bytes come from, never the bytes.
#include <cstdio>
#include <mutex>
#include <new>
#include <vector>

#include "gather_kernel.h"
#include "scan_kernels.h"
#include "taser_internal.h"

namespace {

constexpr int kThreads = 256;
constexpr int32_t kEmpty = -1;
constexpr int32_t kLocZero = -1;                   // request with a negative id
constexpr int32_t kLocHost = INT32_MIN;            // read the host row directly
constexpr int kMaxMissProbes = 128;
constexpr int kTallySlots = 1024;                 // per-block LDS table of the access counting
constexpr uint32_t kTagCache = 0x43414348u;        // hop tag of the residency shuffle
constexpr int kClassifyBlocks = 2048;             // grid-stride: 8 blocks per compute unit
constexpr int32_t kHotBit = 1 << 30;               // in a cache-slot location: a row that drew a large share of the
                                                   // last epoch's requests (see mark_hot_kernel)
constexpr int32_t kSlotMask = kHotBit - 1;
constexpr uint64_t kHotShare = 4096;               // hot = at least 1/4096 of all counted requests

__host__ __device__ inline uint32_t hash_id(int32_t id, uint32_t mask) {
    uint32_t h = (uint32_t)id * 0x9E3779B1u;
    h ^= h >> 15;
    return h & mask;
}
// loc encoding: >= 0 cache slot (| kHotBit); kLocZero; kLocHost; otherwise -2 - s, where s is a slot of the
// miss table between classify and resolve, a row of the staging area afterwards
__host__ __device__ inline int32_t loc_of_stage(uint32_t s) { return -2 - (int32_t)s; }

}  // namespace

struct taser_cache {
    int64_t rows;
    int32_t row_bytes;
    int64_t pitch_bytes;        // of the host table
    int64_t capacity;
    const uint8_t* host_rows;   // device-visible address of the pinned host table
    int32_t dev_pitch;          // pitch of cache_rows / stage_rows
    uint8_t* cache_rows;        // device [capacity][dev_pitch]
    int32_t* hash_key;          // device [hash_size], kEmpty or a resident id
    int32_t* hash_slot;         // device [hash_size]
    uint32_t hash_mask;
    uint8_t* stage_rows;        // device [staging_rows][dev_pitch]
    int64_t staging_rows;
    int32_t* miss_key;          // device [miss_size], all kEmpty between lookups
    int32_t* miss_row;          // device [miss_size]: staging row of a claimed slot (-1: the staging area was full)
    uint32_t* stage_count;      // device [1]: staging rows handed out by the running call, 0 between calls
    uint32_t miss_size;         // 0 or a power of two >= 2 * staging_rows
    int32_t* loc;               // device [loc_capacity], per-request outcome
    int64_t loc_capacity;
    const int32_t* prefetched_ids;   // what `loc` currently describes (set by taser_cache_prefetch)
    int64_t prefetched_n;
    int stage_blocks;                // width of the host -> staging copy, in 256-thread blocks
    bool refresh_before_gather;      // see rewrite_kernel
    int partitioned_gather;          // gather through gather_owned_lines_kernel where it applies (0 off, 1 on, 2: owners by position only, for measurements)
    std::vector<int32_t>* residents;   // host copy, slot order
    int32_t* resident_dev;             // device copy of the same
    uint32_t* access_count;            // device [rows] or null: requests per row since the last epoch end
    bool counting;
    uint32_t* block_tally;             // device [2 * kClassifyBlocks]: hits, misses of every classify block
    // scratch of the epoch-end selection, allocated together with access_count
    uint32_t *epoch_hist, *epoch_rank, *epoch_pos, *epoch_partial;   // [256], [rows], [rows], [num_partials(rows)]
    int32_t* epoch_selected;                                         // [capacity]
    unsigned long long* epoch_overlap;                               // [2]
};

namespace {

__global__ __launch_bounds__(kThreads) void fill_kernel(int32_t* a, uint32_t n, int32_t v) {
    const uint32_t i = blockIdx.x * kThreads + threadIdx.x;
    if (i < n) a[i] = v;
}

// Grid-stride over the requests; hit/miss counts are summed per block and left in
// block_tally for tally_kernel (even one atomic pair per block on the caller's two
// counters, thousands on one address, took longer than the classification itself).
__global__ __launch_bounds__(kThreads) void classify_kernel(
    const int32_t* __restrict__ ids, int64_t n, int64_t rows, const int32_t* __restrict__ hash_key,
    const int32_t* __restrict__ hash_slot, uint32_t hash_mask, int32_t* miss_key, uint32_t miss_size,
    int32_t* __restrict__ loc, uint32_t* __restrict__ block_tally, uint32_t* access_count) {
    __shared__ uint32_t block_hits[kThreads / kWave], block_misses[kThreads / kWave];
    // Access counting: a block first sums its own requests per id in a small LDS
    // hash table and adds each distinct id to the global counter once, so a row
    // that a tenth of all requests name costs one global atomic per block.
    __shared__ int32_t tally_key[kTallySlots];
    __shared__ uint32_t tally_count[kTallySlots];
    if (access_count) {
        for (int s = threadIdx.x; s < kTallySlots; s += kThreads) {
            tally_key[s] = kEmpty;
            tally_count[s] = 0;
        }
        __syncthreads();
    }
    uint32_t hits = 0, misses = 0;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += (int64_t)gridDim.x * kThreads) {
        const int32_t id = ids[i];
        int32_t where = kLocZero;
        if (id >= 0 && id < rows) {
            if (access_count) {
                uint32_t s = hash_id(id, kTallySlots - 1);
                bool done = false;
                for (int probe = 0; probe < 8 && !done; ++probe) {
                    int32_t key = tally_key[s];
                    if (key == kEmpty) key = atomicCAS(&tally_key[s], kEmpty, id);
                    if (key == kEmpty || key == id) {
                        atomicAdd(&tally_count[s], 1u);
                        done = true;
                    }
                    s = (s + 1) & (kTallySlots - 1);
                }
                if (!done) atomicAdd(&access_count[id], 1u);   // table crowded: count directly
            }
            uint32_t h = hash_id(id, hash_mask);
            int32_t slot = -1;
            for (;;) {                               // the table is never full: the loop ends at an empty key
                const int32_t key = hash_key[h];
                if (key == id) { slot = hash_slot[h]; break; }
                if (key == kEmpty) break;
                h = (h + 1) & hash_mask;
            }
            if (slot >= 0) {
                ++hits;
                where = slot;
            } else {
                ++misses;
                where = kLocHost;
                if (miss_size) {
                    uint32_t s = hash_id(id, miss_size - 1);
                    for (int probe = 0; probe < kMaxMissProbes; ++probe) {
                        int32_t key = miss_key[s];
                        if (key == kEmpty) key = atomicCAS(&miss_key[s], kEmpty, id);
                        if (key == kEmpty || key == id) { where = loc_of_stage(s); break; }
                        s = (s + 1) & (miss_size - 1);
                    }
                }
            }
        }
        loc[i] = where;
    }
    if (access_count) {
        __syncthreads();
        for (int s = threadIdx.x; s < kTallySlots; s += kThreads)
            if (tally_key[s] != kEmpty) atomicAdd(&access_count[tally_key[s]], tally_count[s]);
    }
    if (!block_tally) return;
    for (int d = kWave / 2; d > 0; d >>= 1) {
        hits += __shfl_down(hits, d, kWave);
        misses += __shfl_down(misses, d, kWave);
    }
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    if (lane == 0) {
        block_hits[wave] = hits;
        block_misses[wave] = misses;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t h = 0, m = 0;
        for (int w = 0; w < kThreads / kWave; ++w) {
            h += block_hits[w];
            m += block_misses[w];
        }
        block_tally[2 * blockIdx.x] = h;
        block_tally[2 * blockIdx.x + 1] = m;
    }
}

// One block: adds the per-block counts of the classify launch before it to the
// caller's two counters.
__global__ __launch_bounds__(kThreads) void tally_kernel(const uint32_t* __restrict__ block_tally, int blocks,
                                                         unsigned long long* hit_miss) {
    __shared__ unsigned long long part[2][kThreads / kWave];
    unsigned long long h = 0, m = 0;
    for (int b = threadIdx.x; b < blocks; b += kThreads) {
        h += block_tally[2 * b];
        m += block_tally[2 * b + 1];
    }
    for (int d = kWave / 2; d > 0; d >>= 1) {
        h += __shfl_down(h, d, kWave);
        m += __shfl_down(m, d, kWave);
    }
    if ((threadIdx.x & (kWave - 1)) == 0) {
        part[0][threadIdx.x >> 6] = h;
        part[1][threadIdx.x >> 6] = m;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        h = m = 0;
        for (int w = 0; w < kThreads / kWave; ++w) {
            h += part[0][w];
            m += part[1][w];
        }
        if (h) atomicAdd(&hit_miss[0], h);
        if (m) atomicAdd(&hit_miss[1], m);
    }
}

// Copies every claimed row host -> staging. The copy is bound by the bus, not by
// the GPU, so it runs on a few hundred waves only (each keeps a whole row, up to
// 2 KiB, in flight) and leaves the compute units to whatever runs beside it:
// a wave reads 64 table slots at a time and walks the claimed ones.
constexpr int kStageBlocks = 64;

__global__ __launch_bounds__(kThreads) void stage_kernel(int32_t* __restrict__ miss_key, int32_t* __restrict__ miss_row,
                                                         uint32_t miss_size, uint32_t* stage_count, uint32_t staging_rows,
                                                         const uint8_t* __restrict__ host_rows, int64_t pitch_bytes,
                                                         uint32_t row_dwords, uint8_t* __restrict__ stage_rows,
                                                         int32_t dev_pitch) {
    using taser_gather::Chunk16;
    const uint32_t lane = threadIdx.x & (kWave - 1);
    const uint32_t wave = blockIdx.x * (kThreads / kWave) + (threadIdx.x >> 6);
    const uint32_t num_waves = gridDim.x * (kThreads / kWave);
    const uint32_t chunks = row_dwords / 4u, tail = row_dwords & 3u;
    for (uint32_t base = wave * kWave; base < miss_size; base += num_waves * kWave) {   // miss_size % 64 == 0
        const int32_t key = miss_key[base + lane];
        if (key >= 0) miss_key[base + lane] = kEmpty;   // the table is empty again for the next call's claims
        uint64_t claimed = __ballot(key >= 0);
        if (!claimed) continue;
        // consecutive staging rows for this wave's claimed slots: one atomic per 64 slots
        uint32_t first = 0;
        if (lane == 0) first = atomicAdd(stage_count, (uint32_t)__popcll(claimed));
        first = __builtin_amdgcn_readfirstlane(first);
        const uint32_t my_row = first + (uint32_t)__popcll(claimed & (((uint64_t)1 << lane) - 1));
        if (key >= 0) miss_row[base + lane] = my_row < staging_rows ? (int32_t)my_row : -1;
        while (claimed) {
            const int l = __ffsll((long long)claimed) - 1;
            claimed &= claimed - 1;
            const uint32_t row = __builtin_amdgcn_readlane(my_row, l);
            if (row >= staging_rows) break;             // later lanes have later rows: nothing more fits
            const int32_t id = __builtin_amdgcn_readlane(key, l);
            const uint8_t* from = host_rows + (int64_t)id * pitch_bytes;
            uint8_t* to = stage_rows + (int64_t)row * dev_pitch;
            // 16-byte pieces (4-byte aligned on both sides), two per lane in flight
            for (uint32_t c = lane; c < chunks; c += 2 * kWave) {
                const uint32_t c2 = c + kWave;
                const Chunk16 a = reinterpret_cast<const Chunk16*>(from)[c];
                Chunk16 b = a;
                if (c2 < chunks) b = reinterpret_cast<const Chunk16*>(from)[c2];
                reinterpret_cast<Chunk16*>(to)[c] = a;
                if (c2 < chunks) reinterpret_cast<Chunk16*>(to)[c2] = b;
            }
            if (lane < tail)
                reinterpret_cast<uint32_t*>(to)[chunks * 4u + lane] = reinterpret_cast<const uint32_t*>(from)[chunks * 4u + lane];
        }
    }
}

// After the staging: the location of a missed request changes from its miss-table slot to the
// staging row that slot was given (or to "read host memory" when the staging area was full),
// and the row counter goes back to zero for the next call.
__global__ __launch_bounds__(kThreads) void resolve_kernel(int32_t* __restrict__ loc, int64_t n,
                                                           const int32_t* __restrict__ miss_row, uint32_t* stage_count) {
    if (blockIdx.x == 0 && threadIdx.x == 0) *stage_count = 0;   // the stage kernel before this one has finished
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += (int64_t)gridDim.x * kThreads) {
        const int32_t where = loc[i];
        if (where < kLocZero && where != kLocHost) {
            const int32_t row = miss_row[-2 - where];
            loc[i] = row >= 0 ? loc_of_stage((uint32_t)row) : kLocHost;
        }
    }
}

// Re-writes up to three arrays of 32-bit words in place with the bytes they
// already hold (`zero` is 0; it only keeps the stores from being optimised
// away). Why: measured on MI355X, the memory-side cache keeps lines that were
// recently written but does not take lines back in on read misses. When other
// streaming work ran between the staging and the gather, the gather's small
// read working set (locations, resident rows, staged rows) has been evicted,
// every L2 miss then goes to HBM, and the gather runs 1.4x slower. Touching
// the working set (tens of MB) costs a few tens of microseconds.
struct RewriteJob {
    uint32_t* words[3];
    int64_t count[3];
};

__global__ __launch_bounds__(kThreads) void rewrite_kernel(RewriteJob job, uint32_t zero) {
    using taser_gather::u32x4;
    constexpr int kPer = 4;   // 16-byte pieces per thread and round: their loads are issued together
    for (int a = 0; a < 3; ++a) {
        u32x4* quads = reinterpret_cast<u32x4*>(job.words[a]);   // bases are allocation starts: 16-byte aligned
        const int64_t nq = job.count[a] / 4;
        for (int64_t i0 = (int64_t)blockIdx.x * (kThreads * kPer) + threadIdx.x; i0 < nq; i0 += (int64_t)gridDim.x * (kThreads * kPer)) {
            u32x4 v[kPer];
#pragma unroll
            for (int u = 0; u < kPer; ++u) {
                const int64_t i = i0 + u * kThreads;
                v[u] = quads[i < nq ? i : nq - 1];
            }
#pragma unroll
            for (int u = 0; u < kPer; ++u) {
                const int64_t i = i0 + u * kThreads;
                v[u].x ^= zero;
                if (i < nq) quads[i] = v[u];
            }
        }
        const int64_t t = nq * 4 + (int64_t)blockIdx.x * kThreads + threadIdx.x;
        if (t < job.count[a]) job.words[a][t] ^= zero;
    }
}

struct CacheSource {
    const int32_t* loc;
    const int32_t* ids;
    const uint8_t* cache_rows;
    const uint8_t* stage_rows;
    int32_t dev_pitch;
    const uint8_t* host_rows;
    int64_t pitch_bytes;
    int owner_mode;   // 1: by source row; 2: by position only
    __device__ __forceinline__ int32_t key(int64_t i) const { return loc[i]; }
    __device__ __forceinline__ const uint8_t* address(int32_t where, int64_t i) const {
        // cache row or staged row: one multiply-add either way, no branch
        const bool cached = where >= 0;
        const uint8_t* at = (cached ? cache_rows : stage_rows) + (int64_t)(cached ? (where & kSlotMask) : -2 - where) * dev_pitch;
        if (where == kLocZero) at = nullptr;
        if (__builtin_expect(where == kLocHost, 0)) at = host_rows + (int64_t)ids[i] * pitch_bytes;
        return at;
    }
    // Which L2 partition serves request i (see gather_owned_lines_kernel): chosen by the source row,
    // so that a row is read through one partition only; by the request's position for zero rows,
    // rows read from host memory and hot rows (a handful of rows that a large part of all requests
    // name: they stay in every partition's L2 anyway, and tying each to one partition would give
    // that partition several times the others' work).
    __device__ __forceinline__ uint32_t owner(int32_t where, int64_t i) const {
        uint32_t v = (uint32_t)i;
        if (owner_mode == 2) return v % taser_gather::kOwnerClasses;
        if (where >= 0 && !(where & kHotBit)) v = ((uint32_t)where * 0x9E3779B1u) >> 20;
        else if (where < kLocZero && where != kLocHost) v = ((uint32_t)(-2 - where) * 0x9E3779B1u) >> 19;
        return v % taser_gather::kOwnerClasses;
    }
};

// ---- epoch-end maintenance (Alg. 3): the `capacity` most requested rows -----
// Histogram of one byte of the counts, over the rows whose higher bytes equal
// `prefix` (radix select, most significant byte first).
__global__ __launch_bounds__(kThreads) void count_digit_hist_kernel(const uint32_t* __restrict__ count, int64_t rows,
                                                                    int shift, uint32_t prefix, uint32_t* hist) {
    __shared__ uint32_t bins[256];
    bins[threadIdx.x] = 0;
    __syncthreads();
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < rows; i += (int64_t)gridDim.x * kThreads) {
        const uint32_t v = count[i];
        if (shift == 24 || (v >> (shift + 8)) == prefix) atomicAdd(&bins[(v >> shift) & 255u], 1u);
    }
    __syncthreads();
    if (bins[threadIdx.x]) atomicAdd(&hist[threadIdx.x], bins[threadIdx.x]);
}

// flag[i] = 1 where the predicate holds (MODE 0: count == t; MODE 1: count > t,
// or count == t and fewer than `ties` equal rows precede row i).
template <int MODE>
__global__ __launch_bounds__(kThreads) void flag_rows_kernel(const uint32_t* __restrict__ count, int64_t rows, uint32_t t,
                                                             const uint32_t* __restrict__ tie_rank, uint32_t ties,
                                                             uint32_t* __restrict__ flag) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= rows) return;
    const uint32_t v = count[i];
    if (MODE == 0) flag[i] = v == t;
    else flag[i] = (v > t) || (v == t && tie_rank[i] < ties);
}

// Writes the selected ids in ascending order (position = exclusive scan of the
// flags) and counts how many of them are resident already.
__global__ __launch_bounds__(kThreads) void emit_selected_kernel(const uint32_t* __restrict__ count, int64_t rows, uint32_t t,
                                                                 const uint32_t* __restrict__ tie_rank, uint32_t ties,
                                                                 const uint32_t* __restrict__ position,
                                                                 const int32_t* __restrict__ hash_key, uint32_t hash_mask,
                                                                 int32_t* __restrict__ selected, unsigned long long* overlap) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    bool resident = false;
    if (i < rows) {
        const uint32_t v = count[i];
        if ((v > t) || (v == t && tie_rank[i] < ties)) {
            selected[position[i]] = (int32_t)i;
            uint32_t h = hash_id((int32_t)i, hash_mask);
            for (;;) {
                const int32_t key = hash_key[h];
                if (key == (int32_t)i) { resident = true; break; }
                if (key == kEmpty) break;
                h = (h + 1) & hash_mask;
            }
        }
    }
    const unsigned long long both = __ballot(resident);
    if ((threadIdx.x & (kWave - 1)) == 0 && both) atomicAdd(overlap, (unsigned long long)__popcll(both));
}

// Sum of all access counters, added to *total.
__global__ __launch_bounds__(kThreads) void sum_counts_kernel(const uint32_t* __restrict__ count, int64_t rows,
                                                              unsigned long long* total) {
    unsigned long long s = 0;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < rows; i += (int64_t)gridDim.x * kThreads) s += count[i];
    for (int d = kWave / 2; d > 0; d >>= 1) s += __shfl_down(s, d, kWave);
    if ((threadIdx.x & (kWave - 1)) == 0 && s) atomicAdd(total, s);
}

// Marks, in the id -> slot index, the resident rows that drew at least 1/kHotShare of the epoch's
// counted requests (at most kHotShare rows can). Only the gather's choice of which L2 partition
// serves a request looks at the mark.
__global__ __launch_bounds__(kThreads) void mark_hot_kernel(const int32_t* __restrict__ hash_key, int32_t* __restrict__ hash_slot,
                                                            uint32_t hash_size, const uint32_t* __restrict__ count,
                                                            const unsigned long long* __restrict__ total, unsigned long long share) {
    const uint32_t h = blockIdx.x * kThreads + threadIdx.x;
    if (h >= hash_size) return;
    const int32_t id = hash_key[h];
    if (id == kEmpty) return;
    const unsigned long long all = *total;
    const bool hot = all > 0 && (unsigned long long)count[id] * share >= all;
    hash_slot[h] = (hash_slot[h] & kSlotMask) | (hot ? kHotBit : 0);
}

// Philox4x32-10 on the host, for the default residency draw only.
uint64_t host_draw64(uint64_t seed, uint32_t hop, uint64_t root, uint32_t slot) {
    uint32_t c[4] = {(uint32_t)root, (uint32_t)(root >> 32), slot, hop};
    uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c[0], p1 = (uint64_t)0xCD9E8D57u * c[2];
        const uint32_t a = (uint32_t)(p1 >> 32) ^ c[1] ^ k0, b = (uint32_t)(p0 >> 32) ^ c[3] ^ k1;
        c[0] = a; c[1] = (uint32_t)p1; c[2] = b; c[3] = (uint32_t)p0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return ((uint64_t)c[1] << 32) | c[0];
}

uint32_t pow2_at_least(uint64_t x) {
    uint32_t p = 1;
    while (p < x) p <<= 1;
    return p;
}

void destroy(taser_cache* c) {
    if (!c) return;
    void* const owned[] = {c->cache_rows, c->hash_key, c->hash_slot, c->stage_rows, c->miss_key, c->miss_row, c->stage_count,
                           c->loc, c->resident_dev, c->access_count, c->block_tally, c->epoch_hist, c->epoch_rank,
                           c->epoch_pos, c->epoch_partial, c->epoch_selected, c->epoch_overlap};
    int at = 0;
    for (void* p : owned) {
        const hipError_t e = p ? hipFree(p) : hipSuccess;
        if (e != hipSuccess) fprintf(stderr, "taser: cache free: buffer %d (%p): %s\n", at, p, hipGetErrorString(e));
        ++at;
    }
    (void)hipGetLastError();   // a failed free must not poison the caller's next HIP call
    delete c->residents;
    delete c;
}

// Makes `*c->residents` (slot order) the cache content: builds the id -> slot hash
// on the host, uploads it, and fills the cache rows by a gather straight out of
// host memory. Synchronizes the stream.
int install_residents(taser_cache* c, hipStream_t stream) {
    const std::vector<int32_t>& res = *c->residents;
    const uint32_t hash_size = c->hash_mask + 1;
    std::vector<int32_t> h_key, h_slot;
    try {
        h_key.assign(hash_size, kEmpty);
        h_slot.assign(hash_size, -1);
    } catch (const std::bad_alloc&) {
        return taser_fail(TASER_E_OOM, "cache: host allocation failed");
    }
    for (int64_t s = 0; s < c->capacity; ++s) {
        uint32_t h = hash_id(res[(size_t)s], c->hash_mask);
        while (h_key[h] != kEmpty) h = (h + 1) & c->hash_mask;
        h_key[h] = res[(size_t)s];
        h_slot[h] = (int32_t)s;
    }
    TASER_HIP_TRY(hipMemcpyAsync(c->hash_key, h_key.data(), (size_t)hash_size * sizeof(int32_t), hipMemcpyHostToDevice, stream));
    TASER_HIP_TRY(hipMemcpyAsync(c->hash_slot, h_slot.data(), (size_t)hash_size * sizeof(int32_t), hipMemcpyHostToDevice, stream));
    if (c->capacity > 0) {
        TASER_HIP_TRY(hipMemcpyAsync(c->resident_dev, res.data(), (size_t)c->capacity * sizeof(int32_t), hipMemcpyHostToDevice, stream));
        const int rc = taser_launch_gather(c->host_rows, c->rows, c->row_bytes, c->pitch_bytes, c->resident_dev, c->capacity,
                                           c->cache_rows, stream);
        if (rc != TASER_OK) return rc;
    }
    TASER_HIP_TRY(hipStreamSynchronize(stream));   // the host vectors above must outlive the copies
    return TASER_OK;
}

}  // namespace

// ---- lookup that allocates nothing ---------------------------------------------
// Per-request locations and per-block hit/miss counts of taser_cache_lookup_static live
// in this array instead of the handle's growable buffers. Every GPU holds its own copy;
// host code reaches it only through the address looked up once per device below.
constexpr int64_t kStaticRequests = TASER_STATIC_LOOKUP_MAX_REQUESTS;
static __device__ __align__(256) int32_t scratch[kStaticRequests + 2 * kClassifyBlocks];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
int32_t* g_scratch_ptr[kMaxDevices] = {};   // device address of `scratch` on each GPU, null until looked up

// Address of `scratch` on the current device (looked up the first time, with that device current).
int scratch_on_current_device(int32_t** out) {
    int dev = -1;
    TASER_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return taser_fail(TASER_E_RANGE, "cache: device ordinal %d outside [0, %d)", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        TASER_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return taser_fail(TASER_E_HIP, "cache: the lookup scratch has no address on device %d", dev);
        g_scratch_ptr[dev] = static_cast<int32_t*>(p);
    }
    *out = g_scratch_ptr[dev];
    return TASER_OK;
}

}  // namespace

extern "C" int taser_cache_init(const void* host_table, int64_t rows, int32_t row_bytes, int64_t pitch_bytes,
                                int64_t capacity_rows, const int32_t* resident_ids, uint64_t seed,
                                int64_t staging_rows, void* hip_stream, taser_cache** out) {
    if (!out) return taser_fail(TASER_E_ARG, "cache_init: null out");
    *out = nullptr;
    if (!host_table) return taser_fail(TASER_E_ARG, "cache_init: null host table");
    if (rows < 1 || rows >= 0x7fffffffLL) return taser_fail(TASER_E_RANGE, "cache_init: rows = %lld outside [1, 2^31 - 1)", (long long)rows);
    if (row_bytes <= 0 || (row_bytes & 3)) return taser_fail(TASER_E_ARG, "cache_init: row_bytes = %d must be a positive multiple of 4", row_bytes);
    if (pitch_bytes < row_bytes || (pitch_bytes & 3)) return taser_fail(TASER_E_ARG, "cache_init: pitch_bytes = %lld must be a multiple of 4 and >= row_bytes", (long long)pitch_bytes);
    if (capacity_rows < 0 || capacity_rows > rows) return taser_fail(TASER_E_RANGE, "cache_init: capacity_rows = %lld outside [0, rows]", (long long)capacity_rows);
    if (capacity_rows >= kHotBit) return taser_fail(TASER_E_RANGE, "cache_init: capacity_rows = %lld must stay below 2^30", (long long)capacity_rows);
    if (staging_rows < 0 || staging_rows > ((int64_t)1 << 29)) return taser_fail(TASER_E_RANGE, "cache_init: staging_rows = %lld outside [0, 2^29]", (long long)staging_rows);
    if ((uintptr_t)host_table & 3) return taser_fail(TASER_E_ARG, "cache_init: host table must be 4-byte aligned");

    hipPointerAttribute_t attr;
    hipError_t pe = hipPointerGetAttributes(&attr, host_table);
    if (pe != hipSuccess || attr.type != hipMemoryTypeHost || !attr.devicePointer) {
        (void)hipGetLastError();   // the query leaves a sticky error for ordinary host memory
        return taser_fail(TASER_E_ARG, "cache_init: host table is not page-locked, device-mapped host memory");
    }
    hipStream_t stream = (hipStream_t)hip_stream;
    taser_resolve_device_constants();
    {
        int32_t* unused = nullptr;   // the allocation-free lookup's scratch gets its address on this device now
        const int rc = scratch_on_current_device(&unused);
        if (rc != TASER_OK) return rc;
    }

    taser_cache* c = new (std::nothrow) taser_cache();
    if (!c) return taser_fail(TASER_E_OOM, "cache_init: host allocation failed");
    *c = taser_cache{};
    c->rows = rows;
    c->row_bytes = row_bytes;
    c->pitch_bytes = pitch_bytes;
    c->capacity = capacity_rows;
    c->host_rows = static_cast<const uint8_t*>(attr.devicePointer);
    c->dev_pitch = row_bytes;
    c->stage_blocks = kStageBlocks;
    c->refresh_before_gather = false;
    c->partitioned_gather = 1;
    c->residents = new (std::nothrow) std::vector<int32_t>();
    if (!c->residents) { destroy(c); return taser_fail(TASER_E_OOM, "cache_init: host allocation failed"); }

    // ---- resident ids
    std::vector<int32_t>& res = *c->residents;
    try {
        res.resize((size_t)capacity_rows);
        if (resident_ids) {
            std::vector<uint8_t> seen((size_t)rows, 0);
            for (int64_t i = 0; i < capacity_rows; ++i) {
                const int32_t id = resident_ids[i];
                if (id < 0 || id >= rows || seen[(size_t)id]) {
                    destroy(c);
                    return taser_fail(TASER_E_RANGE, "cache_init: resident_ids[%lld] = %d is out of range or repeated", (long long)i, id);
                }
                seen[(size_t)id] = 1;
                res[(size_t)i] = id;
            }
        } else {
            // partial Fisher-Yates over 0..rows-1; `moved` holds the displaced values
            std::vector<int32_t> a((size_t)rows);
            for (int64_t i = 0; i < rows; ++i) a[(size_t)i] = (int32_t)i;
            for (int64_t j = 0; j < capacity_rows; ++j) {
                const uint64_t u = host_draw64(seed, kTagCache, (uint64_t)j, 0u);
                const int64_t r = j + (int64_t)(((unsigned __int128)u * (uint64_t)(rows - j)) >> 64);
                const int32_t t = a[(size_t)r];
                a[(size_t)r] = a[(size_t)j];
                a[(size_t)j] = t;
                res[(size_t)j] = t;
            }
        }
    } catch (const std::bad_alloc&) {
        destroy(c);
        return taser_fail(TASER_E_OOM, "cache_init: host allocation failed");
    }

    const uint32_t hash_size = pow2_at_least((uint64_t)(capacity_rows > 8 ? capacity_rows : 8) * 2);
    c->hash_mask = hash_size - 1;
    c->staging_rows = staging_rows;
    c->miss_size = staging_rows > 0 ? pow2_at_least((uint64_t)(staging_rows > 32 ? staging_rows : 32) * 2) : 0;   // >= 64

#define CACHE_TRY(expr)                                               \
    do {                                                              \
        hipError_t e_ = (expr);                                       \
        if (e_ != hipSuccess) { destroy(c); return taser_fail_hip(e_, #expr); } \
    } while (0)
    CACHE_TRY(hipMalloc((void**)&c->cache_rows, (size_t)(capacity_rows > 0 ? capacity_rows : 1) * c->dev_pitch));
    CACHE_TRY(hipMalloc((void**)&c->hash_key, (size_t)hash_size * sizeof(int32_t)));
    CACHE_TRY(hipMalloc((void**)&c->hash_slot, (size_t)hash_size * sizeof(int32_t)));
    CACHE_TRY(hipMalloc((void**)&c->resident_dev, (size_t)(capacity_rows > 0 ? capacity_rows : 1) * sizeof(int32_t)));
    CACHE_TRY(hipMalloc((void**)&c->block_tally, (size_t)2 * kClassifyBlocks * sizeof(uint32_t)));
    if (c->miss_size) {
        CACHE_TRY(hipMalloc((void**)&c->stage_rows, (size_t)staging_rows * c->dev_pitch));
        CACHE_TRY(hipMalloc((void**)&c->miss_key, (size_t)c->miss_size * sizeof(int32_t)));
        CACHE_TRY(hipMalloc((void**)&c->miss_row, (size_t)c->miss_size * sizeof(int32_t)));
        CACHE_TRY(hipMalloc((void**)&c->stage_count, sizeof(uint32_t)));
        hipLaunchKernelGGL(fill_kernel, dim3((c->miss_size + kThreads - 1) / kThreads), dim3(kThreads), 0, stream,
                           c->miss_key, c->miss_size, kEmpty);
        hipLaunchKernelGGL(fill_kernel, dim3(1), dim3(kThreads), 0, stream, reinterpret_cast<int32_t*>(c->stage_count), 1u, 0);
    }
#undef CACHE_TRY
    const int rc = install_residents(c, stream);
    if (rc != TASER_OK) { destroy(c); return rc; }
    *out = c;
    return TASER_OK;
}

// The kernels of the first half of a lookup: classify into `loc` (block counts into `tally`), stage the misses.
static int enqueue_prefetch(taser_cache* c, const int32_t* ids, int64_t n, uint64_t* hit_miss, hipStream_t stream,
                            int32_t* loc, uint32_t* tally) {
    int64_t blocks = (n + kThreads - 1) / kThreads;
    if (blocks > kClassifyBlocks) blocks = kClassifyBlocks;
    // miss_key is all-empty here: cache_init cleared it and every stage_kernel clears what it consumed
    {
        TaserProfileSpan span(stream, "cache_classify");
        hipLaunchKernelGGL(classify_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, stream, ids, n, c->rows,
                           c->hash_key, c->hash_slot, c->hash_mask, c->miss_key, c->miss_size, loc,
                           hit_miss ? tally : nullptr, c->counting ? c->access_count : nullptr);
        if (hit_miss)
            hipLaunchKernelGGL(tally_kernel, dim3(1), dim3(kThreads), 0, stream, tally, (int)blocks,
                               reinterpret_cast<unsigned long long*>(hit_miss));
    }
    if (c->miss_size) {
        TaserProfileSpan span(stream, "cache_stage_misses");
        hipLaunchKernelGGL(stage_kernel, dim3(c->stage_blocks), dim3(kThreads), 0, stream, c->miss_key, c->miss_row,
                           c->miss_size, c->stage_count, (uint32_t)c->staging_rows, c->host_rows, c->pitch_bytes,
                           (uint32_t)c->row_bytes / 4u, c->stage_rows, c->dev_pitch);
        hipLaunchKernelGGL(resolve_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, stream, loc, n, c->miss_row, c->stage_count);
    }
    TASER_HIP_TRY(hipGetLastError());
    return TASER_OK;
}

// The second half: the dense output from the locations in `loc`.
static int enqueue_gather(taser_cache* c, const int32_t* ids, int64_t n, void* out, hipStream_t stream, int32_t* loc) {
    const CacheSource source{loc, ids, c->cache_rows, c->stage_rows, c->dev_pitch, c->host_rows, c->pitch_bytes, c->partitioned_gather};
    const int align = taser_gather::common_alignment((uint64_t)c->row_bytes | (uint64_t)c->pitch_bytes |
                                                     (uint64_t)(uintptr_t)c->host_rows);
    if (c->refresh_before_gather) {
        RewriteJob job;
        job.words[0] = reinterpret_cast<uint32_t*>(loc);
        job.count[0] = n;
        job.words[1] = reinterpret_cast<uint32_t*>(c->cache_rows);
        job.count[1] = c->capacity * (int64_t)c->dev_pitch / 4;
        job.words[2] = reinterpret_cast<uint32_t*>(c->stage_rows);
        job.count[2] = c->miss_size ? c->staging_rows * (int64_t)c->dev_pitch / 4 : 0;
        TaserProfileSpan span(stream, "cache_refresh_working_set");
        hipLaunchKernelGGL(rewrite_kernel, dim3(2048), dim3(kThreads), 0, stream, job, 0u);
    }
    TaserProfileSpan span(stream, "cache_gather_rows");
    const bool launched = c->partitioned_gather ? taser_gather::launch_owned(source, align, c->row_bytes, n, out, stream)
                                                : taser_gather::launch(source, align, c->row_bytes, n, out, stream);
    if (!launched)
        return taser_fail(TASER_E_RANGE, "cache_gather: %lld rows of %d bytes exceed one launch", (long long)n, c->row_bytes);
    TASER_HIP_TRY(hipGetLastError());
    return TASER_OK;
}

extern "C" int taser_cache_prefetch(taser_cache* c, const int32_t* ids, int64_t n, uint64_t* hit_miss,
                                    void* hip_stream) {
    if (!c) return taser_fail(TASER_E_ARG, "cache_prefetch: null cache");
    if (n < 0) return taser_fail(TASER_E_ARG, "cache_prefetch: n = %lld", (long long)n);
    c->prefetched_ids = nullptr;
    c->prefetched_n = 0;
    if (n == 0) return TASER_OK;
    if (!ids) return taser_fail(TASER_E_ARG, "cache_prefetch: null ids");
    taser_clear_stale_hip_error();
    hipStream_t stream = (hipStream_t)hip_stream;
    if (n > c->loc_capacity) {
        // grows only; the old buffer may still be read by a gather on any stream
        TASER_HIP_TRY(hipDeviceSynchronize());
        (void)hipFree(c->loc);
        c->loc = nullptr;
        c->loc_capacity = 0;
        TASER_HIP_TRY(hipMalloc((void**)&c->loc, (size_t)n * sizeof(int32_t)));
        c->loc_capacity = n;
    }
    const int rc = enqueue_prefetch(c, ids, n, hit_miss, stream, c->loc, c->block_tally);
    if (rc != TASER_OK) return rc;
    c->prefetched_ids = ids;
    c->prefetched_n = n;
    return TASER_OK;
}

extern "C" int taser_cache_gather(taser_cache* c, const int32_t* ids, int64_t n, void* out, void* hip_stream) {
    if (!c) return taser_fail(TASER_E_ARG, "cache_gather: null cache");
    if (n < 0) return taser_fail(TASER_E_ARG, "cache_gather: n = %lld", (long long)n);
    if (ids != c->prefetched_ids || n != c->prefetched_n)
        return taser_fail(TASER_E_ARG, "cache_gather: not preceded by taser_cache_prefetch of the same ids and n");
    if (n == 0) return TASER_OK;
    if (!out) return taser_fail(TASER_E_ARG, "cache_gather: null out");
    if ((uintptr_t)out & 3) return taser_fail(TASER_E_ARG, "cache_gather: out must be 4-byte aligned");
    taser_clear_stale_hip_error();
    return enqueue_gather(c, ids, n, out, (hipStream_t)hip_stream, c->loc);
}

extern "C" int taser_cache_lookup(taser_cache* c, const int32_t* ids, int64_t n, void* out, uint64_t* hit_miss,
                                  void* hip_stream) {
    if (!c) return taser_fail(TASER_E_ARG, "cache_lookup: null cache");
    if (n < 0) return taser_fail(TASER_E_ARG, "cache_lookup: n = %lld", (long long)n);
    if (n == 0) return TASER_OK;
    if (!ids || !out) return taser_fail(TASER_E_ARG, "cache_lookup: null ids or out");
    if ((uintptr_t)out & 3) return taser_fail(TASER_E_ARG, "cache_lookup: out must be 4-byte aligned");
    const int rc = taser_cache_prefetch(c, ids, n, hit_miss, hip_stream);
    if (rc != TASER_OK) return rc;
    return taser_cache_gather(c, ids, n, out, hip_stream);
}

extern "C" int taser_cache_lookup_static(taser_cache* c, const int32_t* ids, int64_t n, void* out, uint64_t* hit_miss,
                                         void* hip_stream) {
    if (!c) return taser_fail(TASER_E_ARG, "cache_lookup_static: null cache");
    if (n < 0) return taser_fail(TASER_E_ARG, "cache_lookup_static: n = %lld", (long long)n);
    if (n > kStaticRequests)
        return taser_fail(TASER_E_RANGE, "cache_lookup_static: n = %lld exceeds the %lld requests its fixed scratch holds",
                          (long long)n, (long long)kStaticRequests);
    if (n == 0) return TASER_OK;
    if (!ids || !out) return taser_fail(TASER_E_ARG, "cache_lookup_static: null ids or out");
    if ((uintptr_t)out & 3) return taser_fail(TASER_E_ARG, "cache_lookup_static: out must be 4-byte aligned");
    taser_clear_stale_hip_error();
    int32_t* base = nullptr;
    int rc = scratch_on_current_device(&base);
    if (rc != TASER_OK) return rc;
    int32_t* loc = base;                                                     // [n]: written before it is read
    uint32_t* tally = reinterpret_cast<uint32_t*>(base + kStaticRequests);   // [2 * blocks]: likewise
    c->prefetched_ids = nullptr;   // the handle's miss table and staging rows are reused: a pending prefetch is void
    c->prefetched_n = 0;
    hipStream_t stream = (hipStream_t)hip_stream;
    rc = enqueue_prefetch(c, ids, n, hit_miss, stream, loc, tally);
    if (rc != TASER_OK) return rc;
    return enqueue_gather(c, ids, n, out, stream, loc);
}

extern "C" int taser_cache_count_accesses(taser_cache* c, int32_t enable, void* hip_stream) {
    if (!c) return taser_fail(TASER_E_ARG, "cache_count_accesses: null cache");
    taser_clear_stale_hip_error();
    hipStream_t stream = (hipStream_t)hip_stream;
    if (enable && !c->access_count) {
        // the counters and everything the epoch-end selection needs, once (access_count last: it
        // marks the set as complete; a buffer that a failed earlier attempt left behind is kept)
#define CACHE_NEED(member, bytes) \
    if (!c->member) TASER_HIP_TRY(hipMalloc((void**)&c->member, (size_t)(bytes)))
        CACHE_NEED(epoch_hist, 256 * sizeof(uint32_t));
        CACHE_NEED(epoch_rank, c->rows * sizeof(uint32_t));
        CACHE_NEED(epoch_pos, c->rows * sizeof(uint32_t));
        CACHE_NEED(epoch_partial, taser_scan::num_partials(c->rows) * sizeof(uint32_t));
        CACHE_NEED(epoch_selected, (c->capacity > 0 ? c->capacity : 1) * sizeof(int32_t));
        CACHE_NEED(epoch_overlap, 2 * sizeof(unsigned long long));
#undef CACHE_NEED
        TASER_HIP_TRY(hipMalloc((void**)&c->access_count, (size_t)c->rows * sizeof(uint32_t)));
        hipLaunchKernelGGL(fill_kernel, dim3((unsigned)((c->rows + kThreads - 1) / kThreads)), dim3(kThreads), 0, stream,
                           reinterpret_cast<int32_t*>(c->access_count), (uint32_t)c->rows, 0);
        TASER_HIP_TRY(hipGetLastError());
    }
    c->counting = enable != 0;
    return TASER_OK;
}

extern "C" int taser_cache_access_counts(const taser_cache* c, uint32_t* counts, void* hip_stream) {
    if (!c || !counts) return taser_fail(TASER_E_ARG, "cache_access_counts: null argument");
    if (!c->access_count) return taser_fail(TASER_E_ARG, "cache_access_counts: counting was never enabled");
    TASER_HIP_TRY(hipMemcpyAsync(counts, c->access_count, (size_t)c->rows * sizeof(uint32_t), hipMemcpyDeviceToDevice,
                                 (hipStream_t)hip_stream));
    return TASER_OK;
}

extern "C" int taser_cache_epoch_end(taser_cache* c, int64_t min_overlap, int64_t* overlap, int32_t* replaced,
                                     void* hip_stream) {
    if (!c) return taser_fail(TASER_E_ARG, "cache_epoch_end: null cache");
    if (!c->access_count) return taser_fail(TASER_E_ARG, "cache_epoch_end: counting was never enabled");
    taser_clear_stale_hip_error();
    hipStream_t stream = (hipStream_t)hip_stream;
    const int64_t rows = c->rows, k = c->capacity;
    const unsigned row_blocks = (unsigned)((rows + kThreads - 1) / kThreads);
    int64_t both = k;       // with k == 0 or k == rows the top-k is what is resident
    bool replace = false;
    if (k > 0 && k < rows) {
        struct {
            uint32_t *hist, *rank, *pos, *partial;
            int32_t* selected;
            unsigned long long* overlap;
        } w = {c->epoch_hist, c->epoch_rank, c->epoch_pos, c->epoch_partial, c->epoch_selected, c->epoch_overlap};
        TaserProfileSpan span(stream, "cache_epoch_end");
        // radix select: the count t of the k-th most requested row, most significant byte first
        uint32_t prefix = 0;
        int64_t above = 0;                      // rows with a count above the prefix range chosen so far
        unsigned grid = row_blocks < 1024 ? row_blocks : 1024;
        for (int shift = 24; shift >= 0; shift -= 8) {
            uint32_t hist[256];
            hipLaunchKernelGGL(fill_kernel, dim3(1), dim3(kThreads), 0, stream, reinterpret_cast<int32_t*>(w.hist), 256u, 0);
            hipLaunchKernelGGL(count_digit_hist_kernel, dim3(grid), dim3(kThreads), 0, stream, c->access_count, rows, shift,
                               prefix, w.hist);
            TASER_HIP_TRY(hipMemcpyAsync(hist, w.hist, sizeof(hist), hipMemcpyDeviceToHost, stream));
            TASER_HIP_TRY(hipStreamSynchronize(stream));
            int bin = 255;
            while (bin > 0 && above + hist[bin] < k) above += hist[bin--];
            prefix = (prefix << 8) | (uint32_t)bin;
        }
        const uint32_t t = prefix;              // `above` rows have a larger count
        const uint32_t ties = (uint32_t)(k - above);   // rows with count == t that still fit, smallest ids first
        hipLaunchKernelGGL(flag_rows_kernel<0>, dim3(row_blocks), dim3(kThreads), 0, stream, c->access_count, rows, t,
                           (const uint32_t*)nullptr, 0u, w.rank);
        taser_scan::exclusive_scan_u32(w.rank, rows, w.partial, stream);
        hipLaunchKernelGGL(flag_rows_kernel<1>, dim3(row_blocks), dim3(kThreads), 0, stream, c->access_count, rows, t,
                           (const uint32_t*)w.rank, ties, w.pos);
        taser_scan::exclusive_scan_u32(w.pos, rows, w.partial, stream);
        hipLaunchKernelGGL(fill_kernel, dim3(1), dim3(kThreads), 0, stream, reinterpret_cast<int32_t*>(w.overlap), 2u, 0);
        hipLaunchKernelGGL(emit_selected_kernel, dim3(row_blocks), dim3(kThreads), 0, stream, c->access_count, rows, t,
                           (const uint32_t*)w.rank, ties, (const uint32_t*)w.pos, c->hash_key, c->hash_mask, w.selected,
                           w.overlap);
        TASER_HIP_TRY(hipGetLastError());
        unsigned long long h_both = 0;
        TASER_HIP_TRY(hipMemcpyAsync(&h_both, w.overlap, sizeof(h_both), hipMemcpyDeviceToHost, stream));
        TASER_HIP_TRY(hipStreamSynchronize(stream));
        both = (int64_t)h_both;
        replace = both < min_overlap;
        if (replace) {
            TASER_HIP_TRY(hipMemcpy(c->residents->data(), w.selected, (size_t)k * sizeof(int32_t), hipMemcpyDeviceToHost));
            const int rc = install_residents(c, stream);
            if (rc != TASER_OK) return rc;
            c->prefetched_ids = nullptr;        // locations computed before the swap are stale
            c->prefetched_n = 0;
        }
    }
    // which of the (new) residents were hot this epoch, then the counters start again
    hipLaunchKernelGGL(fill_kernel, dim3(1), dim3(kThreads), 0, stream, reinterpret_cast<int32_t*>(c->epoch_overlap), 4u, 0);
    hipLaunchKernelGGL(sum_counts_kernel, dim3(row_blocks < 256 ? row_blocks : 256), dim3(kThreads), 0, stream, c->access_count,
                       rows, c->epoch_overlap + 1);
    hipLaunchKernelGGL(mark_hot_kernel, dim3((c->hash_mask + kThreads) / kThreads), dim3(kThreads), 0, stream, c->hash_key,
                       c->hash_slot, c->hash_mask + 1, c->access_count, c->epoch_overlap + 1, (unsigned long long)kHotShare);
    hipLaunchKernelGGL(fill_kernel, dim3(row_blocks), dim3(kThreads), 0, stream, reinterpret_cast<int32_t*>(c->access_count),
                       (uint32_t)rows, 0);
    TASER_HIP_TRY(hipGetLastError());
    TASER_HIP_TRY(hipStreamSynchronize(stream));
    if (overlap) *overlap = both;
    if (replaced) *replaced = replace ? 1 : 0;
    return TASER_OK;
}

extern "C" int taser_cache_tune(taser_cache* c, int32_t stage_blocks, int32_t refresh_before_gather,
                                int32_t partitioned_gather) {
    if (!c) return taser_fail(TASER_E_ARG, "cache_tune: null cache");
    if (stage_blocks < 0 || stage_blocks > 4096) return taser_fail(TASER_E_RANGE, "cache_tune: stage_blocks = %d outside [0, 4096]", stage_blocks);
    if (stage_blocks > 0) c->stage_blocks = stage_blocks;
    c->refresh_before_gather = refresh_before_gather != 0;
    if (partitioned_gather >= 0) c->partitioned_gather = partitioned_gather > 2 ? 1 : partitioned_gather;
    return TASER_OK;
}

extern "C" int taser_cache_residents(const taser_cache* c, int32_t* resident_ids_host) {
    if (!c || (!resident_ids_host && c->capacity > 0)) return taser_fail(TASER_E_ARG, "cache_residents: null argument");
    for (int64_t i = 0; i < c->capacity; ++i) resident_ids_host[i] = (*c->residents)[(size_t)i];
    return TASER_OK;
}

extern "C" void taser_cache_free(taser_cache* c) { destroy(c); }
