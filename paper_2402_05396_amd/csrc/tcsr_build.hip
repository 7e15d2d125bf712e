// taser_tcsr_build: the T-CSR of TASER (arXiv 2402.05396, Sec. 3.3): every
// node's outgoing entries contiguous and ordered by timestamp, ties by input
// position. Built on the device by a stable least-significant-digit radix
// sort over the composite key (node, ts):
//   * digits of the timestamp first (only those bytes in which the timestamps
//     actually differ, and none at all when the input is already time-sorted,
//     which is how event streams arrive), then the digits of the node id;
//   * one pass = per-block digit histogram -> exclusive scan over the
//     (digit, block) counters -> stable scatter. Inside a block the stable rank
//     of an item among equal digits comes from wave ballots (which lanes hold
//     my digit, how many of them are below me) plus per-wave running counters
//     in LDS, so no atomics decide an output position;
//   * the 16-byte record {ts, nbr, eid} the sampler reads travels with the key,
//     so the last pass leaves the final layout in place;
//   * indptr is read off the sorted node column (no atomics, no histogram).
#include <new>
#include <vector>

#include "scan_kernels.h"
#include "taser_internal.h"

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr int kItems = 16;                         // items per thread
constexpr int kTile = kThreads * kItems;           // items per block
constexpr int kBins = 256;                         // 8-bit digits

struct DigitSpec {
    int from_ts;      // 1: digit of the (sign-biased) timestamp, 0: digit of the node id
    int shift;
    uint32_t mask;
};

__device__ __forceinline__ uint64_t biased(int64_t ts) { return (uint64_t)ts ^ 0x8000000000000000ull; }

__device__ __forceinline__ uint32_t digit_at(const TaserRec* rec, const int32_t* key, int64_t i, DigitSpec d) {
    if (d.from_ts) return (uint32_t)(biased(rec[i].ts) >> d.shift) & d.mask;
    return ((uint32_t)key[i] >> d.shift) & d.mask;
}

// Item r of lane `lane` of wave `wave` inside a tile: rows of 64 consecutive
// items per wave, so loads are coalesced and index order = (wave, row, lane).
__device__ __forceinline__ int64_t item_index(int64_t tile0, int wave, int r, int lane) {
    return tile0 + (int64_t)wave * (kWave * kItems) + r * kWave + lane;
}

// Packs the input columns into the 16-byte records + node key the sort moves, and
// inspects them on the way. Per block, partial[4 * block + ...]: [0] != 0: a node id
// outside [0, num_nodes); [1] != 0: timestamps not non-decreasing in input order;
// [2] / [3]: OR / AND of the biased timestamps (bytes in which they agree need no
// sorting pass). fold_info_kernel combines the per-block words (atomics from every
// block onto four shared words took longer than reading the input).
// The block also counts its tile's node ids by their lowest digit, hist[bin * num_blocks +
// tile] as radix_hist_kernel would: time-sorted input (the usual case) is sorted by the node
// digits only, lowest first, and that pass then needs no histogram kernel of its own (the
// counting hides behind this kernel's memory traffic).
__global__ __launch_bounds__(kThreads) void pack_inspect_kernel(const int32_t* __restrict__ src,
                                                                const int32_t* __restrict__ dst,
                                                                const int64_t* __restrict__ ts,
                                                                const int32_t* __restrict__ eid, int64_t n,
                                                                int32_t num_nodes, TaserRec* __restrict__ rec,
                                                                int32_t* __restrict__ key,
                                                                unsigned long long* __restrict__ partial,
                                                                uint32_t low_digit_mask, uint32_t* __restrict__ hist,
                                                                uint32_t num_blocks) {
    __shared__ uint32_t bins[kBins];
    bins[threadIdx.x] = 0;
    __syncthreads();
    unsigned long long any_or = 0, all_and = ~0ull;
    int bad = 0, unsorted = 0;
    constexpr int kPer = 4;   // entries per thread and round: their loads are issued together
    // a block packs one contiguous tile of kTile entries
    const int64_t tile0 = (int64_t)blockIdx.x * kTile;
    for (int round = 0; round < kItems / kPer; ++round) {
        const int64_t i0 = tile0 + (int64_t)round * (kPer * kThreads) + threadIdx.x;
        int32_t s[kPer], dn[kPer], e[kPer];
        int64_t t[kPer], t_next[kPer];
#pragma unroll
        for (int u = 0; u < kPer; ++u) {
            const int64_t i = i0 + u * kThreads;
            const int64_t at = i < n ? i : n - 1;            // clamped: every load stays in bounds
            s[u] = src[at];
            dn[u] = dst[at];
            t[u] = ts[at];
            t_next[u] = ts[at + 1 < n ? at + 1 : at];
            e[u] = eid ? eid[at] : (int32_t)at;
        }
#pragma unroll
        for (int u = 0; u < kPer; ++u) {
            const int64_t i = i0 + u * kThreads;
            if (i >= n) continue;
            bad |= (s[u] < 0 || s[u] >= num_nodes);
            unsorted |= (t_next[u] < t[u]);
            any_or |= biased(t[u]);
            all_and &= biased(t[u]);
            TaserRec r;
            r.ts = t[u];
            r.nbr = dn[u];
            r.eid = e[u];
            rec[i] = r;
            key[i] = s[u];
            atomicAdd(&bins[(uint32_t)s[u] & low_digit_mask], 1u);
        }
    }
    for (int d = 1; d < kWave; d <<= 1) {
        any_or |= __shfl_xor(any_or, d, kWave);
        all_and &= __shfl_xor(all_and, d, kWave);
    }
    __shared__ unsigned long long w_or[kWaves], w_and[kWaves];
    __shared__ int w_bad[kWaves], w_unsorted[kWaves];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    const unsigned long long any_bad = __ballot(bad), any_unsorted = __ballot(unsorted);
    if (lane == 0) {
        w_or[wave] = any_or;
        w_and[wave] = all_and;
        w_bad[wave] = any_bad != 0;
        w_unsorted[wave] = any_unsorted != 0;
    }
    __syncthreads();
    if (hist) hist[(size_t)threadIdx.x * num_blocks + blockIdx.x] = bins[threadIdx.x];
    if (threadIdx.x == 0) {
        unsigned long long o = 0, a = ~0ull;
        int b = 0, u = 0;
        for (int w = 0; w < kWaves; ++w) {
            o |= w_or[w];
            a &= w_and[w];
            b |= w_bad[w];
            u |= w_unsorted[w];
        }
        partial[4 * blockIdx.x + 0] = (unsigned long long)b;
        partial[4 * blockIdx.x + 1] = (unsigned long long)u;
        partial[4 * blockIdx.x + 2] = o;
        partial[4 * blockIdx.x + 3] = a;
    }
}

// info[4 * block + 0..3] = this block's share of the `blocks` per-block word groups of
// pack_inspect_kernel combined (launched twice: many blocks, then one over their results).
__global__ __launch_bounds__(kThreads) void fold_info_kernel(const unsigned long long* __restrict__ partial, uint32_t blocks,
                                                             unsigned long long* __restrict__ info) {
    __shared__ unsigned long long part[4][kThreads];
    unsigned long long v[4] = {0, 0, 0, ~0ull};
    for (uint32_t b = blockIdx.x * kThreads + threadIdx.x; b < blocks; b += gridDim.x * kThreads) {
        v[0] |= partial[4 * (size_t)b + 0];
        v[1] |= partial[4 * (size_t)b + 1];
        v[2] |= partial[4 * (size_t)b + 2];
        v[3] &= partial[4 * (size_t)b + 3];
    }
    for (int j = 0; j < 4; ++j) part[j][threadIdx.x] = v[j];
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int t = 1; t < kThreads; ++t) {
            v[0] |= part[0][t];
            v[1] |= part[1][t];
            v[2] |= part[2][t];
            v[3] &= part[3][t];
        }
        for (int j = 0; j < 4; ++j) info[4 * blockIdx.x + j] = v[j];
    }
}

// Tile of a workgroup of the scatter: workgroups go to the chip's eight L2 partitions round-robin;
// each partition takes a contiguous eighth of the tiles, so that the short runs of one digit that
// its workgroups write one after the other into neighboring addresses (16 records per tile on
// average for 256 digits) meet in its L2 and leave as whole lines. With tile = workgroup index
// those pieces came from eight different L2s as partial lines (5.8 -> 3.6 ms for the 256-digit
// pass over 382 M entries). The grid is rounded up to a multiple of kPartitions; tiles >=
// num_blocks do not exist.
constexpr uint32_t kPartitions = 8;
__device__ __forceinline__ uint32_t tile_of_block(uint32_t block, uint32_t num_blocks) {
    const uint32_t per_part = (num_blocks + kPartitions - 1) / kPartitions;
    return (block % kPartitions) * per_part + block / kPartitions;
}
inline unsigned pass_grid(unsigned num_blocks) { return (num_blocks + kPartitions - 1) / kPartitions * kPartitions; }

// hist[bin * num_blocks + tile] = items of the tile whose digit is bin.
__global__ __launch_bounds__(kThreads) void radix_hist_kernel(const TaserRec* __restrict__ rec,
                                                              const int32_t* __restrict__ key, int64_t n,
                                                              DigitSpec d, uint32_t* __restrict__ hist,
                                                              uint32_t num_blocks) {
    __shared__ uint32_t bins[kBins];
    const uint32_t tile = blockIdx.x;   // (the partition-wise order of the scatter below does not pay here)
    bins[threadIdx.x] = 0;
    __syncthreads();
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    const int64_t tile0 = (int64_t)tile * kTile;
    if (!d.from_ts && tile0 + kTile <= n) {
        // a whole tile of node keys: which thread counts which item does not matter, so every thread
        // takes four runs of four keys with 16-byte loads (tile0 is a multiple of the tile size and
        // `key` the start of an allocation: aligned), all four loads in flight together
        typedef int32_t i32x4 __attribute__((ext_vector_type(4)));
        const i32x4* quads = reinterpret_cast<const i32x4*>(key + tile0);
        i32x4 v[kItems / 4];
#pragma unroll
        for (int r = 0; r < kItems / 4; ++r) v[r] = quads[r * kThreads + threadIdx.x];
#pragma unroll
        for (int r = 0; r < kItems / 4; ++r) {
            atomicAdd(&bins[((uint32_t)v[r].x >> d.shift) & d.mask], 1u);
            atomicAdd(&bins[((uint32_t)v[r].y >> d.shift) & d.mask], 1u);
            atomicAdd(&bins[((uint32_t)v[r].z >> d.shift) & d.mask], 1u);
            atomicAdd(&bins[((uint32_t)v[r].w >> d.shift) & d.mask], 1u);
        }
    } else {
#pragma unroll 4
        for (int r = 0; r < kItems; ++r) {
            const int64_t i = item_index(tile0, wave, r, lane);
            if (i < n) atomicAdd(&bins[digit_at(rec, key, i, d)], 1u);
        }
    }
    __syncthreads();
    hist[(size_t)threadIdx.x * num_blocks + tile] = bins[threadIdx.x];
}

// Stable scatter of one tile. offs = the scanned histogram: offs[bin*num_blocks
// + block] is where this block's first item with digit `bin` goes. The tile is
// first put in digit order in LDS (stable: rank among equal digits = ballots
// inside a row of 64 + running per-wave counters + the waves before), then
// written out in that order, so that consecutive lanes write consecutive
// addresses of one digit's run instead of 64 scattered records. The ordered tile
// passes through LDS in kParts slices (every item knows its place in the order;
// a slice takes the items whose place falls into it): a whole tile of records
// and keys, 80 KB, would leave room for one block per compute unit, a slice of
// half a tile for three, which is what the registers allow.
// `level1` (last pass only, else null): see the write-out.
constexpr int kParts = 2;
constexpr int kPart = kTile / kParts;
__global__ __launch_bounds__(kThreads) void radix_scatter_kernel(
    const TaserRec* __restrict__ rec_in, const int32_t* __restrict__ key_in, int64_t n, DigitSpec d,
    const uint32_t* __restrict__ offs, uint32_t num_blocks, TaserRec* __restrict__ rec_out,
    int32_t* __restrict__ key_out, int64_t* __restrict__ level1) {
    __shared__ uint32_t wave_count[kWaves][kBins];   // items of each wave per digit, then exclusive over waves
    __shared__ uint32_t block_base[kBins];           // global position of the block's first item of a digit
    __shared__ uint32_t local_base[kBins];           // position of that item inside the ordered tile
    __shared__ uint32_t scan_tmp[kWaves];
    __shared__ TaserRec tile_rec[kPart];
    __shared__ int32_t tile_key[kPart];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    const uint32_t tile = tile_of_block(blockIdx.x, num_blocks);
    if (tile >= num_blocks) return;
    const int64_t tile0 = (int64_t)tile * kTile;
    for (int w = 0; w < kWaves; ++w) wave_count[w][threadIdx.x] = 0;
    block_base[threadIdx.x] = offs[(size_t)threadIdx.x * num_blocks + tile];
    __syncthreads();

    uint32_t digit[kItems], rank[kItems];
    TaserRec item_rec[kItems];
    int32_t item_key[kItems];
    const uint64_t below = ((uint64_t)1 << lane) - 1;
#pragma unroll
    for (int r = 0; r < kItems; ++r) {
        const int64_t i = item_index(tile0, wave, r, lane);
        const bool valid = i < n;
        if (valid) {
            item_rec[r] = rec_in[i];
            item_key[r] = key_in[i];
        }
    }
#pragma unroll
    for (int r = 0; r < kItems; ++r) {
        const int64_t i = item_index(tile0, wave, r, lane);
        const bool valid = i < n;
        uint32_t dg = 0;
        if (valid) dg = d.from_ts ? (uint32_t)(biased(item_rec[r].ts) >> d.shift) & d.mask : ((uint32_t)item_key[r] >> d.shift) & d.mask;
        // lanes of this row that hold the same digit as me
        uint64_t same = __ballot(valid);
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const uint64_t has = __ballot(valid && ((dg >> b) & 1u));
            same &= ((dg >> b) & 1u) ? has : ~has;
        }
        const uint32_t before_me = (uint32_t)__popcll(same & below);
        uint32_t seen = 0;
        if (valid) seen = wave_count[wave][dg];            // equal for all lanes of a digit
        if (valid && before_me == 0) wave_count[wave][dg] = seen + (uint32_t)__popcll(same);
        digit[r] = dg;
        rank[r] = seen + before_me;
        __builtin_amdgcn_wave_barrier();   // keep the LDS counter update of row r ahead of row r+1's read
    }
    __syncthreads();
    uint32_t mine_total = 0;
    {   // per digit: exclusive prefix of the wave counts over the waves; thread b owns digit b
        uint32_t run = 0;
        for (int w = 0; w < kWaves; ++w) {
            const uint32_t c = wave_count[w][threadIdx.x];
            wave_count[w][threadIdx.x] = run;
            run += c;
        }
        mine_total = run;
    }
    {   // exclusive prefix of the digit totals over the digits = where a digit's run starts in the tile
        uint32_t inc = mine_total;
        for (int dd = 1; dd < kWave; dd <<= 1) {
            const uint32_t y = __shfl_up(inc, dd, kWave);
            if (lane >= dd) inc += y;
        }
        if (lane == kWave - 1) scan_tmp[wave] = inc;
        __syncthreads();
        uint32_t before = 0;
        for (int w = 0; w < wave; ++w) before += scan_tmp[w];
        local_base[threadIdx.x] = before + inc - mine_total;
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < kItems; ++r)   // rank becomes the item's place in the ordered tile
        if (item_index(tile0, wave, r, lane) < n) rank[r] += local_base[digit[r]] + wave_count[wave][digit[r]];
    const int64_t left = n - tile0;
    const uint32_t count = left < kTile ? (uint32_t)left : (uint32_t)kTile;   // items of this tile
    for (uint32_t part0 = 0; part0 < count; part0 += kPart) {
#pragma unroll
        for (int r = 0; r < kItems; ++r) {
            const uint32_t at = rank[r] - part0;   // wraps far beyond kPart for places before this slice
            if (item_index(tile0, wave, r, lane) < n && at < (uint32_t)kPart) {
                tile_rec[at] = item_rec[r];
                tile_key[at] = item_key[r];
            }
        }
        __syncthreads();
#pragma unroll 4
        for (int r = 0; r < kItems / kParts; ++r) {
            const uint32_t j = (uint32_t)r * kThreads + threadIdx.x;   // place inside the slice
            if (part0 + j < count) {
                const TaserRec rr = tile_rec[j];
                const int32_t kk = tile_key[j];
                const uint32_t dg = d.from_ts ? (uint32_t)(biased(rr.ts) >> d.shift) & d.mask : ((uint32_t)kk >> d.shift) & d.mask;
                const uint32_t to = block_base[dg] + (part0 + j - local_base[dg]);
                rec_out[to] = rr;
                key_out[to] = kk;
                // the last pass knows the final positions: it also leaves level 1 of the search index
                // (the timestamp of the last record of every run of 16, and of the array's last record)
                if (level1 && ((to & 15u) == 15u || (int64_t)to == n - 1)) level1[to >> 4] = rr.ts;
            }
        }
        __syncthreads();   // the slice is free again
    }
}

// indptr[v] = first position whose node id is >= v, from the sorted node column: position p starts
// the lists of the nodes in (key[p - 1], key[p]]. A thread looks at four consecutive positions (one
// 16-byte load; `key` is the start of an allocation) plus the key before them.
__global__ __launch_bounds__(kThreads) void indptr_kernel(const int32_t* __restrict__ key, int64_t n,
                                                          int32_t num_nodes, int64_t* __restrict__ indptr) {
    typedef int32_t i32x4 __attribute__((ext_vector_type(4)));
    const int64_t p0 = ((int64_t)blockIdx.x * kThreads + threadIdx.x) * 4;
    if (p0 > n) return;
    int32_t k[5];   // k[0] = the key before p0, k[1 + j] = key at p0 + j (num_nodes from position n on)
    k[0] = p0 > 0 ? key[p0 - 1] : -1;
    if (p0 + 4 <= n) {
        const i32x4 v = *reinterpret_cast<const i32x4*>(key + p0);
        k[1] = v.x; k[2] = v.y; k[3] = v.z; k[4] = v.w;
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) k[1 + j] = p0 + j < n ? key[p0 + j] : num_nodes;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        if (p0 + j > n) break;
        for (int32_t v = k[j] + 1; v <= k[1 + j]; ++v) indptr[v] = p0 + j;
    }
}

__global__ __launch_bounds__(kThreads) void unpack_kernel(const TaserRec* __restrict__ rec, int64_t n,
                                                          int32_t* __restrict__ nbr, int64_t* __restrict__ ts,
                                                          int32_t* __restrict__ eid) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= n) return;
    const TaserRec r = rec[i];
    if (nbr) nbr[i] = r.nbr;
    if (ts) ts[i] = r.ts;
    if (eid) eid[i] = r.eid;
}

// Device allocation released at scope exit unless taken over.
struct DevBuf {
    void* p = nullptr;
    ~DevBuf() { if (p) (void)hipFree(p); }
    hipError_t alloc(size_t bytes) { return hipMalloc(&p, bytes ? bytes : 1); }
    template <typename T> T* as() const { return static_cast<T*>(p); }
    template <typename T> T* release() { T* t = static_cast<T*>(p); p = nullptr; return t; }
};

inline unsigned blocks_for(int64_t n, int per_block) { return (unsigned)((n + per_block - 1) / per_block); }

// Level 1 of the search index straight from the records, every further level from the one below.
__global__ __launch_bounds__(kThreads) void time_index_first_kernel(const TaserRec* __restrict__ rec, int64_t n,
                                                                    int64_t* __restrict__ out, int64_t len) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= len) return;
    const int64_t last = 16 * (i + 1) - 1;
    out[i] = rec[last < n ? last : n - 1].ts;
}

__global__ __launch_bounds__(kThreads) void time_index_next_kernel(const int64_t* __restrict__ below, int64_t below_len,
                                                                   int64_t* __restrict__ out, int64_t len) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= len) return;
    const int64_t last = 16 * (i + 1) - 1;
    out[i] = below[last < below_len ? last : below_len - 1];
}

}  // namespace


extern "C" int taser_tcsr_build(const int32_t* src, const int32_t* dst, const int64_t* ts,
                                const int32_t* eid, int64_t num_entries, int32_t num_nodes,
                                uint32_t flags, void* hip_stream, taser_tcsr** out) {
    if (!out) return taser_fail(TASER_E_ARG, "tcsr_build: null out");
    *out = nullptr;
    if (num_entries < 0 || num_entries >= 0x7fffffffLL) return taser_fail(TASER_E_RANGE, "tcsr_build: num_entries = %lld outside [0, 2^31 - 1)", (long long)num_entries);
    if (num_nodes < 1 || num_nodes == 0x7fffffff) return taser_fail(TASER_E_RANGE, "tcsr_build: num_nodes = %d outside [1, 2^31 - 1)", num_nodes);
    if (num_entries > 0 && (!src || !dst || !ts)) return taser_fail(TASER_E_ARG, "tcsr_build: null src/dst/ts");
    if (flags & ~(uint32_t)TASER_INPUT_ON_DEVICE) return taser_fail(TASER_E_ARG, "tcsr_build: unknown flags 0x%x", flags);
    taser_clear_stale_hip_error();
    taser_resolve_device_constants();
    hipStream_t stream = (hipStream_t)hip_stream;
    const int64_t n = num_entries;

    // ---- inputs in device memory
    DevBuf in_src, in_dst, in_ts, in_eid;
    if (!(flags & TASER_INPUT_ON_DEVICE) && n > 0) {
        TASER_HIP_TRY(in_src.alloc(n * sizeof(int32_t)));
        TASER_HIP_TRY(in_dst.alloc(n * sizeof(int32_t)));
        TASER_HIP_TRY(in_ts.alloc(n * sizeof(int64_t)));
        TASER_HIP_TRY(hipMemcpyAsync(in_src.p, src, n * sizeof(int32_t), hipMemcpyHostToDevice, stream));
        TASER_HIP_TRY(hipMemcpyAsync(in_dst.p, dst, n * sizeof(int32_t), hipMemcpyHostToDevice, stream));
        TASER_HIP_TRY(hipMemcpyAsync(in_ts.p, ts, n * sizeof(int64_t), hipMemcpyHostToDevice, stream));
        src = in_src.as<int32_t>();
        dst = in_dst.as<int32_t>();
        ts = in_ts.as<int64_t>();
        if (eid) {
            TASER_HIP_TRY(in_eid.alloc(n * sizeof(int32_t)));
            TASER_HIP_TRY(hipMemcpyAsync(in_eid.p, eid, n * sizeof(int32_t), hipMemcpyHostToDevice, stream));
            eid = in_eid.as<int32_t>();
        }
    }

    // ---- pack into records, range check and sort plan in one pass over the input
    DevBuf rec_a, key_a, rec_b, key_b, hist, partial, indptr;
    TASER_HIP_TRY(rec_a.alloc(n * sizeof(TaserRec)));
    TASER_HIP_TRY(key_a.alloc(n * sizeof(int32_t)));
    unsigned long long info[4] = {0, 0, 0, ~0ull};
    int node_bits = 0;
    while (((int64_t)1 << node_bits) < (int64_t)num_nodes) ++node_bits;
    const uint32_t num_blocks = blocks_for(n, kTile);
    const int64_t hist_len = (int64_t)kBins * num_blocks;
    const uint32_t low_digit_mask = (1u << (node_bits < 8 ? node_bits : 8)) - 1u;
    if (n > 0) TASER_HIP_TRY(hist.alloc(hist_len * sizeof(uint32_t)));
    if (n > 0) {
        const unsigned grid = blocks_for(n, kTile);
        constexpr unsigned kFoldBlocks = 128;
        DevBuf d_partial, d_folded, d_info;
        TASER_HIP_TRY(d_partial.alloc((size_t)grid * 4 * sizeof(unsigned long long)));
        TASER_HIP_TRY(d_folded.alloc((size_t)kFoldBlocks * 4 * sizeof(unsigned long long)));
        TASER_HIP_TRY(d_info.alloc(sizeof(info)));
        {
            TaserProfileSpan span(stream, "tcsr_pack_inspect");
            hipLaunchKernelGGL(pack_inspect_kernel, dim3(grid), dim3(kThreads), 0, stream, src, dst, ts, eid, n, num_nodes,
                               rec_a.as<TaserRec>(), key_a.as<int32_t>(), d_partial.as<unsigned long long>(), low_digit_mask,
                               hist.as<uint32_t>(), num_blocks);
            hipLaunchKernelGGL(fold_info_kernel, dim3(kFoldBlocks), dim3(kThreads), 0, stream,
                               d_partial.as<unsigned long long>(), grid, d_folded.as<unsigned long long>());
            hipLaunchKernelGGL(fold_info_kernel, dim3(1), dim3(kThreads), 0, stream, d_folded.as<unsigned long long>(),
                               kFoldBlocks, d_info.as<unsigned long long>());
        }
        TASER_HIP_TRY(hipGetLastError());
        TASER_HIP_TRY(hipMemcpyAsync(info, d_info.p, sizeof(info), hipMemcpyDeviceToHost, stream));
        TASER_HIP_TRY(hipStreamSynchronize(stream));
        if (info[0]) return taser_fail(TASER_E_RANGE, "tcsr_build: a src node id is outside [0, %d)", num_nodes);
    }
    std::vector<DigitSpec> passes;
    if (info[1]) {
        const unsigned long long differ = info[2] & ~info[3];
        for (int b = 0; b < 8; ++b)
            if ((differ >> (8 * b)) & 0xffull) passes.push_back(DigitSpec{1, 8 * b, 0xffu});
    }
    const bool first_hist_known = passes.empty();   // no timestamp passes: the first digit is the one pack_inspect_kernel counted
    for (int shift = 0; shift < node_bits; shift += 8) {
        const int width = node_bits - shift < 8 ? node_bits - shift : 8;
        passes.push_back(DigitSpec{0, shift, (1u << width) - 1u});
    }

    // ---- search index over the sorted timestamps: storage (level 1 is written by the last sorting pass)
    TaserTimeIndex index = {};
    index.num_entries = n;
    int64_t index_total = 0, level_at[kTimeIndexLevels];
    for (int l = 0; l < kTimeIndexLevels; ++l) {
        const int64_t below = l == 0 ? n : index.len[l - 1];
        index.len[l] = (below + 15) / 16;
        level_at[l] = index_total;
        index_total += index.len[l];
    }
    DevBuf index_storage;
    TASER_HIP_TRY(index_storage.alloc((size_t)(index_total > 0 ? index_total : 1) * sizeof(int64_t)));
    for (int l = 0; l < kTimeIndexLevels; ++l) index.level[l] = index_storage.as<int64_t>() + level_at[l];
    // ---- one stable pass per digit, ping-pong between two buffers
    TASER_HIP_TRY(indptr.alloc(((size_t)num_nodes + 1) * sizeof(int64_t)));
    const unsigned scan_blocks = taser_scan::num_partials(hist_len);
    if (n > 0) {
        if (!passes.empty()) {
            TASER_HIP_TRY(rec_b.alloc(n * sizeof(TaserRec)));
            TASER_HIP_TRY(key_b.alloc(n * sizeof(int32_t)));
            TASER_HIP_TRY(partial.alloc((size_t)scan_blocks * sizeof(uint32_t)));
        }
        for (size_t pass = 0; pass < passes.size(); ++pass) {
            const DigitSpec& d = passes[pass];
            if (pass > 0 || !first_hist_known) {
                TaserProfileSpan span(stream, "tcsr_radix_hist");
                hipLaunchKernelGGL(radix_hist_kernel, dim3(num_blocks), dim3(kThreads), 0, stream,
                                   rec_a.as<TaserRec>(), key_a.as<int32_t>(), n, d, hist.as<uint32_t>(), num_blocks);
            }
            {
                TaserProfileSpan span(stream, "tcsr_scan");
                taser_scan::exclusive_scan_u32(hist.as<uint32_t>(), hist_len, partial.as<uint32_t>(), stream);
            }
            {
                TaserProfileSpan span(stream, "tcsr_radix_scatter");
                hipLaunchKernelGGL(radix_scatter_kernel, dim3(pass_grid(num_blocks)), dim3(kThreads), 0, stream,
                                   rec_a.as<TaserRec>(), key_a.as<int32_t>(), n, d, hist.as<uint32_t>(), num_blocks,
                                   rec_b.as<TaserRec>(), key_b.as<int32_t>(),
                                   pass + 1 == passes.size() ? index_storage.as<int64_t>() + level_at[0] : nullptr);
            }
            void* t = rec_a.p; rec_a.p = rec_b.p; rec_b.p = t;
            t = key_a.p; key_a.p = key_b.p; key_b.p = t;
        }
    }
    {
        TaserProfileSpan span(stream, "tcsr_indptr");
        hipLaunchKernelGGL(indptr_kernel, dim3(blocks_for(n + 1, kThreads * 4)), dim3(kThreads), 0, stream,
                           key_a.as<int32_t>(), n, num_nodes, indptr.as<int64_t>());
    }
    if (n > 0) {
        TaserProfileSpan span(stream, "tcsr_time_index");
        if (passes.empty())   // nothing was sorted: level 1 from the records as they are
            hipLaunchKernelGGL(time_index_first_kernel, dim3(blocks_for(index.len[0], kThreads)), dim3(kThreads), 0, stream,
                               rec_a.as<TaserRec>(), n, index_storage.as<int64_t>() + level_at[0], index.len[0]);
        for (int l = 1; l < kTimeIndexLevels; ++l)
            hipLaunchKernelGGL(time_index_next_kernel, dim3(blocks_for(index.len[l], kThreads)), dim3(kThreads), 0, stream,
                               index.level[l - 1], index.len[l - 1], index_storage.as<int64_t>() + level_at[l],
                               index.len[l]);
    }
    TASER_HIP_TRY(hipGetLastError());
    TASER_HIP_TRY(hipStreamSynchronize(stream));

    taser_tcsr* g = new (std::nothrow) taser_tcsr();
    if (!g) return taser_fail(TASER_E_OOM, "tcsr_build: host allocation failed");
    g->num_entries = n;
    g->num_nodes = num_nodes;
    g->indptr = indptr.release<int64_t>();
    g->rec = rec_a.release<TaserRec>();
    g->time_index_storage = index_storage.release<int64_t>();
    g->time_index = index;
    g->ts_only = nullptr;
    *out = g;
    return TASER_OK;
}

extern "C" int taser_tcsr_size(const taser_tcsr* g, int64_t* num_entries, int32_t* num_nodes) {
    if (!g) return taser_fail(TASER_E_ARG, "tcsr_size: null graph");
    if (num_entries) *num_entries = g->num_entries;
    if (num_nodes) *num_nodes = g->num_nodes;
    return TASER_OK;
}

extern "C" int taser_tcsr_view(const taser_tcsr* g, int64_t* indptr, int32_t* nbr, int64_t* ts, int32_t* eid,
                               void* hip_stream) {
    if (!g) return taser_fail(TASER_E_ARG, "tcsr_view: null graph");
    taser_clear_stale_hip_error();
    hipStream_t stream = (hipStream_t)hip_stream;
    if (indptr)
        TASER_HIP_TRY(hipMemcpyAsync(indptr, g->indptr, ((size_t)g->num_nodes + 1) * sizeof(int64_t),
                                     hipMemcpyDeviceToDevice, stream));
    if ((nbr || ts || eid) && g->num_entries > 0) {
        hipLaunchKernelGGL(unpack_kernel, dim3(blocks_for(g->num_entries, kThreads)), dim3(kThreads), 0, stream,
                           g->rec, g->num_entries, nbr, ts, eid);
        TASER_HIP_TRY(hipGetLastError());
    }
    return TASER_OK;
}

extern "C" void taser_tcsr_free(taser_tcsr* g) {
    if (!g) return;
    (void)hipFree(g->indptr);
    (void)hipFree(g->rec);
    (void)hipFree(g->time_index_storage);
    (void)hipFree(g->ts_only);
    delete g;
}
