// Temporal neighbor finding on gfx950: one 64-lane wavefront per root.
//
// What is computed follows TASER (arXiv 2402.05396) Sec. 2.1 (temporal
// neighborhood, uniform / most-recent finders), Alg. 2 (pivot search, then one
// neighbor per slot) and the layer loop of Alg. 1 (kept neighbors become the
// next hop's roots; n of m candidates drawn by given probabilities).
//
// How it is computed differs from Alg. 2's block-per-root / single-thread
// binary search / shared-memory bitmap with atomic retry:
//   * the pivot is found by a wave-wide 64-ary search: every round all 64
//     lanes probe one timestamp each and a ballot narrows the range 65-fold,
//     so a 2^25-entry list needs 5 dependent memory rounds instead of 25;
//   * selection without replacement is a partial Fisher-Yates shuffle whose
//     random draws come from a counter-based generator keyed by
//     (seed, hop, root index, slot). No atomics, no retries: the result is a
//     pure function of the inputs, independent of scheduling;
//   * weighted selection keeps the candidate window in registers (one lane per
//     candidate) and uses integer wave prefix sums.
#include "taser_internal.h"

namespace {

// ---- Philox4x32-10 (Salmon et al., SC'11) --------------------------------
__device__ __forceinline__ void philox_round(uint32_t (&c)[4], uint32_t k0, uint32_t k1) {
    const uint32_t lo0 = 0xD2511F53u * c[0], hi0 = __umulhi(0xD2511F53u, c[0]);
    const uint32_t lo1 = 0xCD9E8D57u * c[2], hi1 = __umulhi(0xCD9E8D57u, c[2]);
    const uint32_t a = hi1 ^ c[1] ^ k0;
    const uint32_t b = hi0 ^ c[3] ^ k1;
    c[0] = a; c[1] = lo1; c[2] = b; c[3] = lo0;
}

// 64 random bits for (seed, hop, root index, slot).
__device__ __forceinline__ uint64_t draw64(uint32_t seed_lo, uint32_t seed_hi, uint32_t hop,
                                           uint64_t root, uint32_t slot) {
    uint32_t c[4] = {(uint32_t)root, (uint32_t)(root >> 32), slot, hop};
    uint32_t k0 = seed_lo, k1 = seed_hi;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        philox_round(c, k0, k1);
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return ((uint64_t)c[1] << 32) | c[0];
}

// ---- wave helpers ----------------------------------------------------------
__device__ __forceinline__ uint32_t bcast32(uint32_t v, int src_lane) {
    return (uint32_t)__builtin_amdgcn_readlane((int)v, src_lane);
}
__device__ __forceinline__ uint64_t bcast64(uint64_t v, int src_lane) {
    return ((uint64_t)bcast32((uint32_t)(v >> 32), src_lane) << 32) | bcast32((uint32_t)v, src_lane);
}
// Number of entries in [lo, hi) with ts < t, for a time-sorted list.
// All lanes take part; lo, hi, t are wave-uniform.
__device__ __forceinline__ int64_t wave_cutoff(const TaserRec* __restrict__ rec, int64_t lo,
                                               int64_t hi, int64_t t, int lane) {
    int64_t a = lo, b = hi;   // entries before a are < t, entries from b on are >= t
    while (b - a > kWave) {
        // 64 pivots that cut [a, b) into 65 nearly equal parts: pivot i sits at
        // a + floor(len * (i + 1) / 65), split as q*(i+1) + floor(r*(i+1)/65) so
        // that everything stays in 32 bits (len < 2^31).
        const uint32_t len = (uint32_t)(b - a);
        const uint32_t q65 = len / 65u, r65 = len - q65 * 65u;
        auto pivot = [&](uint32_t i1) { return a + (int64_t)(q65 * i1 + (r65 * i1) / 65u); };
        const bool before = rec[pivot((uint32_t)lane + 1u)].ts < t;
        const uint32_t c = (uint32_t)__popcll(__ballot(before));   // the predicate is monotone in the lane
        const int64_t na = (c > 0) ? pivot(c) + 1 : a;
        const int64_t nb = (c < (uint32_t)kWave) ? pivot(c + 1u) : b;
        a = na;
        b = nb;
    }
    const int64_t p = a + lane;
    const bool before = (p < b) && (rec[p].ts < t);
    return a + __popcll(__ballot(before)) - lo;
}

__device__ __forceinline__ void store_slot(int32_t* o_nbr, int32_t* o_eid, int64_t* o_ts,
                                           int64_t at, const TaserRec& r) {
    o_nbr[at] = r.nbr;
    o_eid[at] = r.eid;
    o_ts[at] = r.ts;
}

constexpr int kRootsPerBlock = 4;   // 256 threads

template <int POLICY>
__global__ __launch_bounds__(kRootsPerBlock* kWave) void sample_hop_kernel(
    const int64_t* __restrict__ indptr, const TaserRec* __restrict__ rec,
    const int32_t* __restrict__ roots, const int64_t* __restrict__ times, int64_t num_roots,
    int32_t num_nodes, int k, uint32_t seed_lo, uint32_t seed_hi, uint32_t hop, int m, const uint32_t* __restrict__ edge_weight,
    int32_t* __restrict__ o_nbr, int32_t* __restrict__ o_eid, int64_t* __restrict__ o_ts,
    int32_t* __restrict__ o_count) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t q = (int64_t)blockIdx.x * kRootsPerBlock + wave;   // root index, wave-uniform
    if (q >= num_roots) return;

    const int32_t v = roots[q];
    int64_t lo = 0, cnt = 0;
    if (v >= 0 && v < num_nodes) {   // anything else is a root without neighbors
        const int64_t t = times[q];
        lo = indptr[v];
        const int64_t hi = indptr[v + 1];
        cnt = wave_cutoff(rec, lo, hi, t, lane);
    }
    const int64_t out0 = q * k;
    const TaserRec pad = {0, -1, -1};
    int filled;

    if (POLICY == TASER_RECENT || (POLICY == TASER_UNIFORM && cnt <= k)) {
        filled = (int)(cnt < k ? cnt : k);
        if (lane < k) store_slot(o_nbr, o_eid, o_ts, out0 + lane, lane < filled ? rec[lo + cnt - 1 - lane] : pad);
    } else if (POLICY == TASER_UNIFORM) {
        // Partial Fisher-Yates over the virtual array a[x] = x, x in [0, cnt).
        // Lane j owns step j: it remembers the position it overwrote (pos) and
        // the value it put there (val); a lookup of a[x] at step j is the val
        // of the latest earlier step that wrote x, else x itself.
        filled = k;
        uint32_t pos = 0, val = 0, idx = 0;
        if (lane < k) {
            const uint64_t u = draw64(seed_lo, seed_hi, hop, (uint64_t)q, (uint32_t)lane);
            pos = (uint32_t)lane + (uint32_t)__umul64hi(u, (uint64_t)(cnt - lane));
        }
        for (int j = 0; j < k; ++j) {
            const uint32_t r = bcast32(pos, j);
            const bool earlier = lane < j;
            const uint64_t hit_r = __ballot(earlier && pos == r);
            const uint64_t hit_j = __ballot(earlier && pos == (uint32_t)j);
            const uint32_t a_r = hit_r ? bcast32(val, 63 - __clzll((long long)hit_r)) : r;
            const uint32_t a_j = hit_j ? bcast32(val, 63 - __clzll((long long)hit_j)) : (uint32_t)j;
            if (lane == j) {
                idx = a_r;
                val = a_j;
            }
        }
        if (lane < k) store_slot(o_nbr, o_eid, o_ts, out0 + lane, rec[lo + idx]);
    } else {
        // Candidate window: lane i holds candidate i (the i-th most recent).
        const int c = (int)(cnt < m ? cnt : m);
        TaserRec mine = pad;
        uint64_t w = 0;
        if (lane < c) {
            mine = rec[lo + cnt - 1 - lane];
            w = edge_weight[mine.eid];
        }
        if (c <= k) {
            filled = c;
            if (lane < k) store_slot(o_nbr, o_eid, o_ts, out0 + lane, mine);
        } else {
            filled = k;
            uint64_t u = 0;
            if (lane < k) u = draw64(seed_lo, seed_hi, hop, (uint64_t)q, (uint32_t)lane);
            for (int j = 0; j < k; ++j) {
                uint64_t run = w;   // inclusive wave prefix sum of the remaining weights
#pragma unroll
                for (int d = 1; d < kWave; d <<= 1) {
                    const uint32_t lo32 = __shfl_up((uint32_t)run, d, kWave);
                    const uint32_t hi32 = __shfl_up((uint32_t)(run >> 32), d, kWave);
                    if (lane >= d) run += ((uint64_t)hi32 << 32) | lo32;
                }
                const uint64_t total = bcast64(run, kWave - 1);
                const uint64_t x = __umul64hi(bcast64(u, j), total);
                const uint64_t above = __ballot(run > x);
                const int pick = __ffsll((long long)above) - 1;
                if (lane == pick) {
                    store_slot(o_nbr, o_eid, o_ts, out0 + j, mine);
                    w = 0;
                }
            }
        }
    }
    if (lane == 0) o_count[q] = filled;
}

template <int POLICY>
void launch_hop(const taser_tcsr* g, const int32_t* roots, const int64_t* times, int64_t n, int k,
                uint64_t seed, uint32_t hop, int m, const uint32_t* edge_weight,
                const taser_hop_out& o, hipStream_t stream) {
    const unsigned grid = (unsigned)((n + kRootsPerBlock - 1) / kRootsPerBlock);
    static const char* const names[3] = {"sample_hop_recent", "sample_hop_uniform", "sample_hop_weighted"};
    TaserProfileSpan span(stream, names[POLICY]);
    hipLaunchKernelGGL(sample_hop_kernel<POLICY>, dim3(grid), dim3(kRootsPerBlock * kWave), 0, stream,
                       g->indptr, g->rec, roots, times, n, g->num_nodes, k, (uint32_t)seed, (uint32_t)(seed >> 32),
                       hop, m, edge_weight, o.nbr, o.eid, o.ts, o.count);
}

}  // namespace

extern "C" int taser_sample_temporal(const taser_tcsr* g, const int32_t* roots, const int64_t* times,
                                     int64_t num_roots, int32_t k, int32_t hops, int32_t policy,
                                     uint64_t seed, int32_t m, const uint32_t* edge_weight,
                                     const taser_hop_out* out, void* hip_stream) {
    if (!g || !out) return taser_fail(TASER_E_ARG, "sample_temporal: null graph or output array");
    if (num_roots < 0) return taser_fail(TASER_E_ARG, "sample_temporal: num_roots = %lld", (long long)num_roots);
    if (num_roots > 0 && (!roots || !times)) return taser_fail(TASER_E_ARG, "sample_temporal: null roots/times");
    if (k < 1 || k > TASER_MAX_K) return taser_fail(TASER_E_RANGE, "sample_temporal: k = %d outside [1, %d]", k, TASER_MAX_K);
    if (hops < 1 || hops > TASER_MAX_HOPS) return taser_fail(TASER_E_RANGE, "sample_temporal: hops = %d outside [1, %d]", hops, TASER_MAX_HOPS);
    if (policy != TASER_RECENT && policy != TASER_UNIFORM && policy != TASER_WEIGHTED)
        return taser_fail(TASER_E_ARG, "sample_temporal: unknown policy %d", policy);
    if (policy == TASER_WEIGHTED) {
        if (m < 1 || m > TASER_MAX_M) return taser_fail(TASER_E_RANGE, "sample_temporal: m = %d outside [1, %d]", m, TASER_MAX_M);
        if (!edge_weight) return taser_fail(TASER_E_ARG, "sample_temporal: weighted policy needs edge_weight");
    }
    int64_t n = num_roots;
    for (int h = 0; h < hops; ++h) {
        if (n > 0 && (!out[h].nbr || !out[h].eid || !out[h].ts || !out[h].count))
            return taser_fail(TASER_E_ARG, "sample_temporal: null output buffer at hop %d", h);
        if (n * k >= ((int64_t)1 << 31)) return taser_fail(TASER_E_RANGE, "sample_temporal: num_roots * k^hops must stay below 2^31");
        n *= k;
    }
    hipStream_t stream = (hipStream_t)hip_stream;
    const int32_t* cur_roots = roots;
    const int64_t* cur_times = times;
    n = num_roots;
    for (int h = 0; h < hops && n > 0; ++h) {
        switch (policy) {
            case TASER_RECENT: launch_hop<TASER_RECENT>(g, cur_roots, cur_times, n, k, seed, (uint32_t)h, m, edge_weight, out[h], stream); break;
            case TASER_UNIFORM: launch_hop<TASER_UNIFORM>(g, cur_roots, cur_times, n, k, seed, (uint32_t)h, m, edge_weight, out[h], stream); break;
            default: launch_hop<TASER_WEIGHTED>(g, cur_roots, cur_times, n, k, seed, (uint32_t)h, m, edge_weight, out[h], stream); break;
        }
        cur_roots = out[h].nbr;
        cur_times = out[h].ts;
        n *= k;
    }
    TASER_HIP_TRY(hipGetLastError());
    return TASER_OK;
}
