// Candidate-window products of the adaptive sampler on gfx950.
//
// TASER (arXiv 2402.05396) samples in two levels (Sec. 3 overview, Alg. 1): a
// static finder returns m candidates per root, a small network turns them into
// probabilities q(j|i), and n of the m are kept. Two integer inputs of that
// network depend only on the candidate window (Sec. 3.2): freq(u_j), how often
// candidate j's node appears among the candidates, and the identity encoding
// IE[j][l] = 1 if u_j = u_l. The second draw of Alg. 1 then selects by one
// weight per (root, candidate).
//
// Both kernels use a group of G = 16, 32 or 64 lanes per root (G >= m), one
// lane per candidate, so a window never leaves registers: comparisons go
// through lane shuffles, prefix sums through __shfl_up.
#include <type_traits>

#include "sampling_device.h"
#include "taser_internal.h"

namespace {

constexpr int kThreads = 256;

// floor(b / d) for small b: d = 1 is the identity, otherwise a multiply-high with
// magic = ceil(2^32 / d), exact while b * d < 2^32 (here b < 2^13, d <= 2^12).
__device__ __forceinline__ uint32_t small_div(uint32_t b, uint32_t d, uint32_t magic) {
    return d == 1u ? b : __umulhi(b, magic);
}

// freq + identity. Lane j of a group holds u_j and builds a bit mask over l of
// the candidates equal to it; freq is the mask's population count. The m x m
// identity bytes of the roots of one wavefront are contiguous in the output,
// so the wave writes them as one flat range, four bytes per lane and store.
template <int G>
__global__ __launch_bounds__(kThreads) void candidate_encodings_kernel(
    const int32_t* __restrict__ nbr, const int32_t* __restrict__ count, int64_t num_roots, int m, uint32_t magic_m,
    uint32_t magic_mm, int32_t* __restrict__ freq, uint8_t* __restrict__ identity) {
    constexpr int kGroups = kWave / G;
    typedef typename std::conditional<(G > 32), uint64_t, uint32_t>::type Mask;   // one bit per candidate
    const int lane = threadIdx.x & (kWave - 1);
    const int group = lane / G, sub = lane % G;
    const int64_t wave_root0 = ((int64_t)blockIdx.x * (kThreads / kWave) + (threadIdx.x >> 6)) * kGroups;
    const int64_t q = wave_root0 + group;
    const bool live = q < num_roots;

    int c = 0;
    if (live) {
        c = count[q];
        c = c < 0 ? 0 : (c > m ? m : c);
    }
    const bool mine_valid = sub < c;
    int32_t u = -1;
    if (mine_valid) u = nbr[q * m + sub];

    Mask same = 0;   // bit l: candidate l is valid and names the same node as mine
    for (int l = 0; l < m; ++l) {
        const int32_t other = (int32_t)group_get<G>((uint32_t)u, l);
        if (mine_valid && l < c && other == u) same |= (Mask)1 << l;
    }
    if (live && sub < m) freq[q * m + sub] = (G > 32) ? __popcll((uint64_t)same) : __popc((uint32_t)same);

    if (identity == nullptr) return;   // uniform for the whole grid
    // Flat byte range of this wave's roots: [base, end). Byte b of it belongs to root
    // b / (m*m) of the wave, row (b % (m*m)) / m, column b % m.
    const uint32_t mm = (uint32_t)(m * m);
    int64_t roots_here = num_roots - wave_root0;
    if (roots_here <= 0) return;       // uniform for the wave
    if (roots_here > kGroups) roots_here = kGroups;
    const uint64_t base = (uint64_t)(uintptr_t)identity + (uint64_t)wave_root0 * mm;   // address of the first byte
    const uint32_t length = (uint32_t)roots_here * mm;
    const uint32_t head = (uint32_t)(base & 3u);          // bytes between the aligned start and base
    const uint64_t aligned = base - head;
    const uint32_t chunks = (head + length + 3u) >> 2;
    const uint32_t rounds = (chunks + kWave - 1) / kWave;   // the same for every lane: the shuffles below need them all
    for (uint32_t it = 0; it < rounds; ++it) {
        const uint32_t off = (it * kWave + (uint32_t)lane) * 4u;   // from `aligned`
        uint32_t word = 0;
        bool inside[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t o = off + (uint32_t)i;
            inside[i] = o >= head && o < head + length;
            const uint32_t b = inside[i] ? o - head : 0u;
            const uint32_t r = small_div(b, mm, magic_mm), rem = b - r * mm;
            const uint32_t row = small_div(rem, (uint32_t)m, magic_m), col = rem - row * (uint32_t)m;
            // every lane takes part in the shuffle; its source is lane `row` of group r
            const int src = (int)(r * G + row);
            Mask mask;
            if (G > 32) {
                const uint32_t lo = (uint32_t)__shfl((int)(uint32_t)same, src, kWave);
                const uint32_t hi = (uint32_t)__shfl((int)(uint32_t)((uint64_t)same >> 32), src, kWave);
                mask = (Mask)(((uint64_t)hi << 32) | lo);
            } else {
                mask = (Mask)(uint32_t)__shfl((int)(uint32_t)same, src, kWave);
            }
            word |= (uint32_t)((mask >> col) & 1u) << (8 * i);
        }
        const uint64_t at = aligned + off;
        if (inside[0] && inside[3]) {
            *reinterpret_cast<uint32_t*>(at) = word;
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (inside[i]) *reinterpret_cast<uint8_t*>(at + (uint32_t)i) = (uint8_t)(word >> (8 * i));
        }
    }
}

// n of m by per-slot weights: lane i of a group holds the weight of candidate i.
// The running sums of the weights are taken once; each of the k rounds scales one
// 64-bit draw to the remaining total, picks the first lane whose running sum exceeds
// it and takes that lane's weight out of the sums after it. Lane j keeps round j's pick, so the outputs are written coalesced at the end.
template <int G>
__global__ __launch_bounds__(kThreads) void select_weighted_kernel(
    const uint32_t* __restrict__ weight, const int32_t* __restrict__ count, int64_t num_roots, int m, int k,
    uint32_t seed_lo, uint32_t seed_hi, uint32_t hop, int32_t* __restrict__ sel, int32_t* __restrict__ out_count,
    const int32_t* __restrict__ c_nbr, const int32_t* __restrict__ c_eid, const int64_t* __restrict__ c_ts,
    int32_t* __restrict__ k_nbr, int32_t* __restrict__ k_eid, int64_t* __restrict__ k_ts) {
    constexpr int kGroups = kWave / G;
    const int lane = threadIdx.x & (kWave - 1);
    const int group = lane / G, sub = lane % G;
    const int64_t q = ((int64_t)blockIdx.x * (kThreads / kWave) + (threadIdx.x >> 6)) * kGroups + group;
    const bool live = q < num_roots;

    int c = 0;
    if (live) {
        c = count[q];
        c = c < 0 ? 0 : (c > m ? m : c);
    }
    uint64_t w = 0;
    if (sub < c) w = weight[q * m + sub];
    const bool draw = c > k;
    const int filled = draw ? k : c;
    int32_t my_pick = (!draw && sub < c) ? sub : -1;   // slot `sub` of the output
    if (__ballot(draw)) {
        uint64_t u = 0;
        if (draw && sub < k) u = draw64(seed_lo, seed_hi, hop, (uint64_t)q, (uint32_t)sub);
        uint64_t run = group_inclusive_scan64<G>(w, sub);
        uint64_t total = group_get64<G>(run, G - 1);
        for (int j = 0; j < k; ++j) {
            const int pick = group_weighted_pick<G>(run, total, w, group_get64<G>(u, j), draw, group, sub);   // -1 only if every remaining weight is 0
            if (draw && sub == j) my_pick = pick;
        }
    }
    if (live && sub < k) {
        const int64_t at = q * k + sub;
        sel[at] = my_pick;
        if (k_nbr) {
            const bool ok = my_pick >= 0;
            const int64_t from = q * m + (ok ? my_pick : 0);
            k_nbr[at] = ok ? c_nbr[from] : -1;
            k_eid[at] = ok ? c_eid[from] : -1;
            k_ts[at] = ok ? c_ts[from] : 0;
        }
    }
    if (live && sub == 0) out_count[q] = filled;
}

template <int G> unsigned grid_for(int64_t n) {
    constexpr int roots_per_block = (kThreads / kWave) * (kWave / G);
    return (unsigned)((n + roots_per_block - 1) / roots_per_block);
}

}  // namespace

extern "C" int taser_candidate_encodings(const int32_t* nbr, const int32_t* count, int64_t num_roots, int32_t m,
                                         int32_t* freq, uint8_t* identity, void* hip_stream) {
    if (num_roots < 0) return taser_fail(TASER_E_ARG, "candidate_encodings: num_roots = %lld", (long long)num_roots);
    if (m < 1 || m > TASER_MAX_M) return taser_fail(TASER_E_RANGE, "candidate_encodings: m = %d outside [1, %d]", m, TASER_MAX_M);
    if (num_roots * (int64_t)m >= ((int64_t)1 << 31))
        return taser_fail(TASER_E_RANGE, "candidate_encodings: num_roots * m must stay below 2^31");
    if (num_roots == 0) return TASER_OK;
    if (!nbr || !count || !freq) return taser_fail(TASER_E_ARG, "candidate_encodings: null nbr, count or freq");
    taser_clear_stale_hip_error();
    hipStream_t stream = (hipStream_t)hip_stream;
    TaserProfileSpan span(stream, "candidate_encodings");
    const uint32_t mm = (uint32_t)(m * m);
    const uint32_t magic_m = m > 1 ? (uint32_t)((((uint64_t)1 << 32) + (uint32_t)m - 1) / (uint32_t)m) : 0u;
    const uint32_t magic_mm = m > 1 ? (uint32_t)((((uint64_t)1 << 32) + mm - 1) / mm) : 0u;
    if (m <= 16)
        hipLaunchKernelGGL((candidate_encodings_kernel<16>), dim3(grid_for<16>(num_roots)), dim3(kThreads), 0, stream, nbr, count, num_roots, m, magic_m, magic_mm, freq, identity);
    else if (m <= 32)
        hipLaunchKernelGGL((candidate_encodings_kernel<32>), dim3(grid_for<32>(num_roots)), dim3(kThreads), 0, stream, nbr, count, num_roots, m, magic_m, magic_mm, freq, identity);
    else
        hipLaunchKernelGGL((candidate_encodings_kernel<64>), dim3(grid_for<64>(num_roots)), dim3(kThreads), 0, stream, nbr, count, num_roots, m, magic_m, magic_mm, freq, identity);
    TASER_HIP_TRY(hipGetLastError());
    return TASER_OK;
}

extern "C" int taser_select_weighted(const uint32_t* weight, const int32_t* count, int64_t num_roots, int32_t m,
                                     int32_t k, uint64_t seed, uint32_t hop, int32_t* sel, int32_t* out_count,
                                     const taser_hop_out* candidates, const taser_hop_out* kept, void* hip_stream) {
    if (num_roots < 0) return taser_fail(TASER_E_ARG, "select_weighted: num_roots = %lld", (long long)num_roots);
    if (m < 1 || m > TASER_MAX_M) return taser_fail(TASER_E_RANGE, "select_weighted: m = %d outside [1, %d]", m, TASER_MAX_M);
    if (k < 1 || k > TASER_MAX_K) return taser_fail(TASER_E_RANGE, "select_weighted: k = %d outside [1, %d]", k, TASER_MAX_K);
    if (num_roots * (int64_t)(m > k ? m : k) >= ((int64_t)1 << 31))
        return taser_fail(TASER_E_RANGE, "select_weighted: num_roots * max(m, k) must stay below 2^31");
    if ((candidates == nullptr) != (kept == nullptr))
        return taser_fail(TASER_E_ARG, "select_weighted: candidates and kept go together");
    if (num_roots == 0) return TASER_OK;
    if (!weight || !count || !sel || !out_count) return taser_fail(TASER_E_ARG, "select_weighted: null weight, count, sel or out_count");
    if (kept && (!candidates->nbr || !candidates->eid || !candidates->ts || !kept->nbr || !kept->eid || !kept->ts))
        return taser_fail(TASER_E_ARG, "select_weighted: null nbr/eid/ts buffer in candidates or kept");
    taser_clear_stale_hip_error();
    hipStream_t stream = (hipStream_t)hip_stream;
    const int32_t *c_nbr = nullptr, *c_eid = nullptr;
    const int64_t* c_ts = nullptr;
    int32_t *k_nbr = nullptr, *k_eid = nullptr;
    int64_t* k_ts = nullptr;
    if (kept) {
        c_nbr = candidates->nbr; c_eid = candidates->eid; c_ts = candidates->ts;
        k_nbr = kept->nbr; k_eid = kept->eid; k_ts = kept->ts;
    }
    const uint32_t s_lo = (uint32_t)seed, s_hi = (uint32_t)(seed >> 32);
    const int lanes = m > k ? m : k;
    TaserProfileSpan span(stream, "select_weighted");
    if (lanes <= 16)
        hipLaunchKernelGGL((select_weighted_kernel<16>), dim3(grid_for<16>(num_roots)), dim3(kThreads), 0, stream, weight, count, num_roots, m, k, s_lo, s_hi, hop, sel, out_count, c_nbr, c_eid, c_ts, k_nbr, k_eid, k_ts);
    else if (lanes <= 32)
        hipLaunchKernelGGL((select_weighted_kernel<32>), dim3(grid_for<32>(num_roots)), dim3(kThreads), 0, stream, weight, count, num_roots, m, k, s_lo, s_hi, hop, sel, out_count, c_nbr, c_eid, c_ts, k_nbr, k_eid, k_ts);
    else
        hipLaunchKernelGGL((select_weighted_kernel<64>), dim3(grid_for<64>(num_roots)), dim3(kThreads), 0, stream, weight, count, num_roots, m, k, s_lo, s_hi, hop, sel, out_count, c_nbr, c_eid, c_ts, k_nbr, k_eid, k_ts);
    TASER_HIP_TRY(hipGetLastError());
    return TASER_OK;
}
