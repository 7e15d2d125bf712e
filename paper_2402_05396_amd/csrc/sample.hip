// Temporal neighbor finding on gfx950: one group of 16, 32 or 64 lanes of a
// wavefront per root (the smallest that holds the k slots, or the m candidates
// of the weighted policy).
//
// What is computed follows TASER (arXiv 2402.05396) Sec. 2.1 (temporal
// neighborhood, uniform / most-recent finders), Alg. 2 (pivot search, then one
// neighbor per slot) and the layer loop of Alg. 1 (kept neighbors become the
// next hop's roots; n of m candidates drawn by given probabilities).
//
// How it is computed differs from Alg. 2's block-per-root / single-thread
// binary search / shared-memory bitmap with atomic retry:
//   * the pivot is found by a cooperative 16-ary descent through a small index
//     of the timestamps: every level 16 lanes of a root read 16 neighboring
//     entries (one 128-byte line) and a ballot gives the child, so a 2^25-entry
//     list needs 7 dependent reads of one line each instead of 25 scattered ones;
//   * selection without replacement is a partial Fisher-Yates shuffle whose
//     random draws come from a counter-based generator keyed by
//     (seed, hop, root index, slot). No atomics, no retries: the result is a
//     pure function of the inputs, independent of scheduling;
//   * weighted selection keeps the candidate window in registers (one lane per
//     candidate) and uses integer prefix sums across the group's lanes;
//   * the inverse-timespan finder, whose weights depend on the query time, reads
//     the whole valid list with a block per root (see its kernel).
#include <mutex>

#include "gather_kernel.h"
#include "sampling_device.h"
#include "taser_internal.h"

namespace {

// Number of entries in [lo, hi) with ts < t, for a time-sorted list [lo, hi) of the
// record array: the first position p* in [lo, hi] that is not "before", where
// before(p) = p < lo, or p < hi and ts[p] < t (monotone over the whole array).
// The search descends the levels of the time index. Entry i of level L stands for
// the positions [i 16^L, (i+1) 16^L) and holds the timestamp of the last of them;
// p* lies in the first entry whose last position is not before. A group starts at
// the lowest level at which its list touches at most 16 entries, then reads one
// aligned block of 16 entries (one 128-byte line) per level down to the records
// themselves (level 0). 16 lanes of the group probe; whether a position is below
// lo or at/after hi is known without reading it. Groups of one wave start at
// different levels under one wave-uniform loop. lo, hi, t are uniform inside a
// group; every lane of the wave must call this.
// R independent lists per group are searched side by side (their loads of a level are
// issued together): the kernel is bound by how many dependent reads are in flight.
// Positions are 32-bit: a graph has fewer than 2^31 entries, and the last position an index entry
// stands for, ((i + 1) << 4 L) - 1 with i < ceil(n / 16^L), stays below n + 16^L < 2^32.
template <int G, int R>
__device__ __forceinline__ void group_cutoff(const TaserRec* __restrict__ rec, const TaserTimeIndex& index,
                                             const uint32_t (&lo)[R], const uint32_t (&hi)[R], const int64_t (&t)[R],
                                             int group, int sub, uint32_t (&cnt)[R]) {
    const uint32_t n = (uint32_t)index.num_entries;
    int top[R];
    uint32_t at[R];   // entry of the current level that holds p*
#pragma unroll
    for (int r = 0; r < R; ++r) {
        // lowest level at which the list touches at most 16 entries: (hi >> 4 L) - (lo >> 4 L) is
        // floor((hi - lo) / 16^L) or one more, so it is the first L with hi - lo < 16^(L + 1), or the next
        const uint32_t d = hi[r] - lo[r];
        const int bits = d ? 32 - __clz((int)d) : 0;
        int L = bits ? (bits + 3) / 4 - 1 : 0;                          // <= 7 for d < 2^31
        if ((hi[r] >> (4 * L)) - (lo[r] >> (4 * L)) > 15u) ++L;         // never beyond 7: positions below 2^31 differ by < 8 there
        top[r] = L;
        at[r] = 0;
    }
#pragma unroll
    for (int L = kTimeIndexLevels; L >= 0; --L) {
        bool any = false;
#pragma unroll
        for (int r = 0; r < R; ++r) any |= L <= top[r];
        if (!__ballot(any)) continue;   // no list of this wave is at this level yet
        const uint32_t len = L == 0 ? n : (uint32_t)index.len[L - 1];
        uint32_t first[R], probe[R];
        bool known_before[R], read[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {   // what to read
            const bool active = L <= top[r];
            first[r] = at[r] * 16u;
            uint32_t width = 16;
            if (L == top[r]) {
                first[r] = lo[r] >> (4 * L);
                width = (hi[r] >> (4 * L)) - first[r] + 1u;
            }
            known_before[r] = false;
            read[r] = false;
            probe[r] = first[r] + (uint32_t)sub;
            if (active && (uint32_t)sub < width && probe[r] < len) {
                uint32_t pos = ((probe[r] + 1u) << (4 * L)) - 1u;       // last position the entry stands for
                if (pos >= n) pos = n - 1u;
                if (pos < lo[r]) known_before[r] = true;
                else if (pos < hi[r]) read[r] = true;
                if (L == 0) probe[r] = pos;
            }
        }
        int64_t ts[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {   // the reads of all lists, back to back
            ts[r] = 0;
            if (read[r]) ts[r] = L == 0 ? rec[probe[r]].ts : index.level[L - 1][probe[r]];
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const bool before = known_before[r] || (read[r] && ts[r] < t[r]);
            const uint32_t c = (uint32_t)__popcll(group_bits<G>(__ballot(before), group));   // before is monotone in the lane
            if (L <= top[r]) at[r] = first[r] + c;
        }
    }
    // `at` is p*, except past the array's last, partial entry, where it overshoots hi
#pragma unroll
    for (int r = 0; r < R; ++r) cnt[r] = (at[r] < hi[r] ? at[r] : hi[r]) - lo[r];
}

template <int G>
__device__ __forceinline__ int64_t group_cutoff(const TaserRec* __restrict__ rec, const TaserTimeIndex& index,
                                                int64_t lo, int64_t hi, int64_t t, int group, int sub) {
    const uint32_t lo1[1] = {(uint32_t)lo}, hi1[1] = {(uint32_t)hi};
    const int64_t t1[1] = {t};
    uint32_t cnt1[1];
    group_cutoff<G, 1>(rec, index, lo1, hi1, t1, group, sub, cnt1);
    return (int64_t)cnt1[0];
}

__device__ __forceinline__ void store_slot(int32_t* o_nbr, int32_t* o_eid, int64_t* o_ts,
                                           int64_t at, const TaserRec& r) {
    o_nbr[at] = r.nbr;
    o_eid[at] = r.eid;
    o_ts[at] = r.ts;
}

constexpr int kThreads = 256;

// Selection for the R roots of a group whose cutoffs are known. Leaves, in lane `sub` of the
// group, the record of output slot `sub` of every root (padding from slot `filled` on). Written in
// stages over all R roots, so that the loads of one stage (the last k records; the candidate window
// and then its weights; the uniformly drawn records) are in flight for all of them together, with
// the draws' arithmetic in between. Every lane of the wave must call it.
template <int POLICY, int G, int R>
__device__ __forceinline__ void select_slots(
    const TaserRec* __restrict__ rec, int64_t q0, const uint32_t (&lo)[R], const uint32_t (&cnt)[R], int group, int sub, int k,
    uint32_t seed_lo, uint32_t seed_hi, uint32_t hop, int m, const uint32_t* __restrict__ edge_weight,
    TaserRec (&out)[R], int (&filled)[R]) {
    const TaserRec pad = {0, -1, -1};

    // All lanes of the wave walk through the same code; what a group does not need is masked.
    if (POLICY == TASER_RECENT) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            filled[r] = (int)(cnt[r] < (uint32_t)k ? cnt[r] : (uint32_t)k);
            out[r] = pad;
            if (sub < filled[r]) out[r] = rec[lo[r] + cnt[r] - 1u - (uint32_t)sub];
        }
    } else if (POLICY == TASER_UNIFORM) {
        // cnt <= k: everything, most recent first. Otherwise a partial Fisher-Yates
        // over the virtual array a[x] = x, x in [0, cnt): step j draws pos_j in
        // [j, cnt), takes a[pos_j] and puts a[j] there; lane j of the group owns step j.
        uint32_t at[R];   // list position of this lane's slot
        bool some[R];     // false: padding
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const bool shuffle = cnt[r] > (uint32_t)k;
            filled[r] = shuffle ? k : (int)cnt[r];
            uint32_t pos = 0, val = 0, idx = 0;
            if (shuffle && sub < k) {
                const uint64_t u = draw64(seed_lo, seed_hi, hop, (uint64_t)(q0 + r), (uint32_t)sub);
                pos = (uint32_t)sub + mulhi_64x32(u, cnt[r] - (uint32_t)sub);
            }
            if (__ballot(shuffle)) {
                if (G <= 32) {
                    // Every lane resolves its own step from the positions all steps drew (no values
                    // need to travel): a[x] at step j is x unless an earlier step wrote x; the latest
                    // such step i put there what position i held at step i, which is the same question
                    // for (i, i). Chains are short: one pass when no two steps of a root collide.
                    uint32_t drawn[G];
#pragma unroll
                    for (int i = 0; i < G; ++i) drawn[i] = group_get<G>(pos, i);
                    uint32_t x = pos;
                    int before = sub;                       // only steps below this one count
                    bool open = shuffle && sub < k;
                    while (__ballot(open)) {
                        int found = -1;
#pragma unroll
                        for (int i = 0; i < G; ++i)
                            if (i < before && drawn[i] == x) found = i;   // ascending: the latest match stays
                        if (open) {
                            if (found < 0) {
                                open = false;
                            } else {
                                x = (uint32_t)found;
                                before = found;
                            }
                        }
                    }
                    idx = x;
                } else {
                    // lane j of the group owns step j; it remembers the position it overwrote (pos) and
                    // the value it put there (val); a lookup of a[x] at step j is the val of the latest
                    // earlier step that wrote x, else x itself
                    for (int j = 0; j < k; ++j) {
                        const uint32_t x = group_get<G>(pos, j);
                        const bool earlier = sub < j;
                        const uint64_t hit_x = group_bits<G>(__ballot(earlier && pos == x), group);
                        const uint64_t hit_j = group_bits<G>(__ballot(earlier && pos == (uint32_t)j), group);
                        // the shuffles are executed by every lane; lanes without a hit read lane 0 and drop it
                        const uint32_t v_x = group_get<G>(val, hit_x ? 63 - __clzll((long long)hit_x) : 0);
                        const uint32_t v_j = group_get<G>(val, hit_j ? 63 - __clzll((long long)hit_j) : 0);
                        if (sub == j) {
                            idx = hit_x ? v_x : x;
                            val = hit_j ? v_j : (uint32_t)j;
                        }
                    }
                }
            }
            at[r] = 0;
            some[r] = false;
            if (sub < k) {
                if (shuffle) {
                    at[r] = idx;
                    some[r] = true;
                } else if (sub < filled[r]) {
                    at[r] = cnt[r] - 1u - (uint32_t)sub;
                    some[r] = true;
                }
            }
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            out[r] = pad;
            if (some[r]) out[r] = rec[lo[r] + at[r]];
        }
    } else {
        // Candidate window: lane i of the group holds candidate i (the i-th most recent);
        // lane j notes which candidate draw j picked and fetches it from that lane at the end.
        TaserRec mine[R];
        uint64_t w[R];
        int c[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            c[r] = (int)(cnt[r] < (uint32_t)m ? cnt[r] : (uint32_t)m);
            mine[r] = pad;
            if (sub < c[r]) mine[r] = rec[lo[r] + cnt[r] - 1u - (uint32_t)sub];
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            w[r] = 0;
            if (sub < c[r]) w[r] = edge_weight[mine[r].eid];
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const bool draw = c[r] > k;
            filled[r] = draw ? k : c[r];
            int my_pick = (!draw && sub < c[r]) ? sub : -1;
            if (__ballot(draw)) {
                uint64_t u = 0;
                if (draw && sub < k) u = draw64(seed_lo, seed_hi, hop, (uint64_t)(q0 + r), (uint32_t)sub);
                // running sums of the weights once; every draw then only takes its pick out of them
                uint64_t run = group_inclusive_scan64<G>(w[r], sub);
                uint64_t total = group_get64<G>(run, G - 1);
                for (int j = 0; j < k; ++j) {
                    const int pick = group_weighted_pick<G>(run, total, w[r], group_get64<G>(u, j), draw, group, sub);
                    if (draw && sub == j) my_pick = pick;
                }
            }
            const int from = my_pick < 0 ? 0 : my_pick;   // the shuffles are executed by every lane
            const int32_t p_nbr = (int32_t)group_get<G>((uint32_t)mine[r].nbr, from);
            const int32_t p_eid = (int32_t)group_get<G>((uint32_t)mine[r].eid, from);
            const int64_t p_ts = (int64_t)group_get64<G>((uint64_t)mine[r].ts, from);
            out[r] = pad;
            if (my_pick >= 0 && sub < k) out[r] = TaserRec{p_ts, p_nbr, p_eid};
        }
    }
}

// What a hop kernel needs to also write the feature rows of the edges it sampled
// (Sec. 3.4 slices them right after Alg. 2 found the neighbors): the table, and the dense
// output of this hop, one row per slot in slot order. The launcher guarantees: row_bytes a
// multiple of 4 and >= 16, table and pitch 4-byte aligned, `out` 16-byte aligned, and the
// rows of one wavefront's roots a multiple of 16 bytes.
struct RowCopy {
    const uint8_t* table;
    int64_t table_rows, pitch_bytes;
    uint8_t* out;
    const uint8_t* zeros;    // 16 zero bytes
    uint32_t row_bytes;
    uint32_t magic;          // ceil(2^32 / row_bytes)
    uint32_t step_rows, step_rest;   // 1024 = step_rows * row_bytes + step_rest
};

// The rows of one wavefront's roots form one contiguous, 16-byte aligned range of the
// output: `rows_here` rows whose edge ids the wave has just left in `wave_eid` (LDS, slot
// order). The range is copied as a flat stream, 16 bytes per lane and 1 KiB per wave
// instruction, kInFlight of them in flight; a lane finds the row of its first chunk by one
// division and of the following ones by stepping. A chunk inside one row is one 16-byte
// load (4-byte aligned); one that crosses a row end takes two. Padding slots and ids
// outside the table give zero rows.
template <int kInFlight>
__device__ __forceinline__ void copy_wave_rows(const RowCopy& rc, const int32_t* wave_eid, uint32_t rows_here,
                                               int64_t first_row, int lane) {
    using namespace taser_gather;
    const uint32_t bytes_here = rows_here * rc.row_bytes;
    uint8_t* const out = rc.out + first_row * (int64_t)rc.row_bytes;
    uint32_t o = (uint32_t)lane * 16u;
    uint32_t row = __umulhi(o, rc.magic);
    uint32_t off = o - row * rc.row_bytes;
    for (uint32_t base = 0; base < bytes_here; base += kInFlight * 1024u) {
        uint32_t c_o[kInFlight], c_row[kInFlight], c_off[kInFlight];
        bool whole[kInFlight], cross[kInFlight];
#pragma unroll
        for (int u = 0; u < kInFlight; ++u) {
            c_o[u] = o;
            c_row[u] = row;
            c_off[u] = off;
            const bool live = o < bytes_here;
            whole[u] = live && off + 16u <= rc.row_bytes;
            cross[u] = live && !whole[u];
            o += 1024u;
            row += rc.step_rows;
            off += rc.step_rest;
            if (off >= rc.row_bytes) {
                off -= rc.row_bytes;
                ++row;
            }
        }
        u32x4 vals[kInFlight], tail[kInFlight], head[kInFlight];
        uint32_t keep[kInFlight];   // dwords of a crossing chunk that belong to the row it starts in (1..3)
#pragma unroll
        for (int u = 0; u < kInFlight; ++u) {
            const uint32_t r = c_row[u] < rows_here ? c_row[u] : rows_here - 1u;
            const int32_t id = wave_eid[r];
            const bool ok = id >= 0 && id < rc.table_rows;
            const uint8_t* src = rc.table + (int64_t)(ok ? id : 0) * rc.pitch_bytes;
            vals[u] = ((GlobalChunk16Ptr)(whole[u] && ok ? src + c_off[u] : rc.zeros))->v;
            // A chunk that crosses a row end is the last dwords of this row followed by the first of
            // the next one (rows hold at least 16 bytes): the last 16 bytes of the one and the first
            // 16 of the other, read by the crossing lanes only and put together below.
            keep[u] = (rc.row_bytes - c_off[u]) >> 2;
            tail[u] = head[u] = u32x4{0u, 0u, 0u, 0u};
            if (cross[u]) {
                const int32_t id1 = r + 1u < rows_here ? wave_eid[r + 1u] : -1;   // past the range: never stored
                const bool ok1 = id1 >= 0 && id1 < rc.table_rows;
                tail[u] = ((GlobalChunk16Ptr)(ok ? src + (rc.row_bytes - 16u) : rc.zeros))->v;
                head[u] = ((GlobalChunk16Ptr)(ok1 ? rc.table + (int64_t)id1 * rc.pitch_bytes : rc.zeros))->v;
            }
        }
#pragma unroll
        for (int u = 0; u < kInFlight; ++u) {
            // dwords 4 - keep .. 7 - keep of (tail, head), by selects in every lane
            const u32x4 t = tail[u], h = head[u];
            const bool k1 = keep[u] == 1u, k2 = keep[u] == 2u;
            const uint32_t d0 = k1 ? t.w : k2 ? t.z : t.y;
            const uint32_t d1 = k1 ? h.x : k2 ? t.w : t.z;
            const uint32_t d2 = k1 ? h.y : k2 ? h.x : t.w;
            const uint32_t d3 = k1 ? h.z : k2 ? h.y : h.x;
            if (cross[u]) vals[u] = u32x4{d0, d1, d2, d3};
        }
#pragma unroll
        for (int u = 0; u < kInFlight; ++u) {
            if (c_o[u] + 16u <= bytes_here) {
                __builtin_nontemporal_store(vals[u], reinterpret_cast<u32x4*>(out + c_o[u]));
            } else if (c_o[u] < bytes_here) {
                const uint32_t w[4] = {vals[u].x, vals[u].y, vals[u].z, vals[u].w};
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (c_o[u] + 4u * i < bytes_here) *reinterpret_cast<uint32_t*>(out + c_o[u] + 4u * i) = w[i];
            }
        }
    }
}

// G lanes per root: G >= k, and G >= m for the weighted policy. A group serves
// kRootsPerGroup consecutive roots: their searches run side by side, their selections
// stage by stage (measured: two roots per group pay for the most-recent finder on large
// hops, 39 -> 32 us for 120 000 roots; the uniform and weighted finders, whose time is
// mostly the arithmetic of their draws, gain nothing from them).
// With ROWS (one root per group) a wavefront then also copies the table rows of the edges
// it sampled into the hop's dense row output: the finder is bound by instruction issue and
// dependent reads, the copy by memory bandwidth, and in one kernel the wavefronts of a
// compute unit that search overlap with those that copy.
template <int POLICY, int G, int kRootsPerGroup, bool ROWS>
__global__ __launch_bounds__(kThreads) void sample_hop_kernel(
    const int64_t* __restrict__ indptr, const TaserRec* __restrict__ rec, const TaserTimeIndex index,
    const int32_t* __restrict__ roots, const int64_t* __restrict__ times, int64_t num_roots,
    int32_t num_nodes, int k, uint32_t seed_lo, uint32_t seed_hi, uint32_t hop, int m, const uint32_t* __restrict__ edge_weight,
    int32_t* __restrict__ o_nbr, int32_t* __restrict__ o_eid, int64_t* __restrict__ o_ts,
    int32_t* __restrict__ o_count, const RowCopy rows) {
    static_assert(!ROWS || kRootsPerGroup == 1, "the row copy takes one root per group");
    constexpr int kGroups = kWave / G;                         // groups per wave
    const int lane = threadIdx.x & (kWave - 1);
    const int group = lane / G, sub = lane % G;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int64_t wave_q0 = ((int64_t)blockIdx.x * (kThreads / kWave) + wave) * (kGroups * kRootsPerGroup);   // first root of the wave
    const int64_t q0 = wave_q0 + group * kRootsPerGroup;

    uint32_t lo[kRootsPerGroup], hi[kRootsPerGroup], cnt[kRootsPerGroup];   // positions fit 32 bits: fewer than 2^31 entries
    int64_t t[kRootsPerGroup];
    int32_t v[kRootsPerGroup];
#pragma unroll
    for (int r = 0; r < kRootsPerGroup; ++r) {
        lo[r] = hi[r] = 0;
        t[r] = 0;
        v[r] = q0 + r < num_roots ? roots[q0 + r] : -1;
    }
#pragma unroll
    for (int r = 0; r < kRootsPerGroup; ++r) {
        if (v[r] >= 0 && v[r] < num_nodes) {   // anything else is a root without neighbors
            t[r] = times[q0 + r];
            lo[r] = (uint32_t)indptr[v[r]];
            hi[r] = (uint32_t)indptr[v[r] + 1];
        }
    }
    group_cutoff<G, kRootsPerGroup>(rec, index, lo, hi, t, group, sub, cnt);   // 0 for dead roots (lo == hi)
    TaserRec slot[kRootsPerGroup];
    int filled[kRootsPerGroup];
    select_slots<POLICY, G, kRootsPerGroup>(rec, q0, lo, cnt, group, sub, k, seed_lo, seed_hi, hop, m, edge_weight, slot, filled);
#pragma unroll
    for (int r = 0; r < kRootsPerGroup; ++r) {
        if (q0 + r < num_roots) {
            if (sub < k) store_slot(o_nbr, o_eid, o_ts, (q0 + r) * k + sub, slot[r]);
            if (sub == 0) o_count[q0 + r] = filled[r];
        }
    }
    if (ROWS) {
        __shared__ int32_t eid_of_row[kThreads / kWave][kWave];   // per wave: k ids per group, slot order (kGroups * k <= 64)
        if (sub < k) eid_of_row[wave][group * k + sub] = slot[0].eid;
        // only this wave reads them back: its LDS operations complete in order
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        int64_t roots_here = num_roots - wave_q0;
        if (roots_here > kGroups) roots_here = kGroups;
        // wave instructions of the copy in flight: four where a wavefront has four roots' rows to move, two (and
        // 28 registers fewer) where it has one or two roots
        if (roots_here > 0) copy_wave_rows<(G == 16 ? 4 : 2)>(rows, eid_of_row[wave], (uint32_t)roots_here * (uint32_t)k, wave_q0 * k, lane);
    }
}

// ---- inverse-timespan finder -------------------------------------------------
// Weight of an entry at time ts for a query at t > ts: max(1, floor(2^32 / (t - ts))).
__device__ __forceinline__ uint64_t inverse_timespan_weight(int64_t t, int64_t ts) {
    const uint64_t delta = (uint64_t)t - (uint64_t)ts;   // exact difference, >= 1
    if (delta >> 32) return 1;                           // the quotient is 1 (delta = 2^32) or 0
    const uint32_t d = (uint32_t)delta;
    if (d >= 65536u) {
        // quotient < 2^16: a single-precision reciprocal (relative error < 2^-21) lands within one of
        // it; the exact remainder 2^32 - q d says which way to step
        uint32_t q = (uint32_t)(4294967296.0f * __builtin_amdgcn_rcpf((float)d));
        const int64_t rem = ((int64_t)1 << 32) - (int64_t)((uint64_t)q * d);
        if (rem < 0) --q;
        else if (rem >= (int64_t)d) ++q;
        return q;
    }
    const uint32_t q = 0xFFFFFFFFu / d, r = 0xFFFFFFFFu - q * d;   // 2^32 = (2^32 - 1) + 1
    return (uint64_t)q + (r == d - 1u ? 1u : 0u);
}

constexpr int kTileRows = 8;                      // registers of tile sums per lane
constexpr int kMaxTiles = kTileRows * kWave;      // tile sums per root
constexpr int kListThreads = 256;                 // block of the finder that reads whole lists

// One block of four wavefronts per root: the weights 1/(t - ts) depend on the query,
// so the whole valid list has to be read once per root (from a plain array of the
// timestamps: half the bytes of the 16-byte records), and one wavefront walking a
// long list alone waits out a memory round trip every few rows. The list is cut
// into at most 512 tiles of whole 64-entry rows; in pass 1 the waves take the
// tiles in turn and leave every tile's weight sum in LDS. The first wave then holds
// the sums in registers (tile i in lane i % 64, register i / 64) and makes the k
// draws: each walks the tile sums, re-reads only the tile it lands in, and takes the
// picked weight out of the tile's sum, so a draw costs one tile, not the list.
__global__ __launch_bounds__(kListThreads) void sample_hop_inverse_timespan_kernel(
    const int64_t* __restrict__ indptr, const TaserRec* __restrict__ rec, const int64_t* __restrict__ ts_only,
    const TaserTimeIndex index, const int32_t* __restrict__ roots,
    const int64_t* __restrict__ times, int64_t num_roots, int32_t num_nodes, int k, uint32_t seed_lo, uint32_t seed_hi,
    uint32_t hop, int32_t* __restrict__ o_nbr, int32_t* __restrict__ o_eid, int64_t* __restrict__ o_ts,
    int32_t* __restrict__ o_count) {
    __shared__ uint64_t tile_sum_shared[kMaxTiles];
    __shared__ int64_t cnt_shared;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    const int64_t q = blockIdx.x;   // the grid has exactly one block per root

    int64_t lo = 0, hi = 0, t = 0;
    const int32_t v = roots[q];
    if (v >= 0 && v < num_nodes) {
        t = times[q];
        lo = indptr[v];
        hi = indptr[v + 1];
    }
    if (wave == 0) {   // wave-uniform: the search's ballots stay inside the first wave
        const int64_t c = group_cutoff<kWave>(rec, index, lo, hi, t, 0, lane);
        if (lane == 0) cnt_shared = c;
    }
    __syncthreads();
    const int64_t cnt = cnt_shared;
    const int64_t out0 = q * k;
    const TaserRec pad = {0, -1, -1};
    if (cnt <= k) {   // everything, most recent first (block-uniform)
        if (wave == 0) {
            if (lane < k) store_slot(o_nbr, o_eid, o_ts, out0 + lane, lane < cnt ? rec[lo + cnt - 1 - lane] : pad);
            if (lane == 0) o_count[q] = (int32_t)cnt;
        }
        return;
    }

    const int64_t rows = (cnt + kWave - 1) / kWave;                 // 64-entry rows of the valid list
    // Rows per tile: every tile costs pass 1 a wave-wide reduction, every draw re-reads about half
    // a tile with a wave-wide scan per row; the sum is smallest near sqrt(1.2 rows / k). The tiling
    // never changes a result, only the cost. At most kMaxTiles tiles.
    int64_t rows_per_tile = (int64_t)__builtin_sqrtf(1.2f * (float)rows / (float)k);
    if (rows_per_tile < 1) rows_per_tile = 1;
    if (rows_per_tile * kMaxTiles < rows) rows_per_tile = (rows + kMaxTiles - 1) / kMaxTiles;
    const int tiles = (int)((rows + rows_per_tile - 1) / rows_per_tile);
    const int tile_rows = (tiles + kWave - 1) / kWave;              // registers in use

    // Pass 1: tile sums, the waves taking tiles in turn.
    for (int tile = wave; tile < tiles; tile += kListThreads / kWave) {
        const int64_t r0 = (int64_t)tile * rows_per_tile;
        const int64_t r1 = r0 + rows_per_tile < rows ? r0 + rows_per_tile : rows;
        uint64_t s = 0;
        int64_t r = r0;
        for (; r + 4 <= r1; r += 4) {   // four independent loads in flight
            int64_t ts4[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int64_t p = (r + i) * kWave + lane;
                ts4[i] = ts_only[lo + (p < cnt ? p : cnt - 1)];
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if ((r + i) * kWave + lane < cnt) s += inverse_timespan_weight(t, ts4[i]);
        }
        for (; r < r1; ++r) {
            const int64_t p = r * kWave + lane;
            if (p < cnt) s += inverse_timespan_weight(t, ts_only[lo + p]);
        }
        s = wave_sum64(s);
        if (lane == 0) tile_sum_shared[tile] = s;
    }
    __syncthreads();
    if (wave != 0) return;   // the draws are one wavefront's work

    uint64_t tile_sum[kTileRows];
    uint64_t total = 0;
#pragma unroll
    for (int i = 0; i < kTileRows; ++i) {
        const int tile = i * kWave + lane;
        tile_sum[i] = tile < tiles ? tile_sum_shared[tile] : 0;
        total += tile_sum[i];
    }
    total = wave_sum64(total);

    // k successive draws; lane j keeps the position picked by draw j.
    uint64_t u = 0;
    if (lane < k) u = draw64(seed_lo, seed_hi, hop, (uint64_t)q, (uint32_t)lane);
    int64_t my_pick = 0;
    for (int j = 0; j < k; ++j) {
        uint64_t x = __umul64hi(wave_get64(u, j), total);
        // the tile whose running sum first exceeds x
        uint64_t before = 0;
        int tile = -1;
#pragma unroll
        for (int i = 0; i < kTileRows; ++i) {
            if (i < tile_rows && tile < 0) {
                const uint64_t inc = wave_inclusive_scan64(tile_sum[i]);
                const uint64_t hit = __ballot(before + inc > x);
                if (hit) {
                    const int first = __ffsll((long long)hit) - 1;
                    x -= before + wave_get64(inc - tile_sum[i], first);
                    tile = i * kWave + first;
                } else {
                    before += wave_get64(inc, kWave - 1);
                }
            }
        }
        if (tile < 0) tile = tiles - 1;   // cannot happen while the sums are consistent (x < total); keeps reads in bounds
        // inside the tile, row by row; entries picked by earlier draws weigh nothing
        const int64_t r0 = (int64_t)tile * rows_per_tile;
        const int64_t r1 = r0 + rows_per_tile < rows ? r0 + rows_per_tile : rows;
        before = 0;
        int64_t pick = -1;
        uint64_t pick_w = 0;
        for (int64_t r = r0; r < r1 && pick < 0; ++r) {
            const int64_t p = r * kWave + lane;
            uint64_t w = 0;
            if (p < cnt) w = inverse_timespan_weight(t, ts_only[lo + p]);
            for (int e = 0; e < j; ++e) {
                const uint64_t taken = wave_get64((uint64_t)my_pick, e);
                if ((uint64_t)p == taken) w = 0;
            }
            const uint64_t inc = wave_inclusive_scan64(w);
            const uint64_t hit = __ballot(before + inc > x);
            if (hit) {
                const int first = __ffsll((long long)hit) - 1;
                pick = r * kWave + first;
                pick_w = wave_get64(w, first);
            } else {
                before += wave_get64(inc, kWave - 1);
            }
        }
        if (pick < 0) pick = cnt - 1;     // same remark
        if (lane == j) my_pick = pick;
        total -= pick_w;
#pragma unroll
        for (int i = 0; i < kTileRows; ++i)
            if (i == (tile >> 6) && lane == (tile & (kWave - 1))) tile_sum[i] -= pick_w;
    }
    if (lane < k) store_slot(o_nbr, o_eid, o_ts, out0 + lane, rec[lo + my_pick]);
    if (lane == 0) o_count[q] = k;
}

__global__ __launch_bounds__(kThreads) void timestamps_only_kernel(const TaserRec* __restrict__ rec, int64_t n,
                                                                   int64_t* __restrict__ ts_only) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i < n) ts_only[i] = rec[i].ts;
}

// The plain timestamp array of a graph, made on the first call that needs it. The
// call that makes it waits for the fill, so later calls on any stream find it ready.
std::mutex g_ts_only_mutex;
int ensure_ts_only(const taser_tcsr* g_const, hipStream_t stream) {
    taser_tcsr* g = const_cast<taser_tcsr*>(g_const);   // a cache inside the handle, not a change of the graph
    std::lock_guard<std::mutex> lock(g_ts_only_mutex);
    if (g->ts_only || g->num_entries == 0) return TASER_OK;
    int64_t* p = nullptr;
    TASER_HIP_TRY(hipMalloc((void**)&p, (size_t)g->num_entries * sizeof(int64_t)));
    hipLaunchKernelGGL(timestamps_only_kernel, dim3((unsigned)((g->num_entries + kThreads - 1) / kThreads)), dim3(kThreads),
                       0, stream, g->rec, g->num_entries, p);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) e = hipStreamSynchronize(stream);
    if (e != hipSuccess) {
        (void)hipFree(p);
        return taser_fail_hip(e, "sample_temporal: building the timestamp array");
    }
    g->ts_only = p;
    return TASER_OK;
}

template <int POLICY, int G, int kRootsPerGroup, bool ROWS>
void launch_hop_gr(const taser_tcsr* g, const int32_t* roots, const int64_t* times, int64_t n, int k,
                   uint64_t seed, uint32_t hop, int m, const uint32_t* edge_weight, const taser_hop_out& o,
                   const RowCopy& rows, hipStream_t stream) {
    constexpr int roots_per_block = (kThreads / kWave) * (kWave / G) * kRootsPerGroup;
    const unsigned grid = (unsigned)((n + roots_per_block - 1) / roots_per_block);
    hipLaunchKernelGGL((sample_hop_kernel<POLICY, G, kRootsPerGroup, ROWS>), dim3(grid), dim3(kThreads), 0, stream, g->indptr, g->rec, g->time_index,
                       roots, times, n, g->num_nodes, k, (uint32_t)seed, (uint32_t)(seed >> 32), hop, m, edge_weight, o.nbr,
                       o.eid, o.ts, o.count, rows);
}

template <int POLICY, int G>
void launch_hop_g(const taser_tcsr* g, const int32_t* roots, const int64_t* times, int64_t n, int k,
                  uint64_t seed, uint32_t hop, int m, const uint32_t* edge_weight, const taser_hop_out& o,
                  const RowCopy* rows, hipStream_t stream) {
    if (rows) launch_hop_gr<POLICY, G, 1, true>(g, roots, times, n, k, seed, hop, m, edge_weight, o, *rows, stream);
    else if (POLICY == TASER_RECENT && n >= 65536) launch_hop_gr<POLICY, G, 2, false>(g, roots, times, n, k, seed, hop, m, edge_weight, o, RowCopy{}, stream);
    else launch_hop_gr<POLICY, G, 1, false>(g, roots, times, n, k, seed, hop, m, edge_weight, o, RowCopy{}, stream);
}

// Lanes of a wavefront that serve one root.
int group_lanes(int policy, int k, int m) {
    const int lanes = (policy == TASER_WEIGHTED && m > k) ? m : k;   // lanes a root needs
    return lanes <= 16 ? 16 : lanes <= 32 ? 32 : 64;
}

template <int POLICY>
void launch_hop(const taser_tcsr* g, const int32_t* roots, const int64_t* times, int64_t n, int k,
                uint64_t seed, uint32_t hop, int m, const uint32_t* edge_weight,
                const taser_hop_out& o, const RowCopy* rows, hipStream_t stream) {
    static const char* const names[2][3] = {{"sample_hop_recent", "sample_hop_uniform", "sample_hop_weighted"},
                                            {"sample_rows_hop_recent", "sample_rows_hop_uniform", "sample_rows_hop_weighted"}};
    TaserProfileSpan span(stream, names[rows ? 1 : 0][POLICY]);
    const int lanes = group_lanes(POLICY, k, m);
    if (lanes == 16) launch_hop_g<POLICY, 16>(g, roots, times, n, k, seed, hop, m, edge_weight, o, rows, stream);
    else if (lanes == 32) launch_hop_g<POLICY, 32>(g, roots, times, n, k, seed, hop, m, edge_weight, o, rows, stream);
    else launch_hop_g<POLICY, 64>(g, roots, times, n, k, seed, hop, m, edge_weight, o, rows, stream);
}

// The feature table a call wants sliced along with the sampling (null table: none).
struct RowRequest {
    const void* table;
    int64_t table_rows;
    int32_t row_bytes;
    int64_t pitch_bytes;
    void* const* out;   // per hop
};

int check_sampling_arguments(const char* what, const taser_tcsr* g, const int32_t* roots, const int64_t* times,
                             int64_t num_roots, int32_t k, int32_t hops, int32_t policy, int32_t m,
                             const uint32_t* edge_weight, const taser_hop_out* out) {
    if (!g || !out) return taser_fail(TASER_E_ARG, "%s: null graph or output array", what);
    if (num_roots < 0) return taser_fail(TASER_E_ARG, "%s: num_roots = %lld", what, (long long)num_roots);
    if (num_roots > 0 && (!roots || !times)) return taser_fail(TASER_E_ARG, "%s: null roots/times", what);
    if (k < 1 || k > TASER_MAX_K) return taser_fail(TASER_E_RANGE, "%s: k = %d outside [1, %d]", what, k, TASER_MAX_K);
    if (hops < 1 || hops > TASER_MAX_HOPS) return taser_fail(TASER_E_RANGE, "%s: hops = %d outside [1, %d]", what, hops, TASER_MAX_HOPS);
    if (policy != TASER_RECENT && policy != TASER_UNIFORM && policy != TASER_WEIGHTED && policy != TASER_INVERSE_TIMESPAN)
        return taser_fail(TASER_E_ARG, "%s: unknown policy %d", what, policy);
    if (policy == TASER_WEIGHTED) {
        if (m < 1 || m > TASER_MAX_M) return taser_fail(TASER_E_RANGE, "%s: m = %d outside [1, %d]", what, m, TASER_MAX_M);
        if (!edge_weight) return taser_fail(TASER_E_ARG, "%s: weighted policy needs edge_weight", what);
    }
    int64_t n = num_roots;
    for (int h = 0; h < hops; ++h) {
        if (n > 0 && (!out[h].nbr || !out[h].eid || !out[h].ts || !out[h].count))
            return taser_fail(TASER_E_ARG, "%s: null output buffer at hop %d", what, h);
        if (n * k >= ((int64_t)1 << 31)) return taser_fail(TASER_E_RANGE, "%s: num_roots * k^hops must stay below 2^31", what);
        n *= k;
    }
    return TASER_OK;
}

// A wavefront copies the rows of its own roots only while they are few bytes: all wavefronts
// of a launch search at the same time and then copy at the same time, so the two phases add up
// instead of overlapping, and for long rows the plain gather (one launch for all hops) moves
// the same bytes faster. Measured on 2 x 10 slots per root: up to 8 KiB per wavefront the hop
// kernel's own copy is as fast or faster (64-byte rows: 41 against 49 us per batch of 4 000
// roots, 25 against 29 us with 16 lanes per root), beyond it up to 15 % slower.
constexpr int64_t kFinderCopyMaxWaveBytes = 8192;

// All hops of one call. With `want`, hop h also leaves the table rows of its sampled edges in
// want->out[h]: written by the hop kernel where the shapes allow it and the rows are short, else
// by the plain gather launched after the last hop (same bytes either way), one launch for
// consecutive hops whose edge ids and row buffers follow one another in memory.
int sample_hops(const taser_tcsr* g, const int32_t* roots, const int64_t* times, int64_t num_roots, int32_t k,
                int32_t hops, int32_t policy, uint64_t seed, int32_t m, const uint32_t* edge_weight,
                const taser_hop_out* out, const RowRequest* want, hipStream_t stream) {
    taser_clear_stale_hip_error();
    if (policy == TASER_INVERSE_TIMESPAN) {
        const int rc = ensure_ts_only(g, stream);
        if (rc != TASER_OK) return rc;
    }
    const int32_t* cur_roots = roots;
    const int64_t* cur_times = times;
    int64_t n = num_roots;
    struct Pending {
        const int32_t* ids;
        int64_t n;
        uint8_t* out;
    } pending[TASER_MAX_HOPS];
    int n_pending = 0;
    for (int h = 0; h < hops && n > 0; ++h) {
        // Can this hop's kernel write the rows itself? It copies per wavefront, in aligned 16-byte
        // pieces read at 4-byte alignment: rows, pitch and table must allow that, and the rows of
        // one wavefront's roots must be whole 16-byte pieces.
        RowCopy copy{};
        const RowCopy* rows = nullptr;
        if (want && policy != TASER_INVERSE_TIMESPAN) {
            const int64_t wave_bytes = (int64_t)(kWave / group_lanes(policy, k, m)) * k * want->row_bytes;
            const uint64_t bits = (uint64_t)want->row_bytes | (uint64_t)want->pitch_bytes | (uint64_t)(uintptr_t)want->table;
            if (want->row_bytes >= 16 && wave_bytes <= kFinderCopyMaxWaveBytes && (bits & 3) == 0 && (wave_bytes & 15) == 0 &&
                ((uintptr_t)want->out[h] & 15) == 0) {
                const uint8_t* zeros = taser_gather::zero_chunk();
                if (!zeros) return taser_fail(TASER_E_HIP, "sample_temporal_rows: the zero constant is not available on this device");
                const uint32_t rb = (uint32_t)want->row_bytes;
                copy = RowCopy{static_cast<const uint8_t*>(want->table), want->table_rows, want->pitch_bytes,
                               static_cast<uint8_t*>(want->out[h]), zeros, rb, (uint32_t)((((uint64_t)1 << 32) + rb - 1) / rb),
                               1024u / rb, 1024u % rb};
                rows = &copy;
            }
        }
        switch (policy) {
            case TASER_RECENT: launch_hop<TASER_RECENT>(g, cur_roots, cur_times, n, k, seed, (uint32_t)h, m, edge_weight, out[h], rows, stream); break;
            case TASER_UNIFORM: launch_hop<TASER_UNIFORM>(g, cur_roots, cur_times, n, k, seed, (uint32_t)h, m, edge_weight, out[h], rows, stream); break;
            case TASER_INVERSE_TIMESPAN: {
                TaserProfileSpan span(stream, "sample_hop_inverse_timespan");
                const unsigned grid = (unsigned)n;   // one block per root (n < 2^31)
                hipLaunchKernelGGL(sample_hop_inverse_timespan_kernel, dim3(grid), dim3(kListThreads), 0, stream, g->indptr, g->rec,
                                   g->ts_only, g->time_index, cur_roots, cur_times, n, g->num_nodes, k, (uint32_t)seed, (uint32_t)(seed >> 32),
                                   (uint32_t)h, out[h].nbr, out[h].eid, out[h].ts, out[h].count);
                break;
            }
            default: launch_hop<TASER_WEIGHTED>(g, cur_roots, cur_times, n, k, seed, (uint32_t)h, m, edge_weight, out[h], rows, stream); break;
        }
        if (want && !rows) {
            uint8_t* to = static_cast<uint8_t*>(want->out[h]);
            Pending* last = n_pending ? &pending[n_pending - 1] : nullptr;
            if (last && last->ids + last->n == out[h].eid && last->out + last->n * want->row_bytes == to) last->n += n * k;
            else pending[n_pending++] = Pending{out[h].eid, n * k, to};
        }
        cur_roots = out[h].nbr;
        cur_times = out[h].ts;
        n *= k;
    }
    TASER_HIP_TRY(hipGetLastError());
    for (int i = 0; i < n_pending; ++i) {
        const int rc = taser_launch_gather(want->table, want->table_rows, want->row_bytes, want->pitch_bytes, pending[i].ids, pending[i].n,
                                           pending[i].out, stream);
        if (rc != TASER_OK) return rc;
    }
    return TASER_OK;
}

}  // namespace

extern "C" int taser_sample_temporal(const taser_tcsr* g, const int32_t* roots, const int64_t* times,
                                     int64_t num_roots, int32_t k, int32_t hops, int32_t policy,
                                     uint64_t seed, int32_t m, const uint32_t* edge_weight,
                                     const taser_hop_out* out, void* hip_stream) {
    const int rc = check_sampling_arguments("sample_temporal", g, roots, times, num_roots, k, hops, policy, m, edge_weight, out);
    if (rc != TASER_OK) return rc;
    return sample_hops(g, roots, times, num_roots, k, hops, policy, seed, m, edge_weight, out, nullptr, (hipStream_t)hip_stream);
}

extern "C" int taser_sample_temporal_rows(const taser_tcsr* g, const int32_t* roots, const int64_t* times,
                                          int64_t num_roots, int32_t k, int32_t hops, int32_t policy,
                                          uint64_t seed, int32_t m, const uint32_t* edge_weight,
                                          const void* table, int64_t table_rows, int32_t row_bytes, int64_t pitch_bytes,
                                          const taser_hop_out* out, void* const* rows_out, void* hip_stream) {
    const char* what = "sample_temporal_rows";
    const int rc = check_sampling_arguments(what, g, roots, times, num_roots, k, hops, policy, m, edge_weight, out);
    if (rc != TASER_OK) return rc;
    if (table_rows < 0) return taser_fail(TASER_E_ARG, "%s: negative table_rows", what);
    if (row_bytes <= 0 || (row_bytes & 1)) return taser_fail(TASER_E_ARG, "%s: row_bytes = %d must be positive and even", what, row_bytes);
    if (pitch_bytes < row_bytes || (pitch_bytes & 1)) return taser_fail(TASER_E_ARG, "%s: pitch_bytes = %lld must be even and >= row_bytes", what, (long long)pitch_bytes);
    if (!table && table_rows > 0) return taser_fail(TASER_E_ARG, "%s: null table", what);
    if ((uintptr_t)table & 1) return taser_fail(TASER_E_ARG, "%s: table must be 2-byte aligned", what);
    if (!rows_out) return taser_fail(TASER_E_ARG, "%s: null rows_out", what);
    int64_t n = num_roots;
    for (int h = 0; h < hops; ++h) {
        if (n > 0 && !rows_out[h]) return taser_fail(TASER_E_ARG, "%s: null row buffer at hop %d", what, h);
        if ((uintptr_t)rows_out[h] & 1) return taser_fail(TASER_E_ARG, "%s: row buffers must be 2-byte aligned", what);
        n *= k;
    }
    const RowRequest want{table, table_rows, row_bytes, pitch_bytes, rows_out};
    return sample_hops(g, roots, times, num_roots, k, hops, policy, seed, m, edge_weight, out, &want, (hipStream_t)hip_stream);
}
