/*
 * CPU ORACLE — TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, single-purpose implementation of what the temporal neighbor
 * finder + feature gather of TASER (arXiv 2402.05396) computes. It exists so
 * the HIP path can be checked against something written independently of it:
 * it shares no source, header, table or helper with the HIP library, and only
 * tests, the smoke check and the benchmark's CPU-baseline leg may load it.
 *
 * Every function cites the passage of the paper it follows. Where the paper
 * fixes a plain definition (time-sorted per-node lists, "neighbors strictly
 * before t", "the most recent ones", "copy the feature row") the oracle is
 * that definition written out. Where the paper only fixes a distribution
 * (uniform / weighted selection without replacement) the oracle is one stated
 * seeded procedure with that distribution, taken step by step.
 *
 * Pins (tests/test_oracle_*.py): Philox known-answer vectors, numpy.lexsort,
 * numpy.searchsorted, pure-Python brute force from the raw event list,
 * explicit-array Fisher-Yates, closed-form successive-sampling probabilities
 * and chi-square tests, numpy.take, numpy.cumsum + searchsorted, the real-valued
 * 1/delta law, sequential Python replays. No function here is unpinned.
 *
 * Precision: all selection arithmetic is integer (the paper states none);
 * feature rows are copied as bytes.
 */
#include <algorithm>
#include <cstdint>
#include <cstring>
#include <unordered_map>
#include <vector>
#ifdef _OPENMP
#include <omp.h>
#include <parallel/algorithm>
#endif

namespace {

/* ---- Counter-based generator: Philox4x32 with 10 rounds -----------------
 * Salmon, Moraes, Dror, Shaw, "Parallel random numbers: as easy as 1, 2, 3"
 * (SC'11), the Philox-4x32 bijection: each round replaces the counter
 * (c0,c1,c2,c3) by (hi(M1*c2)^c1^k0, lo(M1*c2), hi(M0*c0)^c3^k1, lo(M0*c0))
 * and the key is advanced by the Weyl constants between rounds. */
const uint32_t PHILOX_M0 = 0xD2511F53u;
const uint32_t PHILOX_M1 = 0xCD9E8D57u;
const uint32_t PHILOX_W0 = 0x9E3779B9u;
const uint32_t PHILOX_W1 = 0xBB67AE85u;

void philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        if (round > 0) {
            k0 += PHILOX_W0;
            k1 += PHILOX_W1;
        }
        const uint64_t p0 = (uint64_t)PHILOX_M0 * c0;
        const uint64_t p1 = (uint64_t)PHILOX_M1 * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n1 = (uint32_t)p1;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        const uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* One 64-bit draw per (seed, hop, root index, slot): key = seed split in two
 * words, counter = (root low, root high, slot, hop), result = words 1:0. */
uint64_t draw64(uint64_t seed, uint32_t hop, uint64_t root, uint32_t slot) {
    const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    const uint32_t ctr[4] = {(uint32_t)root, (uint32_t)(root >> 32), slot, hop};
    uint32_t out[4];
    philox4x32_10(ctr, key, out);
    return ((uint64_t)out[1] << 32) | out[0];
}

/* floor(u * n / 2^64): maps a 64-bit draw onto [0, n). */
uint64_t mulhi64(uint64_t u, uint64_t n) {
    return (uint64_t)(((unsigned __int128)u * n) >> 64);
}

struct SortKey {
    int32_t src;
    int64_t ts;
    int64_t pos;
};

bool key_less(const SortKey& a, const SortKey& b) {
    if (a.src != b.src) return a.src < b.src;
    if (a.ts != b.ts) return a.ts < b.ts;
    return a.pos < b.pos;
}

const int32_t PAD_ID = -1;

}  // namespace

extern "C" {

void oracle_philox4x32_10(const uint32_t* ctr, const uint32_t* key, uint32_t* out) {
    philox4x32_10(ctr, key, out);
}

uint64_t oracle_draw64(uint64_t seed, uint32_t hop, uint64_t root, uint32_t slot) {
    return draw64(seed, hop, root, slot);
}

uint64_t oracle_mulhi64(uint64_t u, uint64_t n) { return mulhi64(u, n); }

int oracle_max_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* T-CSR (paper Sec. 3.3: per-node outgoing neighbor lists sorted by
 * timestamp; Sec. 2.1: N(v,t) is defined over edges leaving v).
 * Entries are ordered by (src, ts, input position) — a total order, so the
 * result is unique. indptr[v] = number of entries whose src is below v.
 * threads == 1 uses std::sort; threads > 1 hands the same comparator to
 * libstdc++'s parallel sort (same result, the order is total).
 * Returns 0, or -1 if a node id is outside [0, num_nodes). */
int oracle_tcsr_build(const int32_t* src, const int32_t* dst, const int64_t* ts,
                      const int32_t* eid, int64_t num_entries, int32_t num_nodes,
                      int64_t* indptr, int32_t* out_nbr, int64_t* out_ts, int32_t* out_eid,
                      int threads) {
    for (int64_t i = 0; i < num_entries; ++i)
        if (src[i] < 0 || src[i] >= num_nodes) return -1;
    std::vector<SortKey> keys((size_t)num_entries);
    for (int64_t i = 0; i < num_entries; ++i) keys[(size_t)i] = SortKey{src[i], ts[i], i};
#ifdef _OPENMP
    if (threads > 1) {
        omp_set_num_threads(threads);
        __gnu_parallel::sort(keys.begin(), keys.end(), key_less);
    } else {
        std::sort(keys.begin(), keys.end(), key_less);
    }
#else
    (void)threads;
    std::sort(keys.begin(), keys.end(), key_less);
#endif
    for (int32_t v = 0; v <= num_nodes; ++v) indptr[v] = 0;
    for (int64_t i = 0; i < num_entries; ++i) indptr[src[i] + 1] += 1;
    for (int32_t v = 0; v < num_nodes; ++v) indptr[v + 1] += indptr[v];
    for (int64_t p = 0; p < num_entries; ++p) {
        const int64_t i = keys[(size_t)p].pos;
        out_nbr[p] = dst[i];
        out_ts[p] = ts[i];
        out_eid[p] = eid ? eid[i] : (int32_t)i;
    }
    return 0;
}

/* One hop of temporal neighbor finding (paper Sec. 2.1 and Alg. 2).
 *
 * For root index q with node v = roots[q] and query time t = times[q]:
 *   cnt = number of entries of v's list with ts < t (strict, Sec. 2.1),
 *         counted by scanning the whole list; the list is time-sorted, so
 *         these are its first cnt entries.
 *   policy 0 (most recent, Sec. 2.1 / Alg. 2): slot j takes entry cnt-1-j.
 *   policy 1 (uniform without replacement, Sec. 2.1 / Alg. 2): when cnt <= k
 *         all cnt entries are returned in most-recent order; otherwise a
 *         partial Fisher-Yates shuffle of the positions 0..cnt-1 with one
 *         draw per slot: r = j + floor(draw(seed,hop,q,j) * (cnt-j) / 2^64).
 *   policy 2 (weighted, Alg. 1 second sampling line): candidates are the
 *         c = min(m, cnt) most recent entries, candidate i = entry cnt-1-i,
 *         weight w_i = edge_weight[eid_i] >= 1. When c <= k all candidates
 *         are returned in candidate order; otherwise k successive draws
 *         without replacement, each proportional to the remaining weights:
 *         x = floor(draw * W / 2^64) with W the remaining total, pick the
 *         first remaining candidate whose running weight sum exceeds x.
 *   policy 3 (inverse timespan, the heuristic sampler of TGAT that the paper's
 *         introduction and related work describe: past neighbors are sampled
 *         with probabilities inversely proportional to their time deltas):
 *         over ALL cnt valid entries, entry p has the integer weight
 *         w_p = max(1, floor(2^32 / (t - ts[p]))) (t - ts[p] >= 1 by the strict
 *         cutoff). When cnt <= k all entries are returned in most-recent
 *         order; otherwise k successive draws without replacement as in
 *         policy 2, the running sum taken in list order (oldest entry first).
 * A root with roots[q] < 0 (padding from the previous hop) has no neighbors.
 * Unused slots hold nbr = -1, eid = -1, ts = 0; count[q] = slots filled.
 * Returns 0, -1 on a bad argument. */
int oracle_sample_hop(const int64_t* indptr, const int32_t* nbr, const int64_t* ts,
                      const int32_t* eid, int32_t num_nodes, const int32_t* roots,
                      const int64_t* times, int64_t num_roots, int32_t k, int32_t policy,
                      uint64_t seed, uint32_t hop, int32_t m, const uint32_t* edge_weight,
                      int32_t* out_nbr, int32_t* out_eid, int64_t* out_ts, int32_t* out_count,
                      int threads) {
    if (k < 1 || policy < 0 || policy > 3) return -1;
    if (policy == 2 && (edge_weight == nullptr || m < 1)) return -1;
    int bad = 0;
#ifdef _OPENMP
#pragma omp parallel for schedule(static) reduction(| : bad) num_threads(threads > 1 ? threads : 1)
#else
    (void)threads;
#endif
    for (int64_t q = 0; q < num_roots; ++q) {
        int32_t* o_nbr = out_nbr + q * k;
        int32_t* o_eid = out_eid + q * k;
        int64_t* o_ts = out_ts + q * k;
        for (int32_t j = 0; j < k; ++j) {
            o_nbr[j] = PAD_ID;
            o_eid[j] = PAD_ID;
            o_ts[j] = 0;
        }
        out_count[q] = 0;
        const int32_t v = roots[q];
        if (v < 0) continue;
        if (v >= num_nodes) {
            bad = 1;
            continue;
        }
        const int64_t t = times[q];
        const int64_t lo = indptr[v], hi = indptr[v + 1];
        int64_t cnt = 0;
        for (int64_t p = lo; p < hi; ++p)
            if (ts[p] < t) ++cnt;

        std::vector<int64_t> pick;  // positions inside the list, one per filled slot
        if (policy == 0 || ((policy == 1 || policy == 3) && cnt <= k)) {
            const int64_t c = std::min<int64_t>(k, cnt);
            for (int64_t j = 0; j < c; ++j) pick.push_back(cnt - 1 - j);
        } else if (policy == 1) {
            std::unordered_map<int64_t, int64_t> moved;  // a[x] where it differs from x
            auto a = [&](int64_t x) {
                auto it = moved.find(x);
                return it == moved.end() ? x : it->second;
            };
            for (int32_t j = 0; j < k; ++j) {
                const uint64_t u = draw64(seed, hop, (uint64_t)q, (uint32_t)j);
                const int64_t r = j + (int64_t)mulhi64(u, (uint64_t)(cnt - j));
                const int64_t chosen = a(r);
                moved[r] = a(j);
                pick.push_back(chosen);
            }
        } else if (policy == 3) {
            std::vector<uint64_t> w((size_t)cnt);
            for (int64_t p = 0; p < cnt; ++p) {
                const uint64_t delta = (uint64_t)t - (uint64_t)ts[lo + p];   // exact: t > ts[lo + p]
                const uint64_t inv = (uint64_t)(((unsigned __int128)1 << 32) / delta);
                w[(size_t)p] = inv < 1 ? 1 : inv;
            }
            for (int32_t j = 0; j < k; ++j) {
                uint64_t W = 0;
                for (int64_t p = 0; p < cnt; ++p) W += w[(size_t)p];
                const uint64_t x = mulhi64(draw64(seed, hop, (uint64_t)q, (uint32_t)j), W);
                uint64_t running = 0;
                int64_t chosen = -1;
                for (int64_t p = 0; p < cnt; ++p) {
                    running += w[(size_t)p];
                    if (running > x) {
                        chosen = p;
                        break;
                    }
                }
                w[(size_t)chosen] = 0;
                pick.push_back(chosen);
            }
        } else {
            const int64_t c = std::min<int64_t>(m, cnt);
            if (c <= k) {
                for (int64_t i = 0; i < c; ++i) pick.push_back(cnt - 1 - i);
            } else {
                std::vector<uint64_t> w((size_t)c);
                for (int64_t i = 0; i < c; ++i) w[(size_t)i] = edge_weight[eid[lo + cnt - 1 - i]];
                for (int32_t j = 0; j < k; ++j) {
                    uint64_t W = 0;
                    for (int64_t i = 0; i < c; ++i) W += w[(size_t)i];
                    const uint64_t x = mulhi64(draw64(seed, hop, (uint64_t)q, (uint32_t)j), W);
                    uint64_t running = 0;
                    int64_t chosen = -1;
                    for (int64_t i = 0; i < c; ++i) {
                        running += w[(size_t)i];
                        if (running > x) {
                            chosen = i;
                            break;
                        }
                    }
                    w[(size_t)chosen] = 0;
                    pick.push_back(cnt - 1 - chosen);
                }
            }
        }
        for (size_t j = 0; j < pick.size(); ++j) {
            const int64_t p = lo + pick[j];
            o_nbr[j] = nbr[p];
            o_eid[j] = eid[p];
            o_ts[j] = ts[p];
        }
        out_count[q] = (int32_t)pick.size();
    }
    return bad ? -1 : 0;
}

/* Multi-hop expansion (paper Alg. 1, loop over layers: the neighbors kept
 * at one layer become the next layer's target nodes). Hop h+1 has one root
 * per slot of hop h: root index i*k+j, node = sampled neighbor, query time =
 * the sampled interaction's own timestamp; an empty slot stays empty.
 * out_* are arrays of `hops` pointers: hop h holds R*k^h roots. */
int oracle_sample_temporal(const int64_t* indptr, const int32_t* nbr, const int64_t* ts,
                           const int32_t* eid, int32_t num_nodes, const int32_t* roots,
                           const int64_t* times, int64_t num_roots, int32_t k, int32_t hops,
                           int32_t policy, uint64_t seed, int32_t m, const uint32_t* edge_weight,
                           int32_t** out_nbr, int32_t** out_eid, int64_t** out_ts,
                           int32_t** out_count, int threads) {
    const int32_t* cur_roots = roots;
    const int64_t* cur_times = times;
    int64_t cur_n = num_roots;
    for (int32_t h = 0; h < hops; ++h) {
        const int rc = oracle_sample_hop(indptr, nbr, ts, eid, num_nodes, cur_roots, cur_times,
                                         cur_n, k, policy, seed, (uint32_t)h, m, edge_weight,
                                         out_nbr[h], out_eid[h], out_ts[h], out_count[h], threads);
        if (rc != 0) return rc;
        cur_roots = out_nbr[h];
        cur_times = out_ts[h];
        cur_n *= k;
    }
    return 0;
}

/* Feature slicing (paper Sec. 3.4 / Alg. 3, "serve x_e"): out row i is the
 * row_bytes bytes of table row ids[i]; a negative id gives a zero row. The
 * served bytes do not depend on where the row lives, so the device cache is
 * invisible here. Returns -1 if an id is >= rows. */
int oracle_gather(const uint8_t* table, int64_t rows, int32_t row_bytes, int64_t pitch_bytes,
                  const int32_t* ids, int64_t n, uint8_t* out, int threads) {
    int bad = 0;
#ifdef _OPENMP
#pragma omp parallel for schedule(static) reduction(| : bad) num_threads(threads > 1 ? threads : 1)
#else
    (void)threads;
#endif
    for (int64_t i = 0; i < n; ++i) {
        uint8_t* o = out + i * (int64_t)row_bytes;
        const int64_t id = ids[i];
        if (id < 0) {
            std::memset(o, 0, (size_t)row_bytes);
        } else if (id >= rows) {
            bad = 1;
        } else {
            std::memcpy(o, table + id * pitch_bytes, (size_t)row_bytes);
        }
    }
    return bad ? -1 : 0;
}

/* Initial cache content when none is given (paper Alg. 3: "randomly cache k
 * features"): the first `capacity` elements of a seeded partial Fisher-Yates
 * shuffle of 0..rows-1, one draw per element with hop tag 0x43414348 and the
 * element index as the root index. */
void oracle_cache_random_residents(int64_t rows, int64_t capacity, uint64_t seed, int32_t* out) {
    std::unordered_map<int64_t, int64_t> moved;
    auto a = [&](int64_t x) {
        auto it = moved.find(x);
        return it == moved.end() ? x : it->second;
    };
    for (int64_t j = 0; j < capacity; ++j) {
        const uint64_t u = draw64(seed, 0x43414348u, (uint64_t)j, 0u);
        const int64_t r = j + (int64_t)mulhi64(u, (uint64_t)(rows - j));
        const int64_t chosen = a(r);
        moved[r] = a(j);
        out[j] = (int32_t)chosen;
    }
}

/* Cache accounting (paper Sec. 3.4: a request is a hit when its row is in
 * the device cache): hit_miss[0] = requests whose id is resident,
 * hit_miss[1] = other requests with a valid id. Negative ids count as neither. */
void oracle_cache_hits(const int32_t* resident, int64_t capacity, int64_t rows,
                       const int32_t* ids, int64_t n, uint64_t* hit_miss) {
    std::vector<uint8_t> is_resident((size_t)rows, 0);
    for (int64_t i = 0; i < capacity; ++i) is_resident[(size_t)resident[i]] = 1;
    uint64_t hits = 0, misses = 0;
    for (int64_t i = 0; i < n; ++i) {
        if (ids[i] < 0) continue;
        if (is_resident[(size_t)ids[i]]) ++hits; else ++misses;
    }
    hit_miss[0] = hits;
    hit_miss[1] = misses;
}

/* Access counting (paper Alg. 3: Q[e] <- Q[e] + 1 for every read request e).
 * Requests with an id outside [0, rows) are not counted. */
void oracle_cache_count(const int32_t* ids, int64_t n, int64_t rows, uint32_t* Q) {
    for (int64_t i = 0; i < n; ++i)
        if (ids[i] >= 0 && ids[i] < rows) Q[ids[i]] += 1;
}

/* End of an epoch (paper Alg. 3 and Sec. 3.4): Q_topk = the `capacity` most
 * frequently requested rows of the epoch (ties: the smaller id wins). If fewer
 * than `min_overlap` of them are currently resident, the cache content becomes
 * Q_topk; otherwise it stays. Either way Q is cleared for the next epoch.
 * new_resident receives the resident ids after the step (Q_topk in ascending
 * id order when replaced, the old list unchanged otherwise); *overlap receives
 * |resident n Q_topk|. Returns 1 if the content was replaced, else 0. */
int oracle_cache_epoch_end(uint32_t* Q, int64_t rows, const int32_t* resident, int64_t capacity,
                           int64_t min_overlap, int32_t* new_resident, int64_t* overlap) {
    std::vector<int32_t> order((size_t)rows);
    for (int64_t i = 0; i < rows; ++i) order[(size_t)i] = (int32_t)i;
    std::sort(order.begin(), order.end(), [&](int32_t a, int32_t b) {
        if (Q[a] != Q[b]) return Q[a] > Q[b];
        return a < b;
    });
    std::vector<int32_t> topk(order.begin(), order.begin() + capacity);
    std::sort(topk.begin(), topk.end());
    int64_t both = 0;
    for (int64_t i = 0; i < capacity; ++i)
        if (std::binary_search(topk.begin(), topk.end(), resident[i])) ++both;
    *overlap = both;
    const int replace = both < min_overlap;
    for (int64_t i = 0; i < capacity; ++i) new_resident[i] = replace ? topk[(size_t)i] : resident[i];
    for (int64_t i = 0; i < rows; ++i) Q[i] = 0;
    return replace;
}

/* Candidate-window encodings of the adaptive sampler's neighbor encoder
 * (paper Sec. 3.2). For root i with candidates u_0..u_{c-1} (c = count[i] <= m,
 * most recent first):
 *   freq[i][j]        = number of candidates l < c with u_l == u_j  (the integer
 *                       freq(u) that the frequency encoding takes as input);
 *   identity[i][j][l] = 1 if u_j == u_l else 0, for j, l < c       (the identity
 *                       encoding IE_(u_j, l)).
 * Entries that involve a padding slot (j >= c or l >= c) are 0.
 * identity may be null. */
void oracle_candidate_encodings(const int32_t* nbr, const int32_t* count, int64_t num_roots, int32_t m,
                                int32_t* freq, uint8_t* identity) {
    for (int64_t i = 0; i < num_roots; ++i) {
        const int32_t* u = nbr + i * m;
        const int32_t c = count[i];
        for (int32_t j = 0; j < m; ++j) {
            int32_t f = 0;
            for (int32_t l = 0; l < m; ++l) {
                const int same = (j < c && l < c && u[j] == u[l]) ? 1 : 0;
                f += same;
                if (identity) identity[(i * m + j) * m + l] = (uint8_t)same;
            }
            freq[i * m + j] = f;
        }
    }
}

/* The second sampling line of Alg. 1 with a probability per (root, candidate):
 * root i has c = count[i] candidates (slots 0..c-1 of its row of `m`) with integer
 * weights weight[i][0..c-1] >= 1 (the quantised q(j|i)). If c <= k all candidates
 * are kept in order; otherwise k successive draws without replacement, each
 * proportional to the remaining weights, exactly as policy 2 of oracle_sample_hop:
 * x = floor(draw(seed, hop, i, j) * W / 2^64), first remaining candidate whose
 * running weight sum exceeds x. sel[i][j] = chosen candidate slot (or -1),
 * out_count[i] = number chosen. */
void oracle_select_weighted(const uint32_t* weight, const int32_t* count, int64_t num_roots, int32_t m,
                            int32_t k, uint64_t seed, uint32_t hop, int32_t* sel, int32_t* out_count) {
    for (int64_t i = 0; i < num_roots; ++i) {
        int32_t* s = sel + i * k;
        for (int32_t j = 0; j < k; ++j) s[j] = -1;
        const int32_t c = count[i] < m ? count[i] : m;
        if (c <= k) {
            for (int32_t j = 0; j < c; ++j) s[j] = j;
            out_count[i] = c < 0 ? 0 : c;
            continue;
        }
        std::vector<uint64_t> w((size_t)c);
        for (int32_t j = 0; j < c; ++j) w[(size_t)j] = weight[i * m + j];
        for (int32_t j = 0; j < k; ++j) {
            uint64_t W = 0;
            for (int32_t l = 0; l < c; ++l) W += w[(size_t)l];
            const uint64_t x = mulhi64(draw64(seed, hop, (uint64_t)i, (uint32_t)j), W);
            uint64_t running = 0;
            int32_t chosen = -1;
            for (int32_t l = 0; l < c; ++l) {
                running += w[(size_t)l];
                if (running > x) {
                    chosen = l;
                    break;
                }
            }
            w[(size_t)chosen] = 0;
            s[j] = chosen;
        }
        out_count[i] = k;
    }
}

/* Adaptive mini-batch selection (paper Sec. 3.1: a list of importance scores P
 * over the training edges, initialised uniformly; a batch of training edges is
 * sampled with probability proportional to the scores; after the forward pass
 * the scores of the batch's edges are overwritten).
 *
 * Scores are integers (the quantised sigmoid(y) + gamma of Eq. (4) is produced
 * outside this path). oracle_batch_draw makes b independent draws, draw j:
 *   x = floor(draw(seed, tag 0x4253454C, root = iteration, slot = j) * W / 2^64)
 * with W the sum of all scores, out[j] = the first edge whose running score sum
 * exceeds x (so P(out[j] = e) = score[e] / W up to 2^-64 rounding). W == 0 gives -1. */
void oracle_batch_draw(const uint32_t* score, int64_t n, int64_t b, uint64_t seed, uint64_t iteration,
                       int32_t* out) {
    std::vector<uint64_t> running((size_t)n);
    uint64_t W = 0;
    for (int64_t e = 0; e < n; ++e) {
        W += score[e];
        running[(size_t)e] = W;
    }
    for (int64_t j = 0; j < b; ++j) {
        out[j] = -1;
        if (W == 0) continue;
        const uint64_t x = mulhi64(draw64(seed, 0x4253454Cu, iteration, (uint32_t)j), W);
        for (int64_t e = 0; e < n; ++e) {
            if (running[(size_t)e] > x) {
                out[j] = (int32_t)e;
                break;
            }
        }
    }
}

/* Score update after an iteration: for j = 0..b-1 in order, score[idx[j]] =
 * value[j] (an edge drawn twice keeps the later value); entries with idx
 * outside [0, n) are skipped. */
void oracle_score_update(uint32_t* score, int64_t n, const int32_t* idx, const uint32_t* value, int64_t b) {
    for (int64_t j = 0; j < b; ++j) {
        if (idx[j] < 0 || idx[j] >= n) continue;
        score[idx[j]] = value[j];
    }
}

}  // extern "C"
