/*
 * taser.h — C ABI of the MI355X (gfx950) temporal neighbor finder and feature
 * gather: the mini-batch generation hot path of TASER (arXiv 2402.05396,
 * Sec. 2.1 "Neighbor Finder", Sec. 3.3 "GPU Temporal Neighbor Finding",
 * Sec. 3.4 "GPU Feature Caching", Alg. 1-3).
 *
 * Conventions shared by every call
 *   - Plain pointers and sizes only. Each pointer argument says "device" or
 *     "host". Device pointers must be valid on the current HIP device.
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the null stream).
 *     Unless a call says otherwise it only enqueues work on that stream and
 *     returns without waiting for it.
 *   - Ownership: the caller owns every input and output buffer. The library
 *     owns the opaque handles (and scratch memory inside them), released only
 *     by the matching *_free call. A handle must not be used by two calls that
 *     overlap in time on different streams.
 *   - Return value: TASER_OK (0) or a negative taser_status. Arguments are
 *     validated on the host before anything is launched; on error nothing has
 *     been enqueued and taser_last_error() describes the problem.
 *   - Graph capture: taser_sample_temporal(_rows), taser_gather_features,
 *     taser_candidate_encodings, taser_select_weighted, taser_selector_draw,
 *     taser_selector_update and taser_cache_lookup / _lookup_static /
 *     _prefetch / _gather only launch kernels (no memset or copy nodes, no
 *     synchronization), so a stream
 *     that is being captured into a HIP graph can be passed to them. Three
 *     things happen on first use only and must have happened before a capture:
 *     a cache lookup or prefetch with more requests than any before it on that
 *     handle allocates (and waits for the whole device, see
 *     taser_cache_prefetch); the first TASER_INVERSE_TIMESPAN call on a graph
 *     allocates; the first gather of a process on a device looks up the address
 *     of a constant (taser_cache_init and taser_tcsr_build do that too, so any
 *     handle made on the device is enough). The per-kernel timing session of
 *     taser_profile.h must be off during a capture.
 *   - Padding: an unused output slot holds nbr = -1, eid = -1, ts = 0; a
 *     negative id given to a gather produces a row of zero bytes.
 */
#ifndef TASER_H
#define TASER_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct taser_tcsr taser_tcsr;   /* time-sorted CSR in device memory  */
typedef struct taser_cache taser_cache; /* device cache over a host table    */
typedef struct taser_selector taser_selector; /* importance scores of the training edges */

enum taser_status {
    TASER_OK = 0,
    TASER_E_ARG = -1,         /* null pointer, non-positive size, bad enum          */
    TASER_E_RANGE = -2,       /* a size or id outside the supported/declared range  */
    TASER_E_OOM = -3,         /* device or host allocation failed                   */
    TASER_E_HIP = -4,         /* a HIP runtime call failed                          */
    TASER_E_UNSUPPORTED = -5  /* valid request this build does not implement        */
};

enum taser_policy {
    TASER_RECENT = 0,   /* most recent neighbor finder   (Sec. 2.1, Alg. 2)              */
    TASER_UNIFORM = 1,  /* uniform, without replacement  (Sec. 2.1, Alg. 2)              */
    TASER_WEIGHTED = 2, /* n of the m most recent, by given weights (Alg. 1, 2nd draw)   */
    TASER_INVERSE_TIMESPAN = 3 /* probability inversely proportional to the time delta:
                                  the heuristic finder of TGAT (Sec. 1, Sec. 2.3)        */
};

enum taser_build_flags {
    TASER_INPUT_ON_DEVICE = 1u /* src/dst/ts/eid are device pointers (default: host) */
};

#define TASER_MAX_K 64    /* neighbors kept per root and hop              */
#define TASER_MAX_M 64    /* candidate window of the weighted policy      */
#define TASER_MAX_HOPS 3
#define TASER_STATIC_LOOKUP_MAX_REQUESTS (1 << 21) /* requests per taser_cache_lookup_static call */

/* ---------------------------------------------------------------------------
 * T-CSR (Sec. 3.3: the dynamic graph is stored with every node's outgoing
 * neighbors sorted by timestamp; Sec. 2.1: N(v,t) is defined over the edges
 * leaving v).
 *
 * Groups the `num_entries` entries (src[i] -> dst[i] at ts[i], edge id eid[i])
 * by src and orders each group by (ts, input position): a stable sort, so the
 * result is unique. The library is direction-agnostic; a caller that queries
 * both endpoints of an interaction passes it in both directions.
 *
 *   src, dst   int32[num_entries], node ids in [0, num_nodes)   host (or device
 *   ts         int64[num_entries]                                with the flag)
 *   eid        int32[num_entries], or NULL meaning eid[i] = i
 *   num_entries in [0, 2^31 - 1), num_nodes in [1, 2^31 - 1)
 *   out        receives a new handle
 *
 * Inputs are only read. This call synchronizes `hip_stream` before returning
 * (it reads back the sort plan and the id-range check), so host inputs may be
 * released immediately. Errors: TASER_E_RANGE if any src id is outside
 * [0, num_nodes) (dst ids are carried, not interpreted, and are not checked).
 * ------------------------------------------------------------------------- */
int taser_tcsr_build(const int32_t* src, const int32_t* dst, const int64_t* ts,
                     const int32_t* eid, int64_t num_entries, int32_t num_nodes,
                     uint32_t flags, void* hip_stream, taser_tcsr** out);

/* Size of a built graph (either out-pointer may be NULL). */
int taser_tcsr_size(const taser_tcsr* g, int64_t* num_entries, int32_t* num_nodes);

/* Canonical view for inspection and tests: writes the T-CSR as plain arrays
 * into caller-allocated device buffers indptr int64[num_nodes+1], nbr
 * int32[E'], ts int64[E'], eid int32[E'] (the sampler itself reads a packed
 * layout of the library's own). Any of the four may be NULL to skip it. */
int taser_tcsr_view(const taser_tcsr* g, int64_t* indptr, int32_t* nbr, int64_t* ts, int32_t* eid,
                    void* hip_stream);

void taser_tcsr_free(taser_tcsr* g);

/* ---------------------------------------------------------------------------
 * Temporal neighbor finding over one or more hops (Sec. 2.1; Alg. 2; the layer
 * loop of Alg. 1).
 *
 * Hop 0 has num_roots roots (roots[i], times[i]). For a root (v, t) let cnt be
 * the number of entries of v's list with ts < t (strictly). Output row i of a
 * hop has k slots:
 *   TASER_RECENT    slot j = entry cnt-1-j, for j < min(k, cnt).
 *   TASER_UNIFORM   cnt <= k: as TASER_RECENT. Otherwise k distinct entries,
 *                   a uniformly random ordered k-subset of the cnt valid ones,
 *                   drawn by a partial Fisher-Yates shuffle with one Philox
 *                   4x32-10 draw per slot keyed by (seed, hop, root index,
 *                   slot): r = j + floor(draw * (cnt - j) / 2^64).
 *   TASER_WEIGHTED  candidates = the c = min(m, cnt) most recent entries,
 *                   candidate i = entry cnt-1-i with weight
 *                   edge_weight[eid] (must be >= 1). c <= k: all candidates in
 *                   that order. Otherwise k successive draws without
 *                   replacement, each proportional to the remaining weights:
 *                   x = floor(draw * W / 2^64), first remaining candidate
 *                   whose running weight sum exceeds x.
 *   TASER_INVERSE_TIMESPAN  over all cnt valid entries, entry p weighs
 *                   max(1, floor(2^32 / (t - ts[p]))). cnt <= k: as
 *                   TASER_RECENT. Otherwise k successive draws without
 *                   replacement as for TASER_WEIGHTED, the running sum taken
 *                   in list order (oldest entry first). Costs time linear in
 *                   cnt per root (the weights depend on the query time). The
 *                   first call with this policy on a graph allocates 8 bytes
 *                   per entry inside the handle (the timestamps alone) and
 *                   waits for `hip_stream` once.
 * count[i] = number of filled (leading) slots; the rest are padding.
 * Hop h+1 has one root per slot of hop h, root index i*k + j, node = the
 * sampled neighbor and query time = the sampled interaction's timestamp; a
 * padding slot is a root with no neighbors. A root with a negative node id is
 * treated the same way. Results depend only on (graph, root, time, root
 * index, seed): they are reproducible and independent of launch shape.
 *
 *   roots int32[num_roots], times int64[num_roots]              device
 *   k in [1, TASER_MAX_K], hops in [1, TASER_MAX_HOPS], num_roots * k^hops < 2^31
 *   m in [1, TASER_MAX_M] and edge_weight uint32[max eid + 1] (device):
 *     TASER_WEIGHTED only, ignored otherwise (edge_weight may then be NULL)
 *   out   host array of `hops` structs of caller-allocated device buffers;
 *         hop h holds R_h = num_roots * k^h roots:
 *         nbr int32[R_h*k], eid int32[R_h*k], ts int64[R_h*k], count int32[R_h]
 * A root whose node id is >= num_nodes is treated like a negative one.
 * Edge ids of the graph must index edge_weight (not checked).
 * ------------------------------------------------------------------------- */
typedef struct taser_hop_out {
    int32_t* nbr;
    int32_t* eid;
    int64_t* ts;
    int32_t* count;
} taser_hop_out;

int taser_sample_temporal(const taser_tcsr* g, const int32_t* roots, const int64_t* times,
                          int64_t num_roots, int32_t k, int32_t hops, int32_t policy,
                          uint64_t seed, int32_t m, const uint32_t* edge_weight,
                          const taser_hop_out* out, void* hip_stream);

/* ---------------------------------------------------------------------------
 * Neighbor finding with the sampled edges' feature rows (Alg. 1: every layer's
 * neighbors are found, then their features sliced, Sec. 3.4 / Alg. 3 line 8;
 * here one launch per hop does both). The result is exactly that of
 *   taser_sample_temporal(g, roots, ..., out, stream) followed, for every hop h, by
 *   taser_gather_features(table, table_rows, row_bytes, pitch_bytes,
 *                         out[h].eid, R_h * k, rows_out[h], stream):
 * row q of rows_out[h] holds the table row of slot q's edge id, zeros for a
 * padding slot or an id outside [0, table_rows). While the rows of one
 * wavefront's roots are at most 8 KiB ((64 / G) * k * row_bytes, G = 16, 32 or
 * 64 being the first of them that holds k, and m for TASER_WEIGHTED), the
 * wavefront that has found the neighbors copies their rows itself: no launch of
 * its own for the rows, and the edge ids are not read back from memory. That
 * needs row_bytes a multiple of 4 and >= 16, table and pitch_bytes multiples of
 * 4, rows_out[h] 16-byte aligned and those bytes per wavefront a multiple of
 * 16. A hop for which any of it fails, every hop with longer rows (for which a
 * gather launch is the faster way) and every hop of TASER_INVERSE_TIMESPAN get
 * their rows from the gather kernel after the last hop, in one launch where the
 * hops' edge id arrays and row buffers follow one another in memory. The bytes
 * are the same either way.
 *   sampling arguments, `out`: as for taser_sample_temporal
 *   table, table_rows, row_bytes, pitch_bytes: as for taser_gather_features
 *   rows_out  host array of `hops` device pointers; rows_out[h] receives
 *             R_h * k * row_bytes bytes (2-byte aligned at least)
 * ------------------------------------------------------------------------- */
int taser_sample_temporal_rows(const taser_tcsr* g, const int32_t* roots, const int64_t* times,
                               int64_t num_roots, int32_t k, int32_t hops, int32_t policy,
                               uint64_t seed, int32_t m, const uint32_t* edge_weight,
                               const void* table, int64_t table_rows, int32_t row_bytes, int64_t pitch_bytes,
                               const taser_hop_out* out, void* const* rows_out, void* hip_stream);

/* ---------------------------------------------------------------------------
 * Candidate-window products of the adaptive sampler (Sec. 3 overview, Alg. 1:
 * a static finder returns m candidates per root, a network scores them, n of
 * the m are kept; Sec. 3.2: the network's frequency encoding takes the integer
 * freq(u_j), the identity encoding is the matrix IE[j][l] = 1 if u_j = u_l).
 * The candidates are the output of a taser_sample_temporal hop with k = m
 * (their feature rows: taser_gather_features on its eid array).
 *
 * taser_candidate_encodings, for root i with c = clamp(count[i], 0, m)
 * candidates nbr[i][0..c):
 *   freq[i][j]        = number of l < c with nbr[i][l] == nbr[i][j], for j < c
 *   identity[i][j][l] = 1 if j < c, l < c and nbr[i][j] == nbr[i][l], else 0
 * and 0 wherever a padding slot (index >= c) is involved.
 *   nbr int32[num_roots*m], count int32[num_roots]                   device
 *   freq int32[num_roots*m], identity uint8[num_roots*m*m] or NULL   device
 *   m in [1, TASER_MAX_M], num_roots * m < 2^31
 *
 * taser_select_weighted is the second draw of Alg. 1 with one weight per
 * (root, candidate): weight[i][j] >= 1 is the quantised q(j|i) of candidate j.
 * With c as above: c <= k keeps all candidates, sel[i][j] = j for j < c.
 * Otherwise k successive draws without replacement, each proportional to the
 * remaining weights, exactly as TASER_WEIGHTED: x = floor(draw * W / 2^64)
 * with the Philox draw keyed (seed, hop, i, j); sel[i][j] = first remaining
 * candidate whose running weight sum exceeds x. Unused slots of sel are -1;
 * out_count[i] = min(c, k).
 *   weight uint32[num_roots*m], count int32[num_roots]               device
 *   sel int32[num_roots*k], out_count int32[num_roots]               device
 *   candidates, kept: both NULL, or host pointers to structs of device
 *     buffers (count members unused): kept->nbr/eid/ts [num_roots*k] receive
 *     candidates->nbr/eid/ts [num_roots*m] at the selected slots (padding where
 *     sel is -1), ready to be the next hop's roots and times.
 *   k in [1, TASER_MAX_K], m in [1, TASER_MAX_M], num_roots * max(m,k) < 2^31
 * With weight[i][j] = edge_weight[eid of candidate j] the result equals policy
 * TASER_WEIGHTED of taser_sample_temporal for the same seed, hop and roots.
 * ------------------------------------------------------------------------- */
int taser_candidate_encodings(const int32_t* nbr, const int32_t* count, int64_t num_roots, int32_t m,
                              int32_t* freq, uint8_t* identity, void* hip_stream);

int taser_select_weighted(const uint32_t* weight, const int32_t* count, int64_t num_roots, int32_t m,
                          int32_t k, uint64_t seed, uint32_t hop, int32_t* sel, int32_t* out_count,
                          const taser_hop_out* candidates, const taser_hop_out* kept, void* hip_stream);

/* ---------------------------------------------------------------------------
 * Feature slicing from a table in device memory (Sec. 3.4; Alg. 3 "serve
 * x_e"): out row i = the row_bytes bytes of table row ids[i]; ids[i] < 0 gives
 * a zero row. The output is dense (row i at byte offset i * row_bytes).
 *
 *   table        device, `rows` rows, row r at byte offset r * pitch_bytes
 *   row_bytes    > 0, even; pitch_bytes >= row_bytes, even
 *   ids          int32[n], device; an id >= rows is served like a negative one
 *   out          device, n * row_bytes bytes, must not overlap the table
 * Rows whose size, pitch and base addresses share a 16-, 8- or 4-byte
 * alignment are moved with loads and stores of that width.
 * ------------------------------------------------------------------------- */
int taser_gather_features(const void* table, int64_t rows, int32_t row_bytes,
                          int64_t pitch_bytes, const int32_t* ids, int64_t n, void* out,
                          void* hip_stream);

/* ---------------------------------------------------------------------------
 * Device cache of hot feature rows over a table in pinned host memory
 * (Sec. 3.4, Alg. 3: k rows live in device memory, the rest are read from host
 * memory over the bus; the cache line is one row).
 *
 * taser_cache_init copies `capacity_rows` rows into device memory and builds a
 * hashed id -> slot index there.
 *   host_table      host, allocated page-locked and device-mapped
 *                   (hipHostMalloc / a pinned torch tensor); it must outlive
 *                   the handle. TASER_E_ARG if it is not such memory.
 *   rows, row_bytes, pitch_bytes   as for taser_gather_features; row_bytes % 4 == 0
 *   capacity_rows   in [0, rows], below 2^30
 *   resident_ids    host int32[capacity_rows], distinct, in [0, rows); or NULL:
 *                   the first capacity_rows elements of a partial Fisher-Yates
 *                   shuffle of 0..rows-1 with draw j keyed (seed, hop tag
 *                   0x43414348, root index j, slot 0) ("randomly cache k
 *                   features", Alg. 3)
 *   staging_rows    rows of per-call device staging (>= 0): the distinct rows
 *                   that miss are fetched from host memory once per call into
 *                   it (in consecutive rows, as many as fit), however often the
 *                   call requests them; requests for further rows read host
 *                   memory directly.
 * This call synchronizes `hip_stream` before returning.
 *
 * taser_cache_lookup serves n rows into the dense `out` exactly like
 * taser_gather_features over the host table; which rows are resident never
 * changes the bytes served. hit_miss (device uint64[2], may be NULL) is
 * incremented by the number of requests with a resident id ([0]) and with a
 * valid non-resident id ([1]).
 * ------------------------------------------------------------------------- */
int taser_cache_init(const void* host_table, int64_t rows, int32_t row_bytes,
                     int64_t pitch_bytes, int64_t capacity_rows, const int32_t* resident_ids,
                     uint64_t seed, int64_t staging_rows, void* hip_stream, taser_cache** out);

int taser_cache_lookup(taser_cache* c, const int32_t* ids, int64_t n, void* out,
                       uint64_t* hit_miss, void* hip_stream);

/* The two halves of taser_cache_lookup, for callers that overlap the bus-bound
 * half with other work (e.g. on a second stream, beside the edge-feature
 * gather). taser_cache_prefetch classifies the n requests (updating hit_miss as
 * above) and copies every distinct missing row from host memory into the
 * staging area; taser_cache_gather then writes the dense output. The gather
 * must be given the same ids pointer and n as the latest prefetch on this
 * handle (TASER_E_ARG otherwise), must be ordered after it (same stream, or an
 * event), and ids must be unchanged in between. A new prefetch must not start
 * before the previous gather has finished: both use the handle's scratch.
 * The handle keeps one 32-bit location per request; a call with a larger n than
 * any before it on this handle first waits for the whole device
 * (hipDeviceSynchronize: an earlier gather may still read the old array on any
 * stream), frees that array and allocates a larger one. A caller that must not
 * block or allocate in its loop makes one call with its largest n beforehand. */
int taser_cache_prefetch(taser_cache* c, const int32_t* ids, int64_t n, uint64_t* hit_miss,
                         void* hip_stream);
int taser_cache_gather(taser_cache* c, const int32_t* ids, int64_t n, void* out, void* hip_stream);

/* taser_cache_lookup for callers that cannot allocate device memory: code whose
 * stream is being captured into a HIP graph, tight serving loops, harnesses
 * that forbid hipMalloc. Same arguments, same output and same counters as
 * taser_cache_lookup, but the per-request scratch (one 32-bit location per
 * request, per-block hit/miss counts) lives in a fixed array inside the
 * library's code object (8 MiB + 16 KiB on every GPU the library runs on, held
 * until the process ends) instead of the handle's growable buffer, so the call
 * never allocates, frees or synchronizes: it only launches kernels.
 *   n at most TASER_STATIC_LOOKUP_MAX_REQUESTS, else TASER_E_RANGE (nothing is
 *   launched).
 * All handles on one GPU share that array and it keeps the previous call's
 * contents (every word is written before it is read, nothing has to start at
 * zero): two such calls that overlap in time on one GPU, on any handles or
 * streams, race; order them on one stream or by events. The handle's staging
 * area is used as by taser_cache_lookup, so a taser_cache_prefetch still
 * waiting for its taser_cache_gather on this handle is cancelled. */
int taser_cache_lookup_static(taser_cache* c, const int32_t* ids, int64_t n, void* out,
                              uint64_t* hit_miss, void* hip_stream);

/* Knobs for callers that run the halves of a lookup beside other kernels, and for measurements.
 *   stage_blocks  number of 256-thread blocks the host -> staging copy runs on
 *                 (default 64; 0 keeps the current value). The copy is bound by
 *                 the bus; fewer blocks copy somewhat slower but leave more of
 *                 the memory system's request slots to kernels running beside it.
 *   refresh_before_gather  non-zero: taser_cache_gather first re-writes its read
 *                 working set (request locations, resident rows, staged rows) in
 *                 place. Worth it only when other bandwidth-heavy kernels run
 *                 between prefetch and gather (they push that working set out of
 *                 the memory-side cache, which does not take it back on reads).
 *                 Default off. Never changes results.
 *   partitioned_gather  negative keeps the current setting. 1 (the default): a
 *                 lookup of at least 4096 rows of 512 bytes to 16 KiB hands out
 *                 its output in 128-byte lines, each to a workgroup on the L2
 *                 partition of the chip that serves the line's source row, so
 *                 that a row is read from memory through one partition rather
 *                 than through all eight (a table of a few tens of MB is then
 *                 fetched about once per lookup). Rows that taser_cache_epoch_end
 *                 found to draw at least 1/4096 of all requests are spread by
 *                 request position instead (they sit in every L2 anyway, and the
 *                 partitions' loads stay equal). 0: always the plain gather in
 *                 output order. 2: the partitioned kernel with every row spread
 *                 by position (for measurements). Never changes results. */
int taser_cache_tune(taser_cache* c, int32_t stage_blocks, int32_t refresh_before_gather,
                     int32_t partitioned_gather);

/* ---------------------------------------------------------------------------
 * Cache maintenance (Alg. 3; Sec. 3.4): count how often every row is requested
 * and, at the end of an epoch, swap the cache content for the most requested
 * rows if too few of them are resident.
 *
 * taser_cache_count_accesses(enable != 0): from now on every lookup/prefetch
 * adds 1 to the counter of each requested row with a valid id (hit or miss).
 * The counters (uint32 per row, device memory, zeroed when first enabled) and
 * the scratch of taser_cache_epoch_end (two more uint32 per row, one int32 per
 * cache slot) are allocated when counting is first enabled, so an epoch end
 * allocates no device memory; enable == 0 pauses counting and keeps them.
 *
 * taser_cache_access_counts copies the counters into `counts`
 * (device uint32[rows], caller-allocated), ordered on `hip_stream`.
 *
 * taser_cache_epoch_end: Q_topk = the capacity_rows rows with the largest
 * counters (ties: the smaller id). *overlap (host, may be NULL) receives how
 * many of them are resident. If that is below min_overlap the cache content is
 * replaced by Q_topk (slots in ascending id order: rows re-read from the host
 * table, index rebuilt) and *replaced (host, may be NULL) is set to 1, else 0.
 * Either way the resident rows that drew at least 1/4096 of the epoch's requests
 * are noted (see partitioned_gather above; nothing else uses the note) and the
 * counters are zeroed. Synchronizes `hip_stream`; no lookup on
 * this handle may be in flight. TASER_E_ARG if counting was never enabled.
 * ------------------------------------------------------------------------- */
int taser_cache_count_accesses(taser_cache* c, int32_t enable, void* hip_stream);
int taser_cache_access_counts(const taser_cache* c, uint32_t* counts, void* hip_stream);
int taser_cache_epoch_end(taser_cache* c, int64_t min_overlap, int64_t* overlap, int32_t* replaced,
                          void* hip_stream);

/* Copies the resident row ids (slot order) to host int32[capacity_rows]. */
int taser_cache_residents(const taser_cache* c, int32_t* resident_ids_host);

void taser_cache_free(taser_cache* c);

/* ---------------------------------------------------------------------------
 * Adaptive mini-batch selection (Sec. 3.1: a list of importance scores P over
 * the training edges, initialised uniformly; every iteration samples a batch of
 * training edges with probability proportional to the scores and afterwards
 * overwrites the scores of the batch's edges, Eq. (4)).
 *
 * Scores are uint32; turning sigmoid(y) + gamma into an integer is the
 * caller's business (it needs the model's output). The handle keeps the scores
 * and two levels of partial sums in device memory; a draw or an update costs
 * time proportional to the batch, not to the number of training edges.
 *
 * taser_selector_init: n training edges in [1, 2^31); scores device uint32[n],
 *   or NULL: every score = initial_score. Synchronizes `hip_stream`.
 * taser_selector_draw: batch[j], j < b, = the first edge whose running score
 *   sum (edge 0 first) exceeds floor(draw * W / 2^64), W = the sum of all
 *   scores, draw = the Philox 4x32-10 draw keyed (seed, hop tag 0x4253454C,
 *   root index `iteration`, slot j): b independent draws, so an edge can appear
 *   twice; an edge with score 0 is never drawn; W == 0 gives -1.
 *   batch device int32[b], b in [0, 2^31).
 * taser_selector_update: score[batch[j]] = new_scores[j] for j = 0..b-1 in that
 *   order (an edge named twice keeps the later value); entries outside [0, n)
 *   are skipped. batch device int32[b], new_scores device uint32[b]. Must be
 *   ordered after the draws that should see the old scores.
 * taser_selector_scores: copies the scores to `scores` (device uint32[n], may
 *   be NULL); if `total` (host, may be NULL) is given it receives the sum of
 *   all scores as the partial sums hold it, and the call synchronizes.
 * ------------------------------------------------------------------------- */
int taser_selector_init(const uint32_t* scores, int64_t n, uint32_t initial_score, void* hip_stream,
                        taser_selector** out);
int taser_selector_draw(const taser_selector* s, int64_t b, uint64_t seed, uint64_t iteration,
                        int32_t* batch, void* hip_stream);
int taser_selector_update(taser_selector* s, const int32_t* batch, const uint32_t* new_scores, int64_t b,
                          void* hip_stream);
int taser_selector_scores(const taser_selector* s, uint32_t* scores, uint64_t* total, void* hip_stream);
int taser_selector_size(const taser_selector* s, int64_t* n);
void taser_selector_free(taser_selector* s);

/* Message for the most recent error on the calling thread (static storage). */
const char* taser_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* TASER_H */
