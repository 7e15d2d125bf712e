"""Seeded synthetic inputs shaped like the paper's workloads (Table II shapes).

This module only *draws inputs* (event lists, query roots, feature tables,
weights). It holds none of the method's arithmetic and is the one module both
the HIP path's harness and the CPU checker's tests may use. The paper's
datasets are not available, so every workload is a stand-in with the node and
edge counts, degree skew, timestamp ties, feature widths and batch recipe of
the corresponding dataset; no dataset record is reproduced.

Event list -> T-CSR entries: N(v,t) is defined over edges leaving v (paper
Sec. 2.1) while sources, destinations and negative destinations are all query
roots (Sec. 2), so every event i is emitted twice, (u->v) at entry 2i and
(v->u) at entry 2i+1, same timestamp, same edge id; the entry stream stays
time-sorted.
"""
from dataclasses import dataclass, field
from concurrent.futures import ThreadPoolExecutor

import numpy as np

RECENT, UNIFORM, WEIGHTED = 0, 1, 2


@dataclass
class Workload:
    name: str
    num_nodes: int
    num_edges: int
    src: np.ndarray            # int32 [2E]  entry source
    dst: np.ndarray            # int32 [2E]  entry neighbor
    ts: np.ndarray             # int64 [2E]  non-decreasing
    eid: np.ndarray            # int32 [2E]
    edge_dim: int
    edge_dtype: str            # "float32" | "float16"
    edge_feat: object          # np.ndarray [E, d] or None when procedural
    edge_seed: int             # seed of the procedural table (edge_feat is None)
    node_feat: object          # np.ndarray [N, d_v] float32 or None
    edge_weight: object        # np.ndarray uint32 [E] or None
    batches: list              # [(roots int32[R], times int64[R]), ...]
    k: int
    hops: int
    policies: tuple            # sampling policies this workload is run with
    m: int = 0                 # candidate window (weighted only)
    cache_ratio: float = 0.0   # device cache size / node rows
    notes: dict = field(default_factory=dict)


# ----------------------------------------------------------------------------
# elementary draws
# ----------------------------------------------------------------------------
def _categorical(rng_seed, weights, size, threads=8, chunk=1 << 23):
    """`size` draws from the categorical distribution `weights` by inverse CDF.
    Chunked with one child seed per chunk so the result does not depend on the
    number of worker threads."""
    cdf = np.cumsum(np.asarray(weights, np.float64))
    cdf /= cdf[-1]
    n_chunks = max(1, (size + chunk - 1) // chunk)
    seeds = np.random.SeedSequence(rng_seed).spawn(n_chunks)
    out = np.empty(size, np.int32)

    def work(c):
        lo, hi = c * chunk, min(size, (c + 1) * chunk)
        u = np.random.Generator(np.random.PCG64(seeds[c])).random(hi - lo)
        out[lo:hi] = np.minimum(np.searchsorted(cdf, u, side="right"), len(cdf) - 1)

    if n_chunks == 1:
        work(0)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(work, range(n_chunks)))
    return out


def _zipf_weights(n, s):
    return 1.0 / np.arange(1, n + 1, dtype=np.float64) ** s


def _sorted_uniform_ints(rng, n, span):
    """n sorted draws, uniform on [0, span): normalised partial sums of
    exponential spacings have exactly the law of sorted uniforms."""
    gaps = rng.standard_exponential(n + 1)
    c = np.cumsum(gaps)
    t = np.floor(c[:n] * (float(span) / c[n])).astype(np.int64)
    return np.minimum(t, span - 1)


def _entries(u, v, ts):
    e = u.shape[0]
    src = np.empty(2 * e, np.int32)
    dst = np.empty(2 * e, np.int32)
    src[0::2], src[1::2] = u, v
    dst[0::2], dst[1::2] = v, u
    return src, dst, np.repeat(ts, 2), np.repeat(np.arange(e, dtype=np.int32), 2)


def _link_batch(u, v, ts, edge_idx, neg):
    """Roots of one link-prediction batch: sources, destinations and negative
    destinations, each queried at its edge's timestamp."""
    roots = np.concatenate([u[edge_idx], v[edge_idx], neg]).astype(np.int32)
    times = np.tile(ts[edge_idx], 3).astype(np.int64)
    return roots, times


def _bipartite(rng, seed, n_src, n_dst, n_edges, s_src, s_dst):
    perm_s = rng.permutation(n_src).astype(np.int32)
    perm_d = (n_src + rng.permutation(n_dst)).astype(np.int32)
    if s_src is None:
        u = rng.integers(0, n_src, n_edges, dtype=np.int32)
    else:
        u = _categorical(seed * 16 + 1, _zipf_weights(n_src, s_src), n_edges)
    v = _categorical(seed * 16 + 2, _zipf_weights(n_dst, s_dst), n_edges)
    return perm_s[u], perm_d[v]


# ----------------------------------------------------------------------------
# procedural feature table: a pure integer function of (seed, row, col)
# ----------------------------------------------------------------------------
_PA, _PB, _PC, _PD, _PE = (0x9E3779B97F4A7C15, 0xD1B54A32D192ED03, 0xA24BAED4963EE407,
                           0x8CB92BA72F3D8DD7, 0xF1357AEA2E62A9C5)


def _s64(x):
    """Python int -> the int64 with the same low 64 bits."""
    x &= (1 << 64) - 1
    return x - (1 << 64) if x >= (1 << 63) else x


def procedural_rows(seed, rows, dim, dtype):
    """Rows `rows` (int array) of the procedural table, shape [len(rows), dim].
    Element = (sum of 12 hash bytes - 1530) / 256: an Irwin-Hall stand-in for
    N(0,1) whose values are multiples of 1/256 below 6 in magnitude, hence
    exactly representable in fp16 and fp32."""
    r = np.asarray(rows, np.uint64)[:, None]
    c = np.arange(dim, dtype=np.uint64)[None, :]
    with np.errstate(over="ignore"):
        x = r * np.uint64(_PA) + c * np.uint64(_PB) + np.uint64(seed & ((1 << 64) - 1))
        x ^= x >> np.uint64(32)
        x *= np.uint64(_PC)
        x ^= x >> np.uint64(29)
        x *= np.uint64(_PD)
        x ^= x >> np.uint64(32)
        y = x * np.uint64(_PE)
        y ^= y >> np.uint64(31)
    s = np.zeros(x.shape, np.int64)
    for b in range(8):
        s += ((x >> np.uint64(8 * b)) & np.uint64(255)).astype(np.int64)
    for b in range(4):
        s += ((y >> np.uint64(8 * b + 16)) & np.uint64(255)).astype(np.int64)
    return ((s - 1530).astype(np.float32) / np.float32(256.0)).astype(dtype)


def procedural_table_torch(seed, rows, dim, dtype, pitch_elems, device, chunk_rows=1 << 19):
    """The same table as `procedural_rows`, filled on `device` with torch integer
    ops (int64 wrap-around arithmetic, logical shifts emulated by masking), in
    a [rows, pitch_elems] tensor whose columns >= dim are zero."""
    import torch
    table = torch.zeros((rows, pitch_elems), dtype=dtype, device=device)
    c = torch.arange(dim, dtype=torch.int64, device=device)[None, :] * _s64(_PB) + _s64(seed)

    def lsr(t, s):
        return (t >> s) & ((1 << (64 - s)) - 1)

    for r0 in range(0, rows, chunk_rows):
        r1 = min(rows, r0 + chunk_rows)
        x = torch.arange(r0, r1, dtype=torch.int64, device=device)[:, None] * _s64(_PA) + c
        x ^= lsr(x, 32)
        x *= _s64(_PC)
        x ^= lsr(x, 29)
        x *= _s64(_PD)
        x ^= lsr(x, 32)
        y = x * _s64(_PE)
        y ^= lsr(y, 31)
        s = x & 255
        for b in range(1, 8):
            s += (x >> (8 * b)) & 255
        for b in range(4):
            s += (y >> (8 * b + 16)) & 255
        table[r0:r1, :dim] = ((s - 1530).to(torch.float32) / 256.0).to(dtype)
        del x, y, s
    return table


# ----------------------------------------------------------------------------
# the five workloads
# ----------------------------------------------------------------------------
def _seed(cfg):
    return 0x7A5E0000 + cfg


def make_c1():
    """Tiny bipartite graph, the quick reference case."""
    seed = _seed(1)
    rng = np.random.Generator(np.random.PCG64(seed))
    n_src, n_dst, e = 800, 200, 20000
    u, v = _bipartite(rng, seed, n_src, n_dst, e, None, 1.0)
    ts = _sorted_uniform_ints(rng, e, 10 ** 6)
    feat = rng.standard_normal((e, 16), dtype=np.float32)
    batches = []
    for b in range(10):
        idx = np.arange(2000 * b, 2000 * b + 200)
        neg = n_src + rng.integers(0, n_dst, idx.shape[0])
        batches.append(_link_batch(u, v, ts, idx, neg))
    src, dst, ts2, eid = _entries(u, v, ts)
    return Workload("C1-tiny", n_src + n_dst, e, src, dst, ts2, eid, 16, "float32", feat, 0, None,
                    None, batches, k=10, hops=1, policies=(RECENT, UNIFORM))


def make_c2(edges=160000):
    """Wikipedia-shaped (Table II): bipartite, d_e = 172, chronological pass."""
    seed = _seed(2)
    rng = np.random.Generator(np.random.PCG64(seed))
    n_src, n_dst, e = 8000, 1000, edges
    u, v = _bipartite(rng, seed, n_src, n_dst, e, 1.1, 1.3)
    ts = np.cumsum(np.floor(rng.exponential(16.0, e))).astype(np.int64)
    feat = rng.standard_normal((e, 172), dtype=np.float32)
    batches = []
    for b0 in range(0, e, 600):
        idx = np.arange(b0, min(e, b0 + 600))
        neg = n_src + rng.integers(0, n_dst, idx.shape[0])
        batches.append(_link_batch(u, v, ts, idx, neg))
    src, dst, ts2, eid = _entries(u, v, ts)
    return Workload("C2-wikipedia-shaped", n_src + n_dst, e, src, dst, ts2, eid, 172, "float32",
                    feat, 0, None, None, batches, k=10, hops=1, policies=(RECENT, UNIFORM))


def make_c3(edges=670000, num_batches=20):
    """Reddit-shaped (Table II): bipartite, fp16 d_e = 172, 2-hop uniform 10x10,
    batches drawn at random from the last 30 % of the stream (TASER's batch
    order is not chronological)."""
    seed = _seed(3)
    rng = np.random.Generator(np.random.PCG64(seed))
    n_src, n_dst, e = 10000, 1000, edges
    u, v = _bipartite(rng, seed, n_src, n_dst, e, 1.2, 1.2)
    ts = _sorted_uniform_ints(rng, e, 2700000)
    feat = rng.standard_normal((e, 172), dtype=np.float32).astype(np.float16)
    batches = []
    for _ in range(num_batches):
        idx = rng.integers(int(0.7 * e), e, min(2000, e))
        neg = n_src + rng.integers(0, n_dst, idx.shape[0])
        batches.append(_link_batch(u, v, ts, idx, neg))
    src, dst, ts2, eid = _entries(u, v, ts)
    return Workload("C3-reddit-shaped", n_src + n_dst, e, src, dst, ts2, eid, 172, "float16", feat,
                    0, None, None, batches, k=10, hops=2, policies=(UNIFORM,))


def make_c4(edges=1900000, num_batches=20):
    """Flights-shaped node/edge counts: dense non-bipartite graph, endpoints from
    a degree-corrected power law (degree exponent 2.1), per-edge integer weights
    for the weighted (adaptive) selection with m = 25 candidates, k = 10."""
    seed = _seed(4)
    rng = np.random.Generator(np.random.PCG64(seed))
    n, e = 13000, edges
    theta = (1.0 - rng.random(n)) ** (-1.0 / 1.1)
    for _ in range(64):                       # cap: no node above 5 % of endpoints
        cap = 0.05 * theta.sum()
        if theta.max() <= cap:
            break
        theta = np.minimum(theta, cap)
    u = _categorical(seed * 16 + 1, theta, e)
    v = _categorical(seed * 16 + 2, theta, e)
    ts = _sorted_uniform_ints(rng, e, 10 ** 7)
    feat = rng.standard_normal((e, 16), dtype=np.float32)
    z = rng.standard_normal(e)
    weight = np.clip(np.rint(np.exp(z) * 4096.0), 1, 65536).astype(np.uint32)
    batches = []
    for _ in range(num_batches):
        idx = rng.integers(int(0.7 * e), e, min(4000, e))
        roots = np.where(np.arange(idx.shape[0]) % 2 == 0, u[idx], v[idx]).astype(np.int32)
        batches.append((roots, ts[idx].astype(np.int64)))
    src, dst, ts2, eid = _entries(u, v, ts)
    return Workload("C4-flights-shaped", n, e, src, dst, ts2, eid, 16, "float32", feat, 0, None,
                    weight, batches, k=10, hops=2, policies=(WEIGHTED,), m=25)


def make_c5(edges=191000000, num_batches=20, last=1000000, threads=16):
    """GDELT-shaped (Table II): 17 000 nodes, 191 M events, Zipf(1.0) endpoints,
    heavy timestamp ties, fp16 d_e = 186 edge table (procedural: it only ever
    exists in device memory), fp32 d_v = 413 node table for pinned host memory
    with a 20 % device cache, batches from the latest 1 M events."""
    seed = _seed(5)
    rng = np.random.Generator(np.random.PCG64(seed))
    n, e = 17000, edges
    perm = rng.permutation(n).astype(np.int32)
    w = _zipf_weights(n, 1.0)
    u = perm[_categorical(seed * 16 + 1, w, e, threads)]
    v = perm[_categorical(seed * 16 + 2, w, e, threads)]
    ts = _sorted_uniform_ints(rng, e, int(1e8 * min(1.0, e / 191e6)) or 1)
    node_feat = rng.standard_normal((n, 413), dtype=np.float32)
    batches = []
    lo = max(0, e - last)
    for _ in range(num_batches):
        idx = rng.integers(lo, e, min(4000, e))
        neg = rng.integers(0, n, idx.shape[0])
        batches.append(_link_batch(u, v, ts, idx, neg))
    src, dst, ts2, eid = _entries(u, v, ts)
    del u, v
    return Workload("C5-gdelt-shaped", n, e, src, dst, ts2, eid, 186, "float16", None, seed,
                    node_feat, None, batches, k=10, hops=2, policies=(RECENT,), cache_ratio=0.2,
                    notes={"hot_order": perm})


MAKERS = {1: make_c1, 2: make_c2, 3: make_c3, 4: make_c4, 5: make_c5}


def make(cfg, **kw):
    return MAKERS[cfg](**kw)
