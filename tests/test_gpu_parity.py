"""Parity of the HIP path (through the C ABI) with the CPU oracle, element by
element, on seeded synthetic inputs. Bit-exact: everything on this path is
integer/index/byte work."""
import numpy as np
import pytest
import torch

import oracle
import paper_2402_05396_amd as T
from paper_2402_05396_amd import workloads as W

pytestmark = pytest.mark.gpu

THREADS = min(16, oracle.max_threads())
FIELDS = ("nbr", "eid", "ts", "count")


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def build_both(src, dst, ts, eid, num_nodes, on_device=True):
    g_ref = oracle.tcsr_build(src, dst, ts, eid, num_nodes, THREADS)
    args = [torch.from_numpy(np.ascontiguousarray(x)) for x in (src, dst, ts, eid)]
    if on_device:
        args = [a.cuda() for a in args]
    g = T.tcsr_build(*args, num_nodes)
    return g, g_ref


def assert_tcsr_equal(g, g_ref):
    got = [x.cpu().numpy() for x in T.tcsr_view(g)]
    for name, a, b in zip(("indptr", "nbr", "ts", "eid"), got, g_ref):
        assert a.dtype == b.dtype and np.array_equal(a, b), name


def assert_hops_equal(got, want):
    assert len(got) == len(want)
    for h, (a, b) in enumerate(zip(got, want)):
        for f in FIELDS:
            x = a[f].cpu().numpy()
            assert x.shape == b[f].shape and np.array_equal(x, b[f]), f"hop {h} field {f}"


def run_both(g, g_ref, roots, times, k, hops, policy, seed, m=0, weight=None):
    want = oracle.sample_temporal(g_ref, roots, times, k, hops, policy, seed, m, weight, THREADS)
    w_dev = None if weight is None else dev(weight.view(np.int32))
    got = T.sample_temporal(g, dev(roots), dev(times), k, hops, policy, seed, m, w_dev)
    torch.cuda.synchronize()
    assert_hops_equal(got, want)
    return got, want


def check_gather(table_np, table_dev, ids_dev_2d, ids_np_2d):
    want = oracle.gather(table_np, ids_np_2d.ravel(), threads=THREADS)
    got = T.gather_features(table_dev, ids_dev_2d.reshape(-1), row_elems=table_np.shape[1])
    torch.cuda.synchronize()
    assert got.cpu().numpy().tobytes() == want.tobytes()


# ----------------------------------------------------------------------------- the five workloads
def test_c1_tiny_all_batches():
    w = W.make(1)
    g, g_ref = build_both(w.src, w.dst, w.ts, w.eid, w.num_nodes, on_device=False)
    assert_tcsr_equal(g, g_ref)
    table = dev(w.edge_feat)
    for b, (roots, times) in enumerate(w.batches):
        for policy in w.policies:
            got, want = run_both(g, g_ref, roots, times, w.k, 1, policy, seed=42 + b)
            check_gather(w.edge_feat, table, got[0]["eid"], want[0]["eid"])
    assert sum(int((r >= 0).sum()) for r, _ in w.batches) == 6000


def test_c2_one_hop_recent_and_uniform():
    w = W.make(2)
    g, g_ref = build_both(w.src, w.dst, w.ts, w.eid, w.num_nodes)
    assert_tcsr_equal(g, g_ref)
    table = dev(w.edge_feat)
    assert len(w.batches) == 267 and w.batches[-1][0].shape[0] == 1200
    for b, (roots, times) in enumerate(w.batches):     # the whole chronological pass, cold start to the ragged last batch
        for policy in w.policies:
            got, want = run_both(g, g_ref, roots, times, w.k, 1, policy, seed=42)
            if b in (0, 1, 2, 50, 133, 200, 265, 266):
                check_gather(w.edge_feat, table, got[0]["eid"], want[0]["eid"])


def test_c3_two_hop_uniform_fp16():
    w = W.make(3, num_batches=3)
    g, g_ref = build_both(w.src, w.dst, w.ts, w.eid, w.num_nodes)
    assert_tcsr_equal(g, g_ref)
    table = dev(w.edge_feat)
    for roots, times in w.batches:
        got, want = run_both(g, g_ref, roots, times, w.k, 2, W.UNIFORM, seed=42)
        assert got[1]["nbr"].shape == (60000, 10)
        for h in range(2):
            check_gather(w.edge_feat, table, got[h]["eid"], want[h]["eid"])


def test_c4_two_hop_weighted():
    w = W.make(4, num_batches=2)
    g, g_ref = build_both(w.src, w.dst, w.ts, w.eid, w.num_nodes)
    assert_tcsr_equal(g, g_ref)
    table = dev(w.edge_feat)
    for roots, times in w.batches:
        got, want = run_both(g, g_ref, roots, times, w.k, 2, W.WEIGHTED, seed=42, m=w.m, weight=w.edge_weight)
        for h in range(2):
            check_gather(w.edge_feat, table, got[h]["eid"], want[h]["eid"])


def test_c5_scaled_two_hop_recent_with_cache():
    """The GDELT-shaped workload at 2 M events (same node count, skew and tie density):
    full element-wise parity of sampler, pitched procedural edge table gather and the
    cached node-feature gather from pinned host memory."""
    w = W.make(5, edges=2_000_000, num_batches=2, last=200_000)
    g, g_ref = build_both(w.src, w.dst, w.ts, w.eid, w.num_nodes)
    assert_tcsr_equal(g, g_ref)
    pitch = 192                                                  # 384-byte rows for 372 bytes of data
    table = W.procedural_table_torch(w.edge_seed, w.num_edges, w.edge_dim, torch.float16, pitch, "cuda")
    node_host = torch.from_numpy(w.node_feat).pin_memory()
    cap = int(w.cache_ratio * w.num_nodes)
    hot = torch.from_numpy(np.ascontiguousarray(w.notes["hot_order"][:cap]))
    cache = T.cache_init(node_host, cap, hot, staging_rows=w.num_nodes - cap)
    for roots, times in w.batches:
        got, want = run_both(g, g_ref, roots, times, w.k, 2, W.RECENT, seed=42)
        for h in range(2):
            eids = want[h]["eid"].ravel()
            rows = W.procedural_rows(w.edge_seed, np.maximum(eids, 0), w.edge_dim, np.float16)
            rows[eids < 0] = 0
            out = T.gather_features(table, got[h]["eid"].reshape(-1), row_elems=w.edge_dim)
            assert out.cpu().numpy().tobytes() == rows.tobytes()
        ids_np = np.concatenate([roots, want[0]["nbr"].ravel(), want[1]["nbr"].ravel()])
        ids = torch.cat([dev(roots), got[0]["nbr"].reshape(-1), got[1]["nbr"].reshape(-1)])
        hm = torch.zeros(2, dtype=torch.int64, device="cuda")
        out = T.cache_lookup(cache, ids, hit_miss=hm)
        torch.cuda.synchronize()
        assert out.cpu().numpy().tobytes() == oracle.gather(w.node_feat, ids_np, threads=THREADS).tobytes()
        assert tuple(hm.tolist()) == oracle.cache_hits(hot.numpy(), w.num_nodes, ids_np)


# ----------------------------------------------------------------------------- sampler edge cases
def _graph(rng, n_nodes, n, span, sorted_ts=True, lo=0):
    src = rng.integers(0, n_nodes, n).astype(np.int32)
    dst = rng.integers(0, n_nodes, n).astype(np.int32)
    ts = rng.integers(lo, lo + span, n).astype(np.int64)
    if sorted_ts:
        ts.sort()
    eid = rng.permutation(n).astype(np.int32)
    return src, dst, ts, eid


@pytest.mark.parametrize("sorted_ts,lo,span", [(True, 0, 500), (False, 0, 500), (False, -(1 << 62), 1 << 40),
                                              (False, -300, 70000), (True, 5, 1)])
def test_tcsr_build_general_inputs(sorted_ts, lo, span):
    """Unsorted timestamps (the timestamp digits must then be sorted too), negative and
    huge timestamps, heavy ties, an empty node, host and device inputs, ragged tile."""
    rng = np.random.default_rng(17)
    n_nodes, n = 300, 3 * 4096 + 777
    src, dst, ts, eid = _graph(rng, n_nodes, n, span, sorted_ts, lo)
    src[src == 9] = 10
    for on_device in (True, False):
        g, g_ref = build_both(src, dst, ts, eid, n_nodes, on_device)
        assert_tcsr_equal(g, g_ref)
    g = T.tcsr_build(dev(src), dev(dst), dev(ts), None, n_nodes)            # eid defaults to the position
    _, _, _, got_eid = T.tcsr_view(g)
    ref = oracle.tcsr_build(src, dst, ts, np.arange(n, dtype=np.int32), n_nodes)
    assert np.array_equal(got_eid.cpu().numpy(), ref[3])


@pytest.mark.parametrize("n_nodes", [1, 2, 255, 257, 70000])
def test_tcsr_build_node_count_digits(n_nodes):
    rng = np.random.default_rng(n_nodes)
    src, dst, ts, eid = _graph(rng, n_nodes, 20000, 1000)
    g, g_ref = build_both(src, dst, ts, eid, n_nodes)
    assert_tcsr_equal(g, g_ref)


@pytest.mark.parametrize("n", [1, 63, 64, 65, 4095, 4096, 4097, 8192, 12288])
def test_tcsr_build_sizes_around_the_tile(n):
    """Entry counts at, just below and just above the sort tile (4096) and the row width (64),
    sorted and unsorted timestamps, followed by a sampling call that walks the time index."""
    rng = np.random.default_rng(n)
    for sorted_ts in (True, False):
        src, dst, ts, eid = _graph(rng, 37, n, 200, sorted_ts)
        g, g_ref = build_both(src, dst, ts, eid, 37)
        assert_tcsr_equal(g, g_ref)
        roots = rng.integers(0, 37, 100).astype(np.int32)
        times = rng.integers(-1, 205, 100).astype(np.int64)
        run_both(g, g_ref, roots, times, 5, 2, T.UNIFORM, seed=n)


def test_tcsr_build_empty_and_rejects_bad_ids():
    z32, z64 = torch.zeros(0, dtype=torch.int32), torch.zeros(0, dtype=torch.int64)
    g = T.tcsr_build(z32.cuda(), z32.cuda(), z64.cuda(), None, 5)
    indptr, nbr, _, _ = T.tcsr_view(g)
    assert indptr.tolist() == [0] * 6 and nbr.numel() == 0
    out = T.sample_temporal(g, dev(np.array([0, 4], np.int32)), dev(np.array([5, 5], np.int64)), 3, 2, T.UNIFORM, 1)
    assert out[0]["count"].tolist() == [0, 0] and out[1]["nbr"].shape == (6, 3) and int(out[1]["nbr"].max()) == -1
    with pytest.raises(T.TaserError) as e:
        T.tcsr_build(dev(np.array([0, 5], np.int32)), dev(np.array([1, 1], np.int32)), dev(np.array([0, 1], np.int64)),
                     None, 5)
    assert e.value.code == -2


@pytest.mark.parametrize("policy", [T.RECENT, T.UNIFORM, T.WEIGHTED])
@pytest.mark.parametrize("k,m", [(1, 2), (10, 25), (32, 64), (64, 64), (7, 5)])
def test_sampler_shapes_and_policies(policy, k, m):
    """Small and maximal k / m, three hops, degree mix from empty lists to thousands."""
    rng = np.random.default_rng(100 * k + m)
    n_nodes, n = 60, 30000
    src, dst, ts, eid = _graph(rng, n_nodes, n, 4000)
    src = np.minimum(src, rng.integers(0, n_nodes, n)).astype(np.int32)     # skewed degrees
    src[src == 7] = 8
    g, g_ref = build_both(src, dst, ts, eid, n_nodes)
    weight = rng.integers(1, 1 << 16, n).astype(np.uint32)
    roots = rng.integers(0, n_nodes, 333).astype(np.int32)
    roots[::50] = -1
    times = rng.integers(-5, 4100, 333).astype(np.int64)
    hops = 3 if k <= 7 else (2 if k <= 10 else 1)
    run_both(g, g_ref, roots, times, k, hops, policy, seed=0xABCDEF0123456789, m=m, weight=weight)


@pytest.mark.parametrize("policy", [T.RECENT, T.UNIFORM, T.WEIGHTED])
def test_sampler_long_lists_and_ties(policy):
    """Lists long enough for several rounds of the wave-wide search (64^3 < 300 k), query
    times on, between and outside the timestamps, and long runs of equal timestamps."""
    rng = np.random.default_rng(4)
    n = 300_000
    src = np.zeros(n, np.int32)
    src[-5000:] = 1
    src[-70:-64] = 2
    dst = rng.integers(0, 4, n).astype(np.int32)
    ts = np.sort(rng.integers(0, 3000, n)).astype(np.int64) * 7          # ~100 equal timestamps in a row
    eid = np.arange(n, dtype=np.int32)
    g, g_ref = build_both(src, dst, ts, eid, 4)
    weight = rng.integers(1, 1 << 16, n).astype(np.uint32)
    times = np.concatenate([np.arange(-2, 90), rng.integers(0, 21010, 1500), [21000, 20993, 20994, 1 << 62, -(1 << 62)]])
    roots = rng.integers(0, 4, times.shape[0]).astype(np.int32)
    roots[:92] = 0
    run_both(g, g_ref, roots, times.astype(np.int64), 10, 2, policy, seed=7, m=25, weight=weight)


@pytest.mark.parametrize("policy", [T.RECENT, T.UNIFORM])
def test_sampler_many_roots(policy):
    """Three million roots in one call (both lane-group widths of the most-recent finder's
    launch, tens of thousands of blocks), compared element by element."""
    rng = np.random.default_rng(33)
    n_nodes, n = 500, 20000
    src, dst, ts, eid = _graph(rng, n_nodes, n, 100000)
    g, g_ref = build_both(src, dst, ts, eid, n_nodes)
    R = 3_000_001
    roots = rng.integers(-1, n_nodes, R).astype(np.int32)
    times = rng.integers(0, 100010, R).astype(np.int64)
    run_both(g, g_ref, roots, times, 10, 1, policy, seed=9)


def test_sampler_weight_extremes():
    """uint32 weights up to 2^32 - 1: the running sums need 64 bits."""
    rng = np.random.default_rng(12)
    src, dst, ts, eid = _graph(rng, 5, 4000, 9000)
    g, g_ref = build_both(src, dst, ts, eid, 5)
    weight = rng.integers(1, 1 << 32, 4000, dtype=np.uint64).astype(np.uint32)
    weight[::3] = 0xFFFFFFFF
    weight[1::5] = 1
    roots = rng.integers(0, 5, 500).astype(np.int32)
    times = rng.integers(0, 9000, 500).astype(np.int64)
    run_both(g, g_ref, roots, times, 16, 1, T.WEIGHTED, seed=3, m=64, weight=weight)


def test_sampler_is_deterministic_and_independent_of_batch_split():
    w = W.make(1)
    g, _ = build_both(w.src, w.dst, w.ts, w.eid, w.num_nodes)
    roots, times = w.batches[9]
    a = T.sample_temporal(g, dev(roots), dev(times), 10, 2, T.UNIFORM, 5)
    b = T.sample_temporal(g, dev(roots), dev(times), 10, 2, T.UNIFORM, 5)
    for h in range(2):
        for f in FIELDS:
            assert torch.equal(a[h][f], b[h][f])
    c = T.sample_temporal(g, dev(roots), dev(times), 10, 1, T.UNIFORM, 6)
    assert not torch.equal(a[0]["eid"], c[0]["eid"])                  # the seed matters
    assert torch.equal(a[0]["count"], c[0]["count"])


@pytest.mark.parametrize("seed", range(24))
def test_random_graphs_all_policies(seed):
    """Randomly shaped small graphs (node count, size, time span, sorted or not, degree skew), random
    k, m, hops, root counts around the wave and block sizes: the whole path, build included."""
    rng = np.random.default_rng(9000 + seed)
    n_nodes = int(rng.choice([1, 2, 3, 17, 200, 5000]))
    n = int(rng.choice([1, 50, 700, 5000, 40000]))
    span = int(rng.choice([1, 3, 100, 100000, 1 << 40]))
    src, dst, ts, eid = _graph(rng, n_nodes, n, span, sorted_ts=bool(rng.integers(0, 2)), lo=int(rng.choice([0, -span // 2, -(1 << 50)])))
    if rng.integers(0, 2):
        src = np.minimum(src, rng.integers(0, n_nodes, n)).astype(np.int32)
    g, g_ref = build_both(src, dst, ts, eid, n_nodes)
    assert_tcsr_equal(g, g_ref)
    weight = rng.integers(1, int(rng.choice([2, 1 << 16, (1 << 32) - 1])), n, dtype=np.int64).astype(np.uint32)
    dim = int(rng.choice([4, 6, 16, 43]))
    table = rng.standard_normal((n, dim)).astype(np.float32)
    table_dev = dev(table)
    for _ in range(3):
        k = int(rng.choice([1, 2, 5, 10, 16, 17, 32, 33, 64]))
        m = int(rng.integers(1, 65))
        hops = 3 if k <= 5 else (2 if k <= 10 else 1)
        n_roots = int(rng.choice([1, 3, 4, 5, 63, 64, 65, 255, 257, 1000]))
        roots = rng.integers(-1, n_nodes, n_roots).astype(np.int32)                # some negative (roots without neighbors)
        times = rng.integers(int(ts.min()) - 2, int(ts.max()) + 3, n_roots).astype(np.int64)
        for policy in (T.RECENT, T.UNIFORM, T.WEIGHTED, T.INVERSE_TIMESPAN):
            check_rows_call(g, g_ref, roots, times, k, hops, policy, int(rng.integers(0, 1 << 62)), table, table_dev, m=m, weight=weight)


# ----------------------------------------------------------------------------- inverse-timespan finder
@pytest.mark.parametrize("k", [1, 10, 64])
def test_inverse_timespan_matches_the_oracle(k):
    """Lists from empty to tens of thousands of entries (one and several rows per tile),
    ties, three hops for small k, invalid roots."""
    rng = np.random.default_rng(50 + k)
    n_nodes, n = 40, 120000
    src, dst, ts, eid = _graph(rng, n_nodes, n, 50000)
    src = np.minimum(src, rng.integers(0, n_nodes, n)).astype(np.int32)
    src[:40000] = 0                                                     # one list of > 40 000 entries: > 512 rows
    src[src == 7] = 8
    g, g_ref = build_both(src, dst, ts, eid, n_nodes)
    roots = rng.integers(0, n_nodes, 400).astype(np.int32)
    roots[::9] = 0
    roots[::50] = -1
    times = rng.integers(-5, 50100, 400).astype(np.int64)
    hops = 3 if k == 1 else (2 if k == 10 else 1)
    run_both(g, g_ref, roots, times, k, hops, T.INVERSE_TIMESPAN, seed=0x1234567890ABCDEF)


def test_inverse_timespan_long_list_and_extreme_deltas():
    """A 300 000-entry list (several rows per tile), query times on / between / outside the
    timestamps, time deltas from 1 to beyond 2^32 (weight 1) and int64 extremes."""
    rng = np.random.default_rng(9)
    n = 300_000
    src = np.zeros(n, np.int32)
    src[-4000:] = 1
    dst = rng.integers(0, 3, n).astype(np.int32)
    ts = np.sort(np.concatenate([rng.integers(-(1 << 62), -(1 << 61), 1000), rng.integers(0, 1 << 34, n - 1000)]))
    ts = ts.astype(np.int64)
    g, g_ref = build_both(src, dst, ts, np.arange(n, dtype=np.int32), 3)
    times = np.concatenate([ts[rng.integers(0, n, 150)] + rng.integers(0, 3, 150), [1 << 62, -(1 << 62), 5, (1 << 34) + 7]])
    roots = rng.integers(0, 2, times.shape[0]).astype(np.int32)
    roots[:100] = 0
    run_both(g, g_ref, roots, times.astype(np.int64), 10, 1, T.INVERSE_TIMESPAN, seed=3)


def test_inverse_timespan_on_the_flights_shaped_workload():
    w = W.make(4, num_batches=1)
    g, g_ref = build_both(w.src, w.dst, w.ts, w.eid, w.num_nodes)
    roots, times = w.batches[0]
    run_both(g, g_ref, roots[:1000], times[:1000], w.k, 2, T.INVERSE_TIMESPAN, seed=42)


# ----------------------------------------------------------------------------- candidate-window products
@pytest.mark.parametrize("m", [1, 5, 16, 25, 32, 33, 64])
def test_candidate_encodings_match_the_oracle(m):
    """Frequency and identity encodings for every lane-group width, with repeated
    neighbors, short windows, counts beyond m and below 0, and a ragged last wave."""
    rng = np.random.default_rng(m)
    for R in (0, 1, 3, 64, 1000 + m):
        nbr = rng.integers(0, max(2, m // 3), (R, m)).astype(np.int32)          # few distinct nodes: many repeats
        nbr[::7] = rng.integers(0, 1 << 30, (len(nbr[::7]), m))                  # mostly distinct rows
        count = rng.integers(0, m + 1, R).astype(np.int32)
        count[::5] = m
        count[3::11] = m + 9
        count[4::13] = -2
        want_f, want_i = oracle.candidate_encodings(nbr, count)
        got_f, got_i = T.candidate_encodings(dev(nbr), dev(count))
        torch.cuda.synchronize()
        assert np.array_equal(got_f.cpu().numpy(), want_f)
        assert np.array_equal(got_i.cpu().numpy(), want_i)
        got_f2, none = T.candidate_encodings(dev(nbr), dev(count), want_identity=False)
        assert none is None and torch.equal(got_f, got_f2)


def test_candidate_encodings_unaligned_identity_output():
    """The identity bytes of a wave are written as aligned 4-byte words with byte
    stores at the ragged ends: give the output every alignment, guard bytes around it."""
    rng = np.random.default_rng(2)
    R, m = 37, 7
    nbr = rng.integers(0, 3, (R, m)).astype(np.int32)
    count = rng.integers(0, m + 1, R).astype(np.int32)
    _, want_i = oracle.candidate_encodings(nbr, count)
    nbr_d, count_d = dev(nbr), dev(count)
    freq = torch.empty((R, m), dtype=torch.int32, device="cuda")
    for off in range(4):
        buf = torch.full((R * m * m + 16,), 0xEE, dtype=torch.uint8, device="cuda")
        view = buf[4 + off:4 + off + R * m * m]
        T._check(T.lib().taser_candidate_encodings(T._ptr(nbr_d), T._ptr(count_d), R, m, T._ptr(freq), T._ptr(view),
                                                   T._stream(None)))
        torch.cuda.synchronize()
        got = buf.cpu().numpy()
        assert np.array_equal(got[4 + off:4 + off + R * m * m], want_i.ravel())
        assert (got[:4 + off] == 0xEE).all() and (got[4 + off + R * m * m:] == 0xEE).all()


@pytest.mark.parametrize("m,k", [(2, 1), (25, 10), (16, 16), (32, 10), (64, 32), (64, 64), (5, 10), (40, 3)])
def test_select_weighted_matches_the_oracle(m, k):
    rng = np.random.default_rng(1000 * m + k)
    for R in (0, 1, 65, 2000 + k):
        weight = rng.integers(1, 1 << 16, (R, m), dtype=np.uint64).astype(np.uint32)
        weight[::3] = rng.integers(1, 1 << 32, (len(weight[::3]), m), dtype=np.uint64).astype(np.uint32)
        weight[1::9] = 0xFFFFFFFF
        count = rng.integers(0, m + 1, R).astype(np.int32)
        count[::4] = m
        count[5::17] = m + 3
        for hop in (0, 2):
            want_sel, want_cnt = oracle.select_weighted(weight, count, k, seed=77, hop=hop)
            sel, cnt, kept = T.select_weighted(dev(weight.view(np.int32)), dev(count), k, 77, hop)
            torch.cuda.synchronize()
            assert kept is None
            assert np.array_equal(sel.cpu().numpy(), want_sel)
            assert np.array_equal(cnt.cpu().numpy(), want_cnt)


def test_adaptive_two_hop_pipeline_on_the_flights_shaped_workload():
    """Alg. 1 as the adaptive sampler runs it, per hop: m most recent candidates, their
    encodings and feature rows, a weight per (root, candidate), n of m kept, kept
    neighbors become the next hop's roots. The weights stand in for the network's
    output: here the per-edge table, so the whole pipeline must also reproduce the
    one-call weighted policy."""
    w = W.make(4, num_batches=1)
    g, g_ref = build_both(w.src, w.dst, w.ts, w.eid, w.num_nodes)
    table = dev(w.edge_feat)
    weight_dev = dev(w.edge_weight.view(np.int32))
    roots, times = w.batches[0]
    fused = oracle.sample_temporal(g_ref, roots, times, w.k, 2, W.WEIGHTED, 42, w.m, w.edge_weight, THREADS)
    cur_roots, cur_times = dev(roots), dev(times)
    ref_roots, ref_times = roots, times
    for hop in range(2):
        cand = T.sample_temporal(g, cur_roots, cur_times, w.m, 1, T.RECENT, seed=0)[0]
        ref_cand = oracle.sample_temporal(g_ref, ref_roots, ref_times, w.m, 1, W.RECENT, 0, threads=THREADS)[0]
        freq, ident = T.candidate_encodings(cand["nbr"], cand["count"])
        ref_freq, ref_ident = oracle.candidate_encodings(ref_cand["nbr"], ref_cand["count"])
        check_gather(w.edge_feat, table, cand["eid"], ref_cand["eid"])          # all m candidates' rows
        slot_w = torch.where(cand["eid"] >= 0, weight_dev[cand["eid"].clamp(min=0).long()], 0).contiguous()
        ref_slot_w = np.where(ref_cand["eid"] >= 0, w.edge_weight[np.maximum(ref_cand["eid"], 0)], 0).astype(np.uint32)
        sel, cnt, kept = T.select_weighted(slot_w, cand["count"], w.k, 42, hop, candidates=cand)
        ref_sel, ref_cnt = oracle.select_weighted(ref_slot_w, ref_cand["count"], w.k, 42, hop)
        torch.cuda.synchronize()
        assert np.array_equal(freq.cpu().numpy(), ref_freq) and np.array_equal(ident.cpu().numpy(), ref_ident)
        assert np.array_equal(sel.cpu().numpy(), ref_sel) and np.array_equal(cnt.cpu().numpy(), ref_cnt)
        take = np.maximum(ref_sel, 0)
        for f, pad in (("nbr", -1), ("eid", -1), ("ts", 0)):
            want = np.where(ref_sel >= 0, np.take_along_axis(ref_cand[f], take, axis=1), pad)
            assert np.array_equal(kept[f].cpu().numpy(), want), (hop, f)
            assert np.array_equal(want, fused[hop][f]), (hop, f)                # equals the one-call policy
        assert np.array_equal(ref_cnt, fused[hop]["count"])
        cur_roots, cur_times = kept["nbr"].reshape(-1), kept["ts"].reshape(-1)
        ref_roots, ref_times = fused[hop]["nbr"].ravel(), fused[hop]["ts"].ravel()


# ----------------------------------------------------------------------------- sampling with the rows in one call
def check_rows_call(g, g_ref, roots, times, k, hops, policy, seed, table_np, table_dev, m=0, weight=None, table_rows=None):
    """taser_sample_temporal_rows against the oracle's finder followed by the oracle's gather;
    the row buffers carry guard elements behind the last row."""
    want = oracle.sample_temporal(g_ref, roots, times, k, hops, policy, seed, m, weight, THREADS)
    d = table_np.shape[1]
    guard = 64
    bufs, r = [], roots.shape[0]
    for _ in range(hops):
        r *= k
        bufs.append(torch.full((r * d + guard,), 77, dtype=table_dev.dtype, device="cuda"))
    w_dev = None if weight is None else dev(weight.view(np.int32))
    t_dev = table_dev if table_rows is None else table_dev[:table_rows]
    got, rows = T.sample_temporal_rows(g, dev(roots), dev(times), k, hops, policy, seed, t_dev, m=m, edge_weight=w_dev,
                                       rows_out=bufs, row_elems=d)
    torch.cuda.synchronize()
    assert_hops_equal(got, want)
    for h in range(hops):
        ids = want[h]["eid"].ravel().copy()
        if table_rows is not None:
            ids[ids >= table_rows] = -1
        ref = oracle.gather(table_np, ids, threads=THREADS)
        out = rows[h].cpu().numpy()
        a, b = out[:ids.shape[0] * d].view(np.uint8), ref.ravel().view(np.uint8)
        if a.tobytes() != b.tobytes():
            at = int(np.flatnonzero(a != b)[0])
            rb = d * table_np.itemsize
            raise AssertionError(f"rows of hop {h}: {int((a != b).sum())} bytes differ, the first in row {at // rb} "
                                 f"(id {ids[at // rb]}) at byte {at % rb} of {rb}")
        assert (out[ids.shape[0] * d:] == 77).all(), f"guard behind hop {h}"


@pytest.mark.parametrize("policy", [T.RECENT, T.UNIFORM, T.WEIGHTED, T.INVERSE_TIMESPAN])
@pytest.mark.parametrize("k,m,dtype,dim,pad,offset", [
    (10, 25, np.float16, 172, 0, 0),     # 344-byte rows: every other row starts 8 bytes off a 16-byte boundary
    (10, 25, np.float16, 186, 6, 0),     # 372 bytes at a 384-byte pitch
    (7, 5, np.float16, 186, 0, 0),       # a last wavefront whose rows end inside a 16-byte piece
    (10, 12, np.float32, 16, 0, 0),      # 64-byte rows: sixteen rows per wave instruction
    (10, 25, np.float32, 413, 0, 0),     # 1652 bytes: too many bytes per wavefront for the hop kernel -> gather launch
    (32, 64, np.float32, 4, 0, 0),       # 16-byte rows, the shortest the hop kernel copies itself
    (1, 2, np.float32, 500, 0, 0),       # 2000-byte rows, one slot per root: rows longer than a wave instruction, copied by the hop kernel
    (2, 2, np.float32, 413, 0, 0),       # 1652-byte rows of two slots: beyond what the hop kernel copies itself -> gather launch
    (1, 2, np.float32, 5, 3, 0),         # one slot per root, 20-byte rows
    (64, 64, np.float16, 172, 0, 0),     # one root per wavefront, 22 KB of rows -> gather launch
    (64, 64, np.float16, 62, 0, 0),      # one root per wavefront, 124-byte rows
    (3, 40, np.float16, 10, 0, 0),       # 20-byte rows of three slots: a wavefront's rows are not whole 16-byte pieces -> two launches
    (10, 25, np.float16, 7, 0, 0),       # 14-byte rows -> two launches
    (10, 25, np.float16, 9, 3, 1),       # odd pitch, table starting 2 bytes into an allocation -> two launches
])
def test_sampling_with_rows_equals_the_oracle(policy, k, m, dtype, dim, pad, offset):
    rng = np.random.default_rng(1000 * k + dim)
    n_nodes, n = 60, 30000
    src, dst, ts, eid = _graph(rng, n_nodes, n, 4000)
    src = np.minimum(src, rng.integers(0, n_nodes, n)).astype(np.int32)     # skewed degrees, some empty lists
    src[src == 7] = 8
    g, g_ref = build_both(src, dst, ts, eid, n_nodes)
    weight = rng.integers(1, 1 << 16, n).astype(np.uint32)
    full = rng.standard_normal((n, dim + pad + offset)).astype(dtype)
    table = full[:, offset:offset + dim]
    table_dev = dev(full)[:, offset:offset + dim]
    hops = 3 if k <= 7 else (2 if k <= 10 else 1)
    for n_roots in (333, 1, 64):
        roots = rng.integers(0, n_nodes, n_roots).astype(np.int32)
        roots[::50] = -1
        times = rng.integers(-5, 4100, n_roots).astype(np.int64)
        check_rows_call(g, g_ref, roots, times, k, hops, policy, 0xABCDEF0123456789, table, table_dev, m=m, weight=weight)
    # a table that ends before the largest edge id: zero rows beyond it
    roots = rng.integers(0, n_nodes, 100).astype(np.int32)
    times = rng.integers(2000, 4100, 100).astype(np.int64)
    check_rows_call(g, g_ref, roots, times, k, 1, policy, 5, table, table_dev, m=m, weight=weight, table_rows=n // 2)


def test_sampling_with_rows_on_the_reddit_and_flights_shaped_workloads():
    w = W.make(3, num_batches=2)
    g, g_ref = build_both(w.src, w.dst, w.ts, w.eid, w.num_nodes)
    table = dev(w.edge_feat)
    for roots, times in w.batches:
        check_rows_call(g, g_ref, roots, times, w.k, 2, W.UNIFORM, 42, w.edge_feat, table)
    w = W.make(4, num_batches=2)
    g, g_ref = build_both(w.src, w.dst, w.ts, w.eid, w.num_nodes)
    table = dev(w.edge_feat)
    for roots, times in w.batches:
        check_rows_call(g, g_ref, roots, times, w.k, 2, W.WEIGHTED, 42, w.edge_feat, table, m=w.m, weight=w.edge_weight)


# ----------------------------------------------------------------------------- gather edge cases
@pytest.mark.parametrize("dtype,dim,pad,offset", [
    (np.float32, 16, 0, 0),      # 64-byte rows, 16-byte vectors
    (np.float32, 172, 0, 0),     # 688 bytes
    (np.float16, 172, 0, 0),     # 344 bytes: 8-byte vectors
    (np.float16, 186, 0, 0),     # 372 bytes: 4-byte vectors, unpadded
    (np.float16, 186, 6, 0),     # 372 bytes at a 384-byte pitch
    (np.float32, 413, 0, 0),     # 1652 bytes
    (np.float16, 7, 0, 0),       # 14 bytes: 2-byte path
    (np.float16, 9, 3, 1),       # odd everything, table view starting 2 bytes into an allocation
    (np.float32, 1, 0, 0),       # 4-byte rows
    (np.float32, 300, 20, 4),    # 1200 bytes, 16-byte aligned data inside a wider pitch
])
def test_gather_alignments(dtype, dim, pad, offset):
    rng = np.random.default_rng(dim)
    rows = 3000
    full = rng.standard_normal((rows, dim + pad + offset)).astype(dtype)
    table = full[:, offset:offset + dim]
    full_dev = dev(full)
    table_dev = full_dev[:, offset:offset + dim]
    for n in (0, 1, 63, 1025, 7777):
        ids = rng.integers(0, rows, n).astype(np.int32)
        ids[::11] = -1
        got = T.gather_features(table_dev, dev(ids))
        assert got.shape == (n, dim)
        assert got.cpu().numpy().tobytes() == oracle.gather(table, ids).tobytes()


def test_gather_out_of_range_ids_give_zero_rows():
    table = torch.arange(40, dtype=torch.float32, device="cuda").reshape(10, 4)
    out = T.gather_features(table, dev(np.array([3, 10, 2 ** 31 - 1, -7, 9], np.int32)))
    assert out.tolist() == [[12, 13, 14, 15], [0] * 4, [0] * 4, [0] * 4, [36, 37, 38, 39]]


# ----------------------------------------------------------------------------- cache
@pytest.mark.parametrize("cap_frac,staging", [(0.0, 0), (0.0, 10000), (0.2, 0), (0.2, 16), (0.2, 5000), (1.0, 0)])
def test_cache_serves_identical_bytes_whatever_is_resident(cap_frac, staging):
    rng = np.random.default_rng(77)
    rows, dim = 5000, 413
    host = torch.from_numpy(rng.standard_normal((rows, dim)).astype(np.float32)).pin_memory()
    cap = int(cap_frac * rows)
    ids = np.minimum(rng.zipf(1.3, 60000) - 1, rows - 1).astype(np.int32)
    ids[::97] = -1
    want = oracle.gather(host.numpy(), ids, threads=THREADS)
    for residents in (None, torch.from_numpy(rng.permutation(rows)[:cap].astype(np.int32))):
        c = T.cache_init(host, cap, residents, seed=9, staging_rows=staging)
        res = T.cache_residents(c).numpy()
        if residents is None:
            assert np.array_equal(res, oracle.cache_random_residents(rows, cap, 9))
        else:
            assert np.array_equal(res, residents.numpy())
        hm = torch.zeros(2, dtype=torch.int64, device="cuda")
        for _ in range(2):                                            # the per-call staging state is reset
            out = T.cache_lookup(c, dev(ids), hit_miss=hm)
            torch.cuda.synchronize()
            assert out.cpu().numpy().tobytes() == want.tobytes()
        h, m = oracle.cache_hits(res, rows, ids)
        assert tuple(hm.tolist()) == (2 * h, 2 * m)
        out = T.cache_lookup(c, dev(ids[:100]))                       # shrinking n, no counters
        assert out.cpu().numpy().tobytes() == want[:100].tobytes()
        T.cache_free(c)


@pytest.mark.parametrize("dim,n", [(128, 5000), (129, 4099), (413, 70001), (1025, 4097), (4096, 4096), (4095, 4100), (127, 9000)])
def test_cache_partitioned_gather_equals_the_oracle(dim, n):
    """The gather that hands the output out in 128-byte lines by source row (rows of 512 bytes and
    more), before and after an epoch end has marked the most requested rows, and with every row
    spread by position: same bytes as the oracle, and as the plain gather in output order."""
    rng = np.random.default_rng(dim * 7 + n)
    rows = 900
    host = torch.from_numpy(rng.standard_normal((rows, dim)).astype(np.float32)).pin_memory()
    cap = 300
    c = T.cache_init(host, cap, torch.from_numpy(rng.permutation(rows)[:cap].astype(np.int32)), staging_rows=200)
    T.cache_count_accesses(c)
    for epoch in range(2):
        ids_np = np.minimum(rng.zipf(1.1, n) - 1, rows - 1).astype(np.int32)
        ids_np[::41] = -1
        ids_np[5::577] = rows                                        # out of range: a zero row
        ids_np[-3:] = [-1, 7, -1]                                    # zero rows around the ragged end
        ids = dev(ids_np)
        want = oracle.gather(host.numpy(), np.where(ids_np >= rows, -1, ids_np), threads=THREADS).tobytes()
        for mode in (1, 0, 2):
            T.cache_tune(c, partitioned_gather=mode)
            out = torch.full((n, dim), float("nan"), dtype=torch.float32, device="cuda")
            T.cache_lookup(c, ids, out=out)
            torch.cuda.synchronize()
            assert out.cpu().numpy().tobytes() == want, (epoch, mode)
        T.cache_epoch_end(c, min_overlap=cap if epoch == 0 else 0)     # marks hot rows (and swaps the content once)


@pytest.mark.parametrize("seed", range(16))
def test_cache_random_shapes(seed):
    """Random table shapes (row lengths on both sides of every kernel's limits, fp16 and fp32, padded
    pitch), capacities, staging sizes, request counts and skews; every gather mode, the
    allocation-free lookup, hit/miss counts, access counters and one epoch end in between."""
    rng = np.random.default_rng(31000 + seed)
    rows = int(rng.choice([1, 7, 300, 2000, 9000]))
    dtype = [np.float16, np.float32][int(rng.integers(0, 2))]
    dim = int(rng.choice([1, 2, 3, 8, 31, 64, 127, 128, 129, 256, 413, 1025]))
    pad = int(rng.choice([0, 0, 1, 5]))
    if dtype is np.float16:
        dim, pad = 2 * dim, 2 * pad                                  # the cache wants rows and pitch in whole 4-byte words
    full = torch.from_numpy(rng.standard_normal((rows, dim + pad)).astype(dtype)).pin_memory()
    host = full[:, :dim]
    cap = int(rng.choice([0, 1, rows // 5, rows // 2, rows]))
    staging = int(rng.choice([0, 3, rows // 3, rows]))
    residents = torch.from_numpy(rng.permutation(rows)[:cap].astype(np.int32)) if rng.integers(0, 2) else None
    c = T.cache_init(host, cap, residents, seed=seed, staging_rows=staging)
    res = T.cache_residents(c).numpy()
    T.cache_count_accesses(c)
    Q = np.zeros(rows, np.uint32)
    for call in range(4):
        n = int(rng.choice([1, 63, 500, 4096, 4097, 30000]))
        a = float(rng.choice([1.05, 1.5, 3.0]))
        ids_np = ((rng.zipf(a, n) - 1) % rows).astype(np.int32) if rng.integers(0, 2) else rng.integers(0, rows, n).astype(np.int32)
        ids_np[::13] = -1
        ids = dev(ids_np)
        want = oracle.gather(host.numpy(), ids_np, threads=THREADS).tobytes()
        hm = torch.zeros(2, dtype=torch.int64, device="cuda")
        mode = int(rng.integers(0, 3))
        T.cache_tune(c, partitioned_gather=mode)
        out = torch.full((n, dim), 5.0, dtype=host.dtype, device="cuda")
        if call % 2:
            T.cache_lookup_static(c, ids, out, hit_miss=hm)
        else:
            T.cache_lookup(c, ids, out=out, hit_miss=hm)
        torch.cuda.synchronize()
        assert out.cpu().numpy().tobytes() == want, (call, mode, n)
        assert tuple(hm.tolist()) == oracle.cache_hits(res, rows, ids_np)
        oracle.cache_count(ids_np, rows, Q)
        assert np.array_equal(T.cache_access_counts(c).cpu().numpy().astype(np.uint32), Q)
        if call == 1:
            T.cache_epoch_end(c, min_overlap=cap)                    # replaces the content by the most requested rows
            res = T.cache_residents(c).numpy()
            Q[:] = 0
    T.cache_free(c)


def test_cache_rejects_unpinned_and_bad_residents():
    host = torch.zeros((100, 8), dtype=torch.float32)
    with pytest.raises(T.TaserError) as e:
        T.cache_init(host, 10)
    assert e.value.code == -1 and "page-locked" in str(e.value)
    pinned = host.pin_memory()
    with pytest.raises(T.TaserError) as e:
        T.cache_init(pinned, 2, torch.tensor([5, 5], dtype=torch.int32))
    assert e.value.code == -2
    # an error from the library leaves HIP usable
    c = T.cache_init(pinned, 2, torch.tensor([5, 6], dtype=torch.int32))
    assert T.cache_lookup(c, dev(np.array([5, 1], np.int32))).abs().sum().item() == 0


def test_cache_prefetch_then_gather_on_two_streams():
    """The two halves of a lookup, the bus-bound half on a side stream, joined by events;
    a gather that does not match the latest prefetch is refused."""
    rng = np.random.default_rng(5)
    rows, dim = 3000, 93
    host = torch.from_numpy(rng.standard_normal((rows, dim)).astype(np.float32)).pin_memory()
    c = T.cache_init(host, 600, None, seed=1, staging_rows=2400)
    main, side = torch.cuda.current_stream(), torch.cuda.Stream()
    for n in (50000, 777, 50001):
        T.cache_tune(c, stage_blocks=3 if n == 777 else 16, refresh_before_gather=(n != 50000))
        ids_np = np.minimum(rng.zipf(1.2, n) - 1, rows - 1).astype(np.int32)
        ids = dev(ids_np)
        done_ids, staged = torch.cuda.Event(), torch.cuda.Event()
        done_ids.record(main)
        side.wait_event(done_ids)
        T.cache_prefetch(c, ids, stream=side)
        staged.record(side)
        main.wait_event(staged)
        out = T.cache_gather(c, ids, stream=main)
        torch.cuda.synchronize()
        assert out.cpu().numpy().tobytes() == oracle.gather(host.numpy(), ids_np).tobytes()
    with pytest.raises(T.TaserError) as e:
        T.cache_gather(c, ids[:10])
    assert e.value.code == -1


# ----------------------------------------------------------------------------- cache maintenance (Alg. 3)
def test_cache_access_counts_and_epoch_end_match_the_oracle():
    """Counters, top-k with ties, overlap threshold, replacement and what is served afterwards,
    over several epochs of a drifting skewed request stream."""
    rng = np.random.default_rng(31)
    rows, dim, cap = 5000, 24, 700
    host_np = rng.standard_normal((rows, dim)).astype(np.float32)
    host = torch.from_numpy(host_np).pin_memory()
    c = T.cache_init(host, cap, None, seed=2, staging_rows=512)
    with pytest.raises(T.TaserError):
        T.cache_epoch_end(c, 1)                                    # counting not enabled yet
    T.cache_count_accesses(c)
    resident = oracle.cache_random_residents(rows, cap, 2)
    Q = np.zeros(rows, np.uint32)
    p = 1.0 / np.arange(1, rows + 1) ** 1.1
    p /= p.sum()
    perm = rng.permutation(rows)
    replaced_any = kept_any = False
    for epoch in range(6):
        if epoch % 2 == 0:
            perm = np.roll(perm, 37 * epoch)                       # the hot set drifts
        for batch in range(3):
            n = (70000, 333, 20001)[batch]
            ids = perm[rng.choice(rows, n, p=p)].astype(np.int32)
            ids[::53] = -1
            ids[5::97] = rows + 3                                  # out of range: served as zero rows, not counted
            hm = torch.zeros(2, dtype=torch.int64, device="cuda")
            out = T.cache_lookup(c, dev(ids), hit_miss=hm)
            torch.cuda.synchronize()
            ok = np.where(ids < rows, ids, -1)
            assert out.cpu().numpy().tobytes() == oracle.gather(host_np, ok).tobytes()
            assert tuple(hm.tolist()) == oracle.cache_hits(resident, rows, ok)
            oracle.cache_count(ids, rows, Q)
        assert np.array_equal(T.cache_access_counts(c).cpu().numpy().view(np.uint32), Q)
        thr = (cap, 0, cap // 2, cap, cap - 5, 1)[epoch]
        want_rep, want_ov, resident = oracle.cache_epoch_end(Q, resident, thr)
        rep, ov = T.cache_epoch_end(c, thr)
        assert (rep, ov) == (want_rep, want_ov)
        assert np.array_equal(T.cache_residents(c).numpy(), resident)
        assert not T.cache_access_counts(c).any()
        replaced_any |= rep
        kept_any |= not rep
    assert replaced_any and kept_any


def test_cache_epoch_end_ties_and_extremes():
    """Nothing requested (all ties at zero: the smallest ids win), everything requested equally,
    one row requested 2^20 times by a single batch, capacity 0 and capacity = rows."""
    rows, dim = 1000, 4
    host_np = np.arange(rows * dim, dtype=np.float32).reshape(rows, dim)
    host = torch.from_numpy(host_np).pin_memory()
    for cap in (0, 1, 37, rows):
        c = T.cache_init(host, cap, None, seed=7)
        T.cache_count_accesses(c)
        resident = oracle.cache_random_residents(rows, cap, 7)
        Q = np.zeros(rows, np.uint32)
        streams = [np.zeros(0, np.int32), np.arange(rows, dtype=np.int32).repeat(3),
                   np.concatenate([np.full(1 << 20, 999, np.int32), np.arange(0, rows, 7, dtype=np.int32)])]
        for ids in streams:
            if ids.shape[0]:
                T.cache_lookup(c, dev(ids))
                oracle.cache_count(ids, rows, Q)
            assert np.array_equal(T.cache_access_counts(c).cpu().numpy().view(np.uint32), Q)
            want_rep, want_ov, resident = oracle.cache_epoch_end(Q, resident, cap)
            assert T.cache_epoch_end(c, cap) == (want_rep, want_ov)
            assert np.array_equal(T.cache_residents(c).numpy(), resident)
            probe = np.arange(rows, dtype=np.int32)
            hm = torch.zeros(2, dtype=torch.int64, device="cuda")
            out = T.cache_lookup(c, dev(probe), hit_miss=hm)
            assert out.cpu().numpy().tobytes() == host_np.tobytes()
            assert tuple(hm.tolist()) == (cap, rows - cap)
            oracle.cache_count(probe, rows, Q)


def test_cache_policy_replay_tracks_the_all_knowing_cache():
    """The replay script of the Fig. 3(b) experiment on a small drifting stream: after the first
    epoch the policy's hit rate stays close to the cache that knows the epoch's frequencies, and
    both grow with the cache size."""
    from paper_2402_05396_amd import cache_policy_replay
    res = cache_policy_replay.main(["--rows", "3000", "--dim", "8", "--epochs", "4", "--batches", "3",
                                    "--requests", "60000"])
    later = {k: v[1:] for k, v in res["ratios"].items()}
    for rows in later.values():
        for r in rows:
            assert r["all_knowing"] - 0.05 < r["hit_rate"] <= r["all_knowing"] + 1e-9
    assert later["10%"][-1]["hit_rate"] < later["20%"][-1]["hit_rate"] < later["30%"][-1]["hit_rate"]
    assert res["ratios"]["20%"][0]["hit_rate"] < 0.5 < later["20%"][0]["hit_rate"]          # random start, then learned


# ----------------------------------------------------------------------------- adaptive mini-batch selection
@pytest.mark.parametrize("n", [1, 63, 1024, 1025, 70000, (1 << 20) + 5, 3_000_000])
def test_selector_draws_and_updates_match_the_oracle(n):
    """Several iterations of draw -> update (with edges named twice, padding and out-of-range
    entries), sizes around the partial-sum boundaries (1024, 1024^2)."""
    rng = np.random.default_rng(n)
    score = rng.integers(0, 1 << 17, n, dtype=np.uint64).astype(np.uint32)
    score[rng.integers(0, n, n // 4)] = 0
    if n > 2000:
        score[1024:2048] = 0                                       # a whole level-1 block of zeros
        score[-3:] = 0xFFFFFFFF
    score[0] = max(score[0], 1)
    s = T.selector_init(dev(score.view(np.int32)))
    assert T.selector_size(s) == n
    for it, b in enumerate((600, 1, 4000, 65)):
        want = oracle.batch_draw(score, b, seed=11, iteration=it)
        got = T.selector_draw(s, b, 11, it)
        torch.cuda.synchronize()
        assert np.array_equal(got.cpu().numpy(), want)
        idx = want.copy()
        idx[::7] = idx[0]                                          # the same edge several times: the last value stays
        idx[3::11] = -1
        idx[5::13] = n + 2
        val = rng.integers(0, 1 << 32, b, dtype=np.uint64).astype(np.uint32)
        val[::5] = 0
        oracle.score_update(score, idx, val)
        T.selector_update(s, dev(idx), dev(val.view(np.int32)))
        got_scores, total = T.selector_scores(s)
        assert np.array_equal(got_scores.cpu().numpy().view(np.uint32), score)
        assert total == int(score.astype(np.uint64).sum())
    T.selector_free(s)


def test_selector_uniform_start_and_all_zero():
    s = T.selector_init(n=5000, initial_score=6554)
    want = oracle.batch_draw(np.full(5000, 6554, np.uint32), 600, seed=1, iteration=0)
    assert np.array_equal(T.selector_draw(s, 600, 1, 0).cpu().numpy(), want)
    every = torch.arange(5000, dtype=torch.int32, device="cuda")
    T.selector_update(s, every, torch.zeros(5000, dtype=torch.int32, device="cuda"))
    assert T.selector_draw(s, 10, 1, 1).tolist() == [-1] * 10
    assert T.selector_scores(s)[1] == 0
    one = torch.tensor([4321], dtype=torch.int32, device="cuda")
    T.selector_update(s, one, torch.tensor([-1], dtype=torch.int32, device="cuda"))     # 2^32 - 1
    assert T.selector_draw(s, 10, 1, 2).tolist() == [4321] * 10


# ----------------------------------------------------------------------------- HIP graph capture
def test_whole_step_replays_from_a_hip_graph():
    """Sampling, edge gather and cached node lookup of one step captured into a HIP graph and
    replayed with new roots written into the same input buffers, with eager work and
    synchronisations between the replays; every replay equals the oracle. (The per-call state of
    the library is kernels only: no memset nodes, no allocation once the buffers are warm.)"""
    w = W.make(1)
    g, g_ref = build_both(w.src, w.dst, w.ts, w.eid, w.num_nodes)
    rng = np.random.default_rng(3)
    node_np = rng.standard_normal((w.num_nodes, 12)).astype(np.float32)
    node_host = torch.from_numpy(node_np).pin_memory()
    cache = T.cache_init(node_host, 200, None, seed=5, staging_rows=256)
    table = dev(w.edge_feat)
    R, k = 600, 10
    roots_d = torch.empty(R, dtype=torch.int32, device="cuda")
    times_d = torch.empty(R, dtype=torch.int64, device="cuda")
    hit_miss = torch.zeros(2, dtype=torch.int64, device="cuda")

    def step(out=None, edge_out=None, node_out=None):
        out = T.sample_temporal(g, roots_d, times_d, k, 2, T.UNIFORM, 77, out=out)
        edge_out = T.gather_features(table, out[1]["eid"].reshape(-1), out=edge_out)
        node_out = T.cache_lookup(cache, out[1]["nbr"].reshape(-1), out=node_out, hit_miss=hit_miss)
        return out, edge_out, node_out

    roots, times = w.batches[5]
    roots_d.copy_(torch.from_numpy(roots))
    times_d.copy_(torch.from_numpy(times))
    bufs = step()                                                     # warm-up: every buffer exists afterwards
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step(*bufs)
    torch.cuda.current_stream().wait_stream(side)
    out, edge_out, node_out = bufs
    for b in (9, 0, 7, 3):
        roots, times = w.batches[b]
        roots_d.copy_(torch.from_numpy(roots))                        # eager work between the replays
        times_d.copy_(torch.from_numpy(times))
        hit_miss.zero_()
        graph.replay()
        torch.cuda.synchronize()
        want = oracle.sample_temporal(g_ref, roots, times, k, 2, W.UNIFORM, 77, threads=THREADS)
        assert_hops_equal(out, want)
        assert edge_out.cpu().numpy().tobytes() == oracle.gather(w.edge_feat, want[1]["eid"].ravel()).tobytes()
        ids = want[1]["nbr"].ravel()
        assert node_out.cpu().numpy().tobytes() == oracle.gather(node_np, ids).tobytes()
        assert tuple(hit_miss.tolist()) == oracle.cache_hits(T.cache_residents(cache).numpy(), w.num_nodes, ids)


def test_sampling_with_rows_into_one_buffer_for_all_hops():
    """Edge ids and rows of all hops as consecutive views of one buffer each (the benchmark's layout):
    for rows too long for the hop kernels the call then launches one gather for all hops."""
    w = W.make(3, num_batches=1)
    g, g_ref = build_both(w.src, w.dst, w.ts, w.eid, w.num_nodes)
    table = dev(w.edge_feat)
    roots, times = w.batches[0]
    roots, times = roots[:1501], times[:1501]
    k, hops, d = w.k, 3, w.edge_feat.shape[1]
    n_slots = [roots.shape[0] * k ** (h + 1) for h in range(hops)]
    eids = torch.full((sum(n_slots),), -7, dtype=torch.int32, device="cuda")
    rows = torch.full((sum(n_slots) + 3, d), 5.0, dtype=table.dtype, device="cuda")
    out, views, at, r = [], [], 0, roots.shape[0]
    for h in range(hops):
        out.append(dict(nbr=torch.empty(n_slots[h], dtype=torch.int32, device="cuda"), eid=eids[at:at + n_slots[h]],
                        ts=torch.empty(n_slots[h], dtype=torch.int64, device="cuda"), count=torch.empty(r, dtype=torch.int32, device="cuda")))
        views.append(rows[at:at + n_slots[h]])
        at += n_slots[h]
        r *= k
    T.sample_temporal_rows(g, dev(roots), dev(times), k, hops, T.UNIFORM, 11, table, out=out, rows_out=views)
    torch.cuda.synchronize()
    want = oracle.sample_temporal(g_ref, roots, times, k, hops, W.UNIFORM, 11, threads=THREADS)
    all_eids = np.concatenate([o["eid"].ravel() for o in want])
    assert np.array_equal(eids.cpu().numpy(), all_eids)
    got = rows.cpu().numpy()
    assert got[:sum(n_slots)].tobytes() == oracle.gather(w.edge_feat, all_eids, threads=THREADS).tobytes()
    assert (got[sum(n_slots):] == 5.0).all()


def test_finder_with_rows_replays_from_a_hip_graph():
    """taser_sample_temporal_rows (hop kernels writing the rows: C1 has 64-byte edge rows) captured
    into a HIP graph and replayed with new roots in the same buffers; every replay equals the oracle."""
    w = W.make(1)
    g, g_ref = build_both(w.src, w.dst, w.ts, w.eid, w.num_nodes)
    table = dev(w.edge_feat)
    R, k = 600, 10
    roots_d = torch.empty(R, dtype=torch.int32, device="cuda")
    times_d = torch.empty(R, dtype=torch.int64, device="cuda")
    roots, times = w.batches[2]
    roots_d.copy_(torch.from_numpy(roots))
    times_d.copy_(torch.from_numpy(times))
    out, rows = T.sample_temporal_rows(g, roots_d, times_d, k, 2, T.UNIFORM, 77, table)      # warm-up and buffers
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            T.sample_temporal_rows(g, roots_d, times_d, k, 2, T.UNIFORM, 77, table, out=out, rows_out=rows)
    torch.cuda.current_stream().wait_stream(side)
    for b in (8, 0, 5):
        roots, times = w.batches[b]
        roots_d.copy_(torch.from_numpy(roots))                        # eager work between the replays
        times_d.copy_(torch.from_numpy(times))
        for r in rows:
            r.fill_(9.0)
        graph.replay()
        torch.cuda.synchronize()
        want = oracle.sample_temporal(g_ref, roots, times, k, 2, W.UNIFORM, 77, threads=THREADS)
        assert_hops_equal(out, want)
        for h in range(2):
            assert rows[h].cpu().numpy().tobytes() == oracle.gather(w.edge_feat, want[h]["eid"].ravel()).tobytes()


def test_two_stream_step_replays_from_a_hip_graph():
    """The same step with the lookup split over two streams, as the benchmark's pipelined schedule
    issues it: the classification and the staging of missed rows on a side stream that is forked
    from and joined to the capturing stream by events inside the capture, beside the edge gather;
    the node gather after the join. Replayed with new roots; every replay equals the oracle."""
    w = W.make(1)
    g, g_ref = build_both(w.src, w.dst, w.ts, w.eid, w.num_nodes)
    rng = np.random.default_rng(4)
    node_np = rng.standard_normal((w.num_nodes, 413)).astype(np.float32)
    node_host = torch.from_numpy(node_np).pin_memory()
    cache = T.cache_init(node_host, 200, None, seed=6, staging_rows=800)
    T.cache_tune(cache, stage_blocks=8, refresh_before_gather=True)
    table = dev(w.edge_feat)
    R, k = 600, 10
    roots_d = torch.empty(R, dtype=torch.int32, device="cuda")
    times_d = torch.empty(R, dtype=torch.int64, device="cuda")
    hit_miss = torch.zeros(2, dtype=torch.int64, device="cuda")
    ids = torch.empty(R + R * k + R * k * k, dtype=torch.int32, device="cuda")      # roots | hop-1 nodes | hop-2 nodes
    out = [dict(nbr=ids[R:R + R * k], eid=torch.empty(R * k, dtype=torch.int32, device="cuda"),
                ts=torch.empty(R * k, dtype=torch.int64, device="cuda"), count=torch.empty(R, dtype=torch.int32, device="cuda")),
           dict(nbr=ids[R + R * k:], eid=torch.empty(R * k * k, dtype=torch.int32, device="cuda"),
                ts=torch.empty(R * k * k, dtype=torch.int64, device="cuda"), count=torch.empty(R * k, dtype=torch.int32, device="cuda"))]
    edge_out = torch.empty((R * k * k, w.edge_feat.shape[1]), dtype=torch.float32, device="cuda")
    node_out = torch.empty((ids.numel(), 413), dtype=torch.float32, device="cuda")
    side = torch.cuda.Stream()
    forked, joined = torch.cuda.Event(), torch.cuda.Event()

    def step(main):
        ids[:R].copy_(roots_d)
        T.sample_temporal(g, roots_d, times_d, k, 2, T.RECENT, 11, out=out, stream=main)
        forked.record(main)
        side.wait_event(forked)
        T.cache_prefetch(cache, ids, hit_miss=hit_miss, stream=side)
        joined.record(side)
        T.gather_features(table, out[1]["eid"], out=edge_out, stream=main)
        main.wait_event(joined)
        T.cache_gather(cache, ids, out=node_out, stream=main)

    roots, times = w.batches[2]
    roots_d.copy_(torch.from_numpy(roots))
    times_d.copy_(torch.from_numpy(times))
    step(torch.cuda.current_stream())                                 # warm-up: the handle's scratch has its final size
    torch.cuda.synchronize()
    capture = torch.cuda.Stream()
    capture.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(capture):
        with torch.cuda.graph(graph, stream=capture):
            step(capture)
    torch.cuda.current_stream().wait_stream(capture)
    for b in (8, 1, 6):
        roots, times = w.batches[b]
        roots_d.copy_(torch.from_numpy(roots))                        # eager work between the replays
        times_d.copy_(torch.from_numpy(times))
        hit_miss.zero_()
        graph.replay()
        torch.cuda.synchronize()
        want = oracle.sample_temporal(g_ref, roots, times, k, 2, W.RECENT, 11, threads=THREADS)
        for h in range(2):
            for f in FIELDS:
                assert np.array_equal(out[h][f].cpu().numpy().reshape(want[h][f].shape), want[h][f]), (b, h, f)
        assert edge_out.cpu().numpy().tobytes() == oracle.gather(w.edge_feat, want[1]["eid"].ravel()).tobytes()
        ids_np = np.concatenate([roots, want[0]["nbr"].ravel(), want[1]["nbr"].ravel()])
        assert node_out.cpu().numpy().tobytes() == oracle.gather(node_np, ids_np).tobytes()
        assert tuple(hit_miss.tolist()) == oracle.cache_hits(T.cache_residents(cache).numpy(), w.num_nodes, ids_np)
