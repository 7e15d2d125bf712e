"""Pins for the CPU oracle: everything it computes is checked against something
other than itself — published known-answer vectors, numpy library routines,
pure-Python brute force from the raw event list, closed-form probabilities.
No GPU needed."""
import itertools
import os

import numpy as np
import pytest
from scipy import stats

import oracle

MASK64 = (1 << 64) - 1


# --------------------------------------------------------------------------- RNG
def test_philox_known_answers(golden_dir):
    """Published known-answer vectors of Philox4x32-10 (Salmon et al., SC'11)."""
    rows = [l.split() for l in open(os.path.join(golden_dir, "philox4x32_10_kat.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        v = [int(x, 16) for x in r]
        out = oracle.philox4x32_10(v[0:4], v[4:6])
        assert [int(x) for x in out] == v[6:10]


def test_draw64_counter_layout():
    """key = seed halves, counter = (root lo, root hi, slot, hop), result = word1:word0."""
    for seed, hop, root, slot in [(42, 0, 0, 0), (0xDEADBEEFCAFEF00D, 1, (1 << 33) + 7, 9),
                                  (1, 3, 599999, 31)]:
        out = oracle.philox4x32_10([root & 0xFFFFFFFF, root >> 32, slot, hop],
                                   [seed & 0xFFFFFFFF, seed >> 32])
        assert oracle.draw64(seed, hop, root, slot) == (int(out[1]) << 32) | int(out[0])


def test_mulhi64_against_bigints():
    rng = np.random.default_rng(0)
    cases = [(0, 5), (MASK64, 1), (MASK64, MASK64), (1 << 63, 3), (12345, 0)]
    cases += [(int(a), int(b)) for a, b in rng.integers(0, 1 << 63, (200, 2), dtype=np.uint64)]
    cases += [(int(a) * 2 + 1, int(b)) for a, b in rng.integers(0, 1 << 63, (200, 2), dtype=np.uint64)]
    for u, n in cases:
        assert oracle.mulhi64(u, n) == (u * n) >> 64


def test_draw64_bits_equidistributed():
    """Low and high bytes of the draws are uniform (chi-square, fixed seed)."""
    d = np.array([oracle.draw64(7, 0, r, 0) for r in range(40000)], dtype=np.uint64)
    for shift in (0, 24, 56):
        obs = np.bincount(((d >> np.uint64(shift)) & np.uint64(255)).astype(np.int64), minlength=256)
        chi = ((obs - 40000 / 256) ** 2 / (40000 / 256)).sum()
        assert chi < stats.chi2.ppf(1 - 1e-4, 255)


# --------------------------------------------------------------------------- T-CSR
def _random_events(rng, n_nodes, n, t_span, sorted_ts):
    src = rng.integers(0, n_nodes, n).astype(np.int32)
    dst = rng.integers(0, n_nodes, n).astype(np.int32)
    ts = rng.integers(0, t_span, n).astype(np.int64)
    if sorted_ts:
        ts.sort()
    eid = rng.permutation(n).astype(np.int32)
    return src, dst, ts, eid


@pytest.mark.parametrize("sorted_ts", [True, False])
@pytest.mark.parametrize("threads", [1, 4])
def test_tcsr_equals_lexsort(sorted_ts, threads):
    """Per-node lists sorted by timestamp (Sec. 3.3), ties by input position:
    the same thing as numpy.lexsort with keys (src, ts, position)."""
    rng = np.random.default_rng(11)
    n_nodes, n = 37, 5000
    src, dst, ts, eid = _random_events(rng, n_nodes, n, 300, sorted_ts)   # heavy ties
    src[src == 5] = 6                                                     # an empty node
    indptr, o_nbr, o_ts, o_eid = oracle.tcsr_build(src, dst, ts, eid, n_nodes, threads)
    perm = np.lexsort((np.arange(n), ts, src))
    assert np.array_equal(o_nbr, dst[perm])
    assert np.array_equal(o_ts, ts[perm])
    assert np.array_equal(o_eid, eid[perm])
    assert np.array_equal(indptr, np.concatenate([[0], np.cumsum(np.bincount(src, minlength=n_nodes))]))
    assert indptr[5] == indptr[6] and indptr[-1] == n
    for v in range(n_nodes):
        seg = o_ts[indptr[v]:indptr[v + 1]]
        assert np.all(np.diff(seg) >= 0)
        got = sorted(zip(o_nbr[indptr[v]:indptr[v + 1]], seg, o_eid[indptr[v]:indptr[v + 1]]))
        want = sorted(zip(dst[src == v], ts[src == v], eid[src == v]))
        assert got == want


def test_tcsr_rejects_bad_node():
    with pytest.raises(ValueError):
        oracle.tcsr_build([0, 3], [1, 1], [0, 1], [0, 1], 3)


# --------------------------------------------------------------------------- cutoff + most recent
def _brute_force_neighborhood(src, dst, ts, eid, v, t):
    """N(v,t) = {(u,t_u) : (v,u,t_u) in E, t_u < t} (Sec. 2.1) straight from the raw
    event list, latest first, ties by later input position first."""
    cand = [(int(ts[i]), i) for i in range(len(src)) if src[i] == v and ts[i] < t]
    cand.sort(reverse=True)
    return [(int(dst[i]), int(eid[i]), tt) for tt, i in cand]


def _check_padding(o, q, c, k):
    assert o["count"][q] == c
    assert np.all(o["nbr"][q, c:] == -1) and np.all(o["eid"][q, c:] == -1) and np.all(o["ts"][q, c:] == 0)


@pytest.mark.parametrize("sorted_ts", [True, False])
def test_most_recent_equals_brute_force(sorted_ts):
    rng = np.random.default_rng(5)
    n_nodes, n, k = 12, 600, 7
    src, dst, ts, eid = _random_events(rng, n_nodes, n, 80, sorted_ts)
    src[src == 3] = 4
    g = oracle.tcsr_build(src, dst, ts, eid, n_nodes)
    roots = rng.integers(0, n_nodes, 300).astype(np.int32)
    times = rng.integers(-2, 85, 300).astype(np.int64)
    o = oracle.sample_temporal(g, roots, times, k, 1, oracle.RECENT, seed=1)[0]
    for q in range(300):
        want = _brute_force_neighborhood(src, dst, ts, eid, roots[q], times[q])[:k]
        c = len(want)
        _check_padding(o, q, c, k)
        got = list(zip(o["nbr"][q, :c].tolist(), o["eid"][q, :c].tolist(), o["ts"][q, :c].tolist()))
        assert got == want


def test_cutoff_equals_searchsorted_and_edge_cases():
    """count (with k above every degree) is numpy.searchsorted(side='left') on the
    node's time-sorted list: strict '<' (Sec. 2.1)."""
    rng = np.random.default_rng(9)
    n_nodes, n = 9, 2000
    src, dst, ts, eid = _random_events(rng, n_nodes, n, 50, True)
    src[src == 2] = 1
    ts[src == 7] = 20                                  # a node whose timestamps are all equal
    g = oracle.tcsr_build(src, dst, ts, eid, n_nodes)
    indptr, _, gts, _ = g
    k = int(np.diff(indptr).max()) + 1
    roots = np.repeat(np.arange(n_nodes, dtype=np.int32), 56)
    times = np.tile(np.arange(-3, 53, dtype=np.int64), n_nodes)
    o = oracle.sample_temporal(g, roots, times, k, 1, oracle.RECENT, seed=0)[0]
    for q in range(roots.shape[0]):
        seg = gts[indptr[roots[q]]:indptr[roots[q] + 1]]
        assert o["count"][q] == np.searchsorted(seg, times[q], side="left")
        assert np.all(o["ts"][q, :o["count"][q]] < times[q])
    sel = roots == 2
    assert np.all(o["count"][sel] == 0)                # empty list
    sel7 = roots == 7
    deg7 = indptr[8] - indptr[7]
    assert np.all(o["count"][sel7 & (times <= 20)] == 0)      # a tie with t is excluded
    assert np.all(o["count"][sel7 & (times > 20)] == deg7)


def test_most_recent_invariant_under_root_order():
    """Arbitrary (non-chronological) root order must work (Sec. 1, 4.3)."""
    rng = np.random.default_rng(2)
    src, dst, ts, eid = _random_events(rng, 20, 1500, 1000, True)
    g = oracle.tcsr_build(src, dst, ts, eid, 20)
    roots = rng.integers(0, 20, 200).astype(np.int32)
    times = rng.integers(0, 1000, 200).astype(np.int64)
    a = oracle.sample_temporal(g, roots, times, 5, 1, oracle.RECENT, seed=0)[0]
    p = rng.permutation(200)
    b = oracle.sample_temporal(g, roots[p], times[p], 5, 1, oracle.RECENT, seed=0)[0]
    for name in ("nbr", "eid", "ts", "count"):
        assert np.array_equal(a[name][p], b[name])


# --------------------------------------------------------------------------- uniform
def _single_node_graph(cnt, extra_after=3):
    """One node (id 0) with `cnt` entries before t = 10**6 and a few after it.
    Entry p has neighbor id p, edge id 1000 + p, timestamp 10 * p."""
    n = cnt + extra_after
    src = np.zeros(n, np.int32)
    dst = np.arange(n, dtype=np.int32)
    ts = np.arange(n, dtype=np.int64) * 10
    ts[cnt:] += 10 ** 6
    eid = (1000 + np.arange(n)).astype(np.int32)
    return oracle.tcsr_build(src, dst, ts, eid, 1), 10 ** 6


def _fisher_yates_positions(seed, hop, q, cnt, k):
    """Partial Fisher-Yates on an explicit array, Python integers only."""
    a = list(range(cnt))
    out = []
    for j in range(k):
        r = j + ((oracle.draw64(seed, hop, q, j) * (cnt - j)) >> 64)
        a[j], a[r] = a[r], a[j]
        out.append(a[j])
    return out


@pytest.mark.parametrize("cnt,k", [(11, 10), (12, 3), (64, 10), (1000, 10), (33, 32)])
def test_uniform_equals_explicit_fisher_yates(cnt, k):
    g, t = _single_node_graph(cnt)
    R = 400
    o = oracle.sample_hop(g, np.zeros(R, np.int32), np.full(R, t, np.int64), k, oracle.UNIFORM,
                          seed=99, hop=1)
    for q in range(R):
        pos = _fisher_yates_positions(99, 1, q, cnt, k)
        assert o["nbr"][q].tolist() == pos                      # neighbor id == position
        assert o["eid"][q].tolist() == [1000 + p for p in pos]
        assert o["ts"][q].tolist() == [10 * p for p in pos]
        assert len(set(pos)) == k and max(pos) < cnt            # distinct, strictly before t
        assert o["count"][q] == k


def test_uniform_small_neighborhood_returns_all_most_recent_first():
    for cnt in (0, 1, 4, 10):
        g, t = _single_node_graph(cnt)
        u = oracle.sample_hop(g, np.zeros(5, np.int32), np.full(5, t, np.int64), 10, oracle.UNIFORM, 3, 0)
        r = oracle.sample_hop(g, np.zeros(5, np.int32), np.full(5, t, np.int64), 10, oracle.RECENT, 3, 0)
        for name in ("nbr", "eid", "ts", "count"):
            assert np.array_equal(u[name], r[name])
        assert np.all(u["count"] == cnt)


def test_uniform_ordered_pairs_equiprobable():
    """cnt = 5, k = 2: the 20 ordered pairs are equiprobable (exact multinomial)."""
    g, t = _single_node_graph(5)
    R = 100000
    o = oracle.sample_hop(g, np.zeros(R, np.int32), np.full(R, t, np.int64), 2, oracle.UNIFORM, 2024, 0,
                          threads=4)
    code = o["nbr"][:, 0] * 5 + o["nbr"][:, 1]
    obs = np.bincount(code, minlength=25)
    pairs = [a * 5 + b for a in range(5) for b in range(5) if a != b]
    assert obs.sum() == obs[pairs].sum()
    chi = ((obs[pairs] - R / 20) ** 2 / (R / 20)).sum()
    assert chi < stats.chi2.ppf(1 - 1e-4, 19)


@pytest.mark.parametrize("cnt", [11, 64, 1000])
def test_uniform_slot_marginals(cnt):
    """Each slot's marginal is uniform over the cnt valid positions."""
    g, t = _single_node_graph(cnt)
    R = 60000
    o = oracle.sample_hop(g, np.zeros(R, np.int32), np.full(R, t, np.int64), 10, oracle.UNIFORM, 5, 1,
                          threads=4)
    for slot in (0, 4, 9):
        obs = np.bincount(o["nbr"][:, slot], minlength=cnt)
        assert obs.shape[0] == cnt
        chi = ((obs - R / cnt) ** 2 / (R / cnt)).sum()
        assert chi < stats.chi2.ppf(1 - 1e-4, cnt - 1)


# --------------------------------------------------------------------------- weighted
def _weighted_graph(weights_recent_first, extra_older=0):
    """One node whose candidate i (most recent first) carries weights_recent_first[i]."""
    c = len(weights_recent_first)
    cnt = c + extra_older
    g, t = _single_node_graph(cnt)
    ew = np.ones(1000 + cnt + 3, np.uint32)
    for i, w in enumerate(weights_recent_first):
        ew[1000 + (cnt - 1 - i)] = w                    # candidate i = entry cnt-1-i
    return g, t, ew, cnt


def _successive_probs(w, k):
    """Closed form for successive sampling without replacement:
    P(i1,..,ik) = prod_j w_ij / (W - sum of earlier picks)."""
    out = {}
    for seq in itertools.permutations(range(len(w)), k):
        p, rest = 1.0, float(sum(w))
        for i in seq:
            p *= w[i] / rest
            rest -= w[i]
        out[seq] = p
    return out


def test_weighted_equals_stepwise_python():
    w = [5, 1, 9, 2, 2, 7, 1, 30, 4, 4, 6, 3]
    g, t, ew, cnt = _weighted_graph(w, extra_older=20)
    R, k, m = 300, 4, len(w)
    o = oracle.sample_hop(g, np.zeros(R, np.int32), np.full(R, t, np.int64), k, oracle.WEIGHTED, 8, 1,
                          m=m, edge_weight=ew)
    for q in range(R):
        rem = list(w)
        for j in range(k):
            x = (oracle.draw64(8, 1, q, j) * sum(rem)) >> 64
            acc, pick = 0, None
            for i, wi in enumerate(rem):
                acc += wi
                if acc > x:
                    pick = i
                    break
            rem[pick] = 0
            assert o["nbr"][q, j] == cnt - 1 - pick      # neighbor id == entry position
        assert o["count"][q] == k


def test_weighted_ordered_pairs_closed_form():
    w = [1, 2, 3, 4, 10]
    g, t, ew, cnt = _weighted_graph(w)
    R = 120000
    o = oracle.sample_hop(g, np.zeros(R, np.int32), np.full(R, t, np.int64), 2, oracle.WEIGHTED, 77, 0,
                          m=5, edge_weight=ew, threads=4)
    cand = cnt - 1 - o["nbr"]                            # back to candidate indices
    probs = _successive_probs(w, 2)
    obs = np.array([np.sum((cand[:, 0] == a) & (cand[:, 1] == b)) for (a, b) in probs])
    exp = np.array(list(probs.values())) * R
    assert obs.sum() == R
    assert (((obs - exp) ** 2) / exp).sum() < stats.chi2.ppf(1 - 1e-4, len(exp) - 1)


def test_weighted_slot0_marginal_m25_and_window():
    """Slot 0 is drawn with probability w_i / W over the m = 25 most recent candidates;
    older entries are never candidates."""
    rng = np.random.default_rng(3)
    w = [int(x) for x in np.clip(np.rint(np.exp(rng.standard_normal(25)) * 4096), 1, 65536)]
    g, t, ew, cnt = _weighted_graph(w, extra_older=40)
    R = 100000
    o = oracle.sample_hop(g, np.zeros(R, np.int32), np.full(R, t, np.int64), 10, oracle.WEIGHTED, 4, 0,
                          m=25, edge_weight=ew, threads=4)
    cand = cnt - 1 - o["nbr"]
    assert cand.min() >= 0 and cand.max() < 25
    assert all(len(set(row)) == 10 for row in cand[:2000].tolist())
    obs = np.bincount(cand[:, 0], minlength=25)
    exp = np.array(w) / sum(w) * R
    assert (((obs - exp) ** 2) / exp).sum() < stats.chi2.ppf(1 - 1e-4, 24)


def test_weighted_equal_weights_is_uniform_and_dominant_weight():
    g, t, ew, cnt = _weighted_graph([7] * 5)
    R = 100000
    o = oracle.sample_hop(g, np.zeros(R, np.int32), np.full(R, t, np.int64), 2, oracle.WEIGHTED, 12, 0,
                          m=5, edge_weight=ew, threads=4)
    cand = cnt - 1 - o["nbr"]
    code = cand[:, 0] * 5 + cand[:, 1]
    pairs = [a * 5 + b for a in range(5) for b in range(5) if a != b]
    obs = np.bincount(code, minlength=25)[pairs]
    assert obs.sum() == R
    assert (((obs - R / 20) ** 2) / (R / 20)).sum() < stats.chi2.ppf(1 - 1e-4, 19)
    w = [1, 1, 60000, 1, 1, 1]
    g, t, ew, cnt = _weighted_graph(w)
    o = oracle.sample_hop(g, np.zeros(R, np.int32), np.full(R, t, np.int64), 2, oracle.WEIGHTED, 13, 0,
                          m=6, edge_weight=ew, threads=4)
    first = cnt - 1 - o["nbr"][:, 0]
    p = 60000 / 60005
    assert abs((first == 2).mean() - p) < 5 * np.sqrt(p * (1 - p) / R)


def test_weighted_inclusion_probabilities_by_enumeration():
    """m = 6, k = 3 (and c = k + 1): inclusion probabilities from enumerating every
    ordered outcome of successive sampling."""
    for w, k in (([3, 1, 4, 1, 5, 9], 3), ([2, 7, 1, 8], 3)):
        g, t, ew, cnt = _weighted_graph(w)
        R = 100000
        o = oracle.sample_hop(g, np.zeros(R, np.int32), np.full(R, t, np.int64), k, oracle.WEIGHTED, 31, 1,
                              m=len(w), edge_weight=ew, threads=4)
        cand = cnt - 1 - o["nbr"]
        probs = _successive_probs(w, k)
        for i in range(len(w)):
            p = sum(pr for seq, pr in probs.items() if i in seq)
            f = np.any(cand == i, axis=1).mean()
            assert abs(f - p) < 5 * np.sqrt(p * (1 - p) / R) + 1e-9


def test_weighted_few_candidates_returns_all_in_candidate_order():
    g, t, ew, cnt = _weighted_graph([9, 1, 5])
    o = oracle.sample_hop(g, np.zeros(3, np.int32), np.full(3, t, np.int64), 4, oracle.WEIGHTED, 1, 0,
                          m=25, edge_weight=ew)
    assert np.all(o["count"] == 3)
    assert np.all(o["nbr"][:, :3] == np.array([2, 1, 0])) and np.all(o["nbr"][:, 3] == -1)


# --------------------------------------------------------------------------- two hops
@pytest.mark.parametrize("policy", [oracle.RECENT, oracle.UNIFORM, oracle.WEIGHTED])
def test_two_hop_composition(policy):
    """Hop 2 of slot q is a 1-hop query on (nbr1[q], ts1[q]) (Alg. 1 layer loop), so every
    second-hop sample is strictly earlier than the first-hop interaction it hangs off."""
    rng = np.random.default_rng(21)
    src, dst, ts, eid = _random_events(rng, 30, 4000, 5000, True)
    src, dst = np.concatenate([src, dst]), np.concatenate([dst, src])
    ts, eid = np.concatenate([ts, ts]), np.concatenate([eid, eid])
    g = oracle.tcsr_build(src, dst, ts, eid, 30)
    ew = rng.integers(1, 1 << 16, 4000).astype(np.uint32)
    roots = rng.integers(0, 30, 64).astype(np.int32)
    times = rng.integers(0, 5000, 64).astype(np.int64)
    k = 4
    h = oracle.sample_temporal(g, roots, times, k, 2, policy, seed=6, m=9, edge_weight=ew)
    assert h[1]["nbr"].shape == (64 * k, k)
    one = oracle.sample_hop(g, h[0]["nbr"].ravel(), h[0]["ts"].ravel(), k, policy, 6, 1, m=9, edge_weight=ew)
    for name in ("nbr", "eid", "ts", "count"):
        assert np.array_equal(h[1][name], one[name])
    flat_valid = h[0]["nbr"].ravel() >= 0
    assert np.all(h[1]["count"][~flat_valid] == 0)
    parent_t = h[0]["ts"].ravel()[:, None]
    valid2 = h[1]["nbr"] >= 0
    assert np.all((h[1]["ts"] < parent_t)[valid2])
    # every sampled (root, nbr, eid, ts) is an entry of the event list
    events = set(zip(src.tolist(), dst.tolist(), eid.tolist(), ts.tolist()))
    r1 = np.repeat(h[0]["nbr"].ravel(), k).reshape(-1, k)
    for a, b, c, d in zip(r1[valid2], h[1]["nbr"][valid2], h[1]["eid"][valid2], h[1]["ts"][valid2]):
        assert (int(a), int(b), int(c), int(d)) in events


# --------------------------------------------------------------------------- gather + cache
@pytest.mark.parametrize("dtype,dim,pad", [(np.float32, 16, 0), (np.float16, 172, 0), (np.float16, 186, 6),
                                           (np.float32, 413, 3)])
def test_gather_equals_numpy_take(dtype, dim, pad):
    rng = np.random.default_rng(8)
    rows = 500
    full = rng.standard_normal((rows, dim + pad)).astype(dtype)
    table = full[:, :dim]                                  # a padded row pitch
    ids = rng.integers(0, rows, 2000).astype(np.int32)
    ids[::7] = -1
    out = oracle.gather(table, ids, threads=3)
    want = np.take(table, np.maximum(ids, 0), axis=0)
    want[ids < 0] = 0
    assert out.tobytes() == want.tobytes()
    with pytest.raises(ValueError):
        oracle.gather(table, np.array([rows], np.int32))


def test_cache_residents_and_hit_accounting():
    rows, cap = 1000, 200
    res = oracle.cache_random_residents(rows, cap, seed=5)
    assert len(set(res.tolist())) == cap and res.min() >= 0 and res.max() < rows
    # the draw is the same partial Fisher-Yates as the uniform policy
    a = list(range(rows))
    for j in range(cap):
        r = j + ((oracle.draw64(5, 0x43414348, j, 0) * (rows - j)) >> 64)
        a[j], a[r] = a[r], a[j]
    assert res.tolist() == a[:cap]
    rng = np.random.default_rng(1)
    ids = rng.integers(-1, rows, 5000).astype(np.int32)
    hits, misses = oracle.cache_hits(res, rows, ids)
    assert hits == int(np.isin(ids, res).sum())
    assert hits + misses == int((ids >= 0).sum())
    # first-element marginal is uniform over the rows
    firsts = np.array([oracle.cache_random_residents(50, 1, seed=s)[0] for s in range(20000)])
    obs = np.bincount(firsts, minlength=50)
    assert (((obs - 400) ** 2) / 400).sum() < stats.chi2.ppf(1 - 1e-4, 49)


# --------------------------------------------------------------------------- cache maintenance (Alg. 3)
def test_cache_counting_equals_bincount():
    rng = np.random.default_rng(4)
    rows = 300
    ids = rng.integers(-2, rows + 3, 20000).astype(np.int32)
    Q = np.zeros(rows, np.uint32)
    oracle.cache_count(ids, rows, Q)
    oracle.cache_count(ids[:100], rows, Q)
    ok = (ids >= 0) & (ids < rows)
    want = np.bincount(ids[ok], minlength=rows) + np.bincount(ids[:100][ok[:100]], minlength=rows)
    assert np.array_equal(Q, want.astype(np.uint32))


def test_cache_epoch_end_is_topk_with_threshold():
    """Q_topk by numpy (stable argsort of -count: ties keep the smaller id), overlap by set
    intersection, replacement only below the threshold, Q cleared either way."""
    rng = np.random.default_rng(6)
    rows, cap = 500, 60
    for trial in range(20):
        Q = rng.integers(0, 8, rows).astype(np.uint32)            # heavy ties
        if trial == 0:
            Q[:] = 0                                                # nothing was requested
        resident = rng.permutation(rows)[:cap].astype(np.int32)
        topk = np.sort(np.argsort(-Q.astype(np.int64), kind="stable")[:cap])
        overlap = len(set(topk.tolist()) & set(resident.tolist()))
        for thr in (0, overlap, overlap + 1, cap):
            q = Q.copy()
            rep, ov, new = oracle.cache_epoch_end(q, resident, thr)
            assert ov == overlap and rep == (overlap < thr)
            assert np.array_equal(new, topk if rep else resident)
            assert not q.any()
        # brute force: every kept row is requested at least as often as every dropped row
        kept = np.zeros(rows, bool)
        kept[topk] = True
        assert Q[kept].min() >= Q[~kept].max()


def test_cache_policy_converges_on_a_stationary_stream():
    """With a stationary access distribution the previous epoch's top-k is close to the best
    possible content (Sec. 3.4, Fig. 3b): after one refresh the hit rate is within a few percent
    of the cache that knows the epoch's frequencies in advance, and it grows with the cache size."""
    rng = np.random.default_rng(8)
    rows, per_epoch = 2000, 100000
    p = 1.0 / np.arange(1, rows + 1)
    p /= p.sum()
    perm = rng.permutation(rows)
    rates = []
    for frac in (0.1, 0.2, 0.3):
        cap = int(frac * rows)
        resident = oracle.cache_random_residents(rows, cap, seed=3)
        Q = np.zeros(rows, np.uint32)
        hit_rate = []
        for epoch in range(3):
            ids = perm[rng.choice(rows, per_epoch, p=p)].astype(np.int32)
            h, m = oracle.cache_hits(resident, rows, ids)
            hit_rate.append(h / (h + m))
            best = np.sort(np.bincount(ids, minlength=rows))[::-1][:cap].sum() / per_epoch   # knows this epoch
            oracle.cache_count(ids, rows, Q)
            _, _, resident = oracle.cache_epoch_end(Q, resident, cap)                         # always below cap+...: refresh
            if epoch >= 1:
                assert best - hit_rate[-1] < 0.03
        assert hit_rate[1] > hit_rate[0] + 0.2
        rates.append(hit_rate[-1])
    assert rates[0] < rates[1] < rates[2]


# --------------------------------------------------------------------------- candidate-window products (Sec. 3.2)
def test_candidate_encodings_equal_numpy():
    """freq(u) = how often u appears among the valid candidates; IE = pairwise equality."""
    rng = np.random.default_rng(10)
    R, m = 200, 25
    nbr = rng.integers(0, 6, (R, m)).astype(np.int32)               # few distinct ids: many repeats
    count = rng.integers(0, m + 1, R).astype(np.int32)
    count[:3] = (0, 1, m)
    for i in range(R):
        nbr[i, count[i]:] = -1                                      # padding never matches anything
    freq, ident = oracle.candidate_encodings(nbr, count)
    valid = np.arange(m)[None, :] < count[:, None]
    eq = (nbr[:, :, None] == nbr[:, None, :]) & valid[:, :, None] & valid[:, None, :]
    assert np.array_equal(ident, eq.astype(np.uint8))
    assert np.array_equal(freq, eq.sum(axis=2).astype(np.int32))
    for i in (3, 50, 199):                                          # and through numpy.unique, independently
        ids, cnt = np.unique(nbr[i, :count[i]], return_counts=True)
        lut = dict(zip(ids.tolist(), cnt.tolist()))
        assert freq[i, :count[i]].tolist() == [lut[u] for u in nbr[i, :count[i]].tolist()]
        assert not freq[i, count[i]:].any()
    f2, none = oracle.candidate_encodings(nbr, count, want_identity=False)
    assert none is None and np.array_equal(f2, freq)


def test_select_weighted_replay_and_closed_form():
    """Per-slot weights: step-by-step replay in Python integers, the closed form of successive
    sampling (chi-square over ordered pairs), agreement with the per-edge-weight policy when the
    per-slot weights are those edge weights, and the keep-everything case."""
    rng = np.random.default_rng(12)
    R, m, k = 300, 9, 4
    weight = rng.integers(1, 1 << 16, (R, m)).astype(np.uint32)
    count = rng.integers(0, m + 1, R).astype(np.int32)
    sel, oc = oracle.select_weighted(weight, count, k, seed=5, hop=1)
    for i in range(R):
        c = int(count[i])
        if c <= k:
            assert sel[i].tolist() == list(range(c)) + [-1] * (k - c) and oc[i] == c
            continue
        rem = [int(x) for x in weight[i, :c]]
        for j in range(k):
            x = (oracle.draw64(5, 1, i, j) * sum(rem)) >> 64
            acc = 0
            for l, wl in enumerate(rem):
                acc += wl
                if acc > x:
                    break
            rem[l] = 0
            assert sel[i, j] == l
        assert oc[i] == k
    w = np.array([1, 2, 3, 4, 10], np.uint32)
    n = 120000
    sel, _ = oracle.select_weighted(np.tile(w, (n, 1)), np.full(n, 5, np.int32), 2, seed=77, hop=0)
    probs = _successive_probs([int(x) for x in w], 2)
    obs = np.array([np.sum((sel[:, 0] == a) & (sel[:, 1] == b)) for (a, b) in probs])
    exp = np.array(list(probs.values())) * n
    assert obs.sum() == n and (((obs - exp) ** 2) / exp).sum() < stats.chi2.ppf(1 - 1e-4, len(exp) - 1)
    # same draws as the per-edge-weight policy of the finder when the weights coincide
    src, dst, ts, eid = _random_events(rng, 15, 3000, 4000, True)
    g = oracle.tcsr_build(src, dst, ts, eid, 15)
    ew = rng.integers(1, 1 << 16, 3000).astype(np.uint32)
    roots = rng.integers(0, 15, 100).astype(np.int32)
    times = rng.integers(0, 4000, 100).astype(np.int64)
    cand = oracle.sample_hop(g, roots, times, 9, oracle.RECENT, 3, 0)
    kept = oracle.sample_hop(g, roots, times, 4, oracle.WEIGHTED, 3, 0, m=9, edge_weight=ew)
    sel, oc = oracle.select_weighted(ew[np.maximum(cand["eid"], 0)], cand["count"], 4, seed=3, hop=0)
    assert np.array_equal(oc, kept["count"])
    picked = np.where(sel >= 0, np.take_along_axis(cand["eid"], np.maximum(sel, 0), axis=1), -1)
    assert np.array_equal(picked, kept["eid"])


# --------------------------------------------------------------------------- inverse-timespan policy
def _timed_node(ts_list, t_after=3):
    """One node (id 0) whose entries have the given ascending timestamps (neighbor id =
    position), plus a few later entries that a query must not see."""
    ts = np.array(list(ts_list) + [max(ts_list) + 10 ** 9 + i for i in range(t_after)], np.int64)
    n = ts.shape[0]
    return oracle.tcsr_build(np.zeros(n, np.int32), np.arange(n, dtype=np.int32), ts,
                             (500 + np.arange(n)).astype(np.int32), 1)


def _inverse_weights(ts_list, t):
    return [max(1, (1 << 32) // (t - x)) for x in ts_list]           # Python big integers


def test_inverse_timespan_equals_stepwise_python():
    """Replay with Python integers: weights floor(2^32 / delta), running sums in list order,
    one draw per slot scaled to the remaining total."""
    rng = np.random.default_rng(8)
    ts_list = sorted(int(x) for x in rng.integers(0, 5000, 40))
    g, t = _timed_node(ts_list), 5003
    R, k = 300, 6
    o = oracle.sample_hop(g, np.zeros(R, np.int32), np.full(R, t, np.int64), k, oracle.INVERSE_TIMESPAN, 21, 2)
    w0 = _inverse_weights(ts_list, t)
    for q in range(R):
        rem = list(w0)
        for j in range(k):
            x = (oracle.draw64(21, 2, q, j) * sum(rem)) >> 64
            acc, pick = 0, None
            for p, wp in enumerate(rem):
                acc += wp
                if acc > x:
                    pick = p
                    break
            rem[pick] = 0
            assert o["nbr"][q, j] == pick and o["ts"][q, j] == ts_list[pick]
        assert o["count"][q] == k and len(set(o["nbr"][q].tolist())) == k


def test_inverse_timespan_probabilities_are_inverse_to_the_time_delta():
    """Slot 0 is drawn with probability (1/delta_p) / sum(1/delta): chi-square against the
    real-valued law the heuristic states (the integer weights deviate from it by < 2^-20
    relative here); ordered pairs against the successive-sampling closed form."""
    deltas = [1, 2, 3, 5, 8, 13, 100, 1000]
    t = 10 ** 6
    ts_list = sorted(t - d for d in deltas)                            # oldest first
    g = _timed_node(ts_list)
    R = 120000
    o = oracle.sample_hop(g, np.zeros(R, np.int32), np.full(R, t, np.int64), 2, oracle.INVERSE_TIMESPAN, 5, 0,
                          threads=4)
    inv = np.array([1.0 / (t - x) for x in ts_list])
    obs = np.bincount(o["nbr"][:, 0], minlength=len(deltas))
    exp = inv / inv.sum() * R
    assert (((obs - exp) ** 2) / exp).sum() < stats.chi2.ppf(1 - 1e-4, len(deltas) - 1)
    assert obs.argmax() == len(deltas) - 1                             # the most recent entry is the likeliest
    probs = _successive_probs(list(inv), 2)
    big = {s: p for s, p in probs.items() if p * R >= 5}
    obs2 = np.array([np.sum((o["nbr"][:, 0] == a) & (o["nbr"][:, 1] == b)) for (a, b) in big])
    exp2 = np.array(list(big.values())) * R
    assert (((obs2 - exp2) ** 2) / exp2).sum() < stats.chi2.ppf(1 - 1e-4, len(exp2))


def test_inverse_timespan_special_cases():
    """Equal deltas reduce to the uniform law; cnt <= k returns everything, most recent first;
    entries at or after t are never drawn; deltas beyond 2^32 still get weight 1 (never 0);
    extreme timestamps do not overflow."""
    t = 777
    g = _timed_node([700] * 5)                                          # five entries, same delta
    R = 100000
    o = oracle.sample_hop(g, np.zeros(R, np.int32), np.full(R, t, np.int64), 2, oracle.INVERSE_TIMESPAN, 3, 0,
                          threads=4)
    code = o["nbr"][:, 0] * 5 + o["nbr"][:, 1]
    pairs = [a * 5 + b for a in range(5) for b in range(5) if a != b]
    obs = np.bincount(code, minlength=25)[pairs]
    assert obs.sum() == R
    assert (((obs - R / 20) ** 2) / (R / 20)).sum() < stats.chi2.ppf(1 - 1e-4, 19)

    g = _timed_node([10, 20, 30])
    o = oracle.sample_hop(g, np.zeros(2, np.int32), np.array([31, 25], np.int64), 4, oracle.INVERSE_TIMESPAN, 1, 0)
    assert o["nbr"].tolist() == [[2, 1, 0, -1], [1, 0, -1, -1]] and o["count"].tolist() == [3, 2]

    far = -(1 << 62)
    ts_list = [far, far + 1, far + 2, 0, 1 << 40, (1 << 62) - 5]
    g = _timed_node(ts_list)
    tq = (1 << 62)                                                      # deltas up to 2^63
    w = _inverse_weights(ts_list, tq)
    assert w[:5] == [1, 1, 1, 1, 1] and w[5] == (1 << 32) // 5
    R = 20000
    o = oracle.sample_hop(g, np.zeros(R, np.int32), np.full(R, tq, np.int64), 3, oracle.INVERSE_TIMESPAN, 9, 0)
    assert (o["ts"] < tq).all() and o["nbr"].max() == 5 and o["nbr"].min() == 0
    first_old = (o["nbr"][:, 0] < 5).mean()
    p = 5 / (5 + w[5])
    assert abs(first_old - p) < 5 * np.sqrt(p / R) + 1e-4
    assert all(len(set(r)) == 3 for r in o["nbr"].tolist())


def test_inverse_timespan_two_hops_respect_time():
    rng = np.random.default_rng(2)
    n, nodes = 6000, 30
    src = rng.integers(0, nodes, n).astype(np.int32)
    dst = rng.integers(0, nodes, n).astype(np.int32)
    ts = np.sort(rng.integers(0, 10000, n)).astype(np.int64)
    g = oracle.tcsr_build(src, dst, ts, np.arange(n, dtype=np.int32), nodes)
    roots = rng.integers(0, nodes, 200).astype(np.int32)
    times = rng.integers(0, 10000, 200).astype(np.int64)
    h = oracle.sample_temporal(g, roots, times, 5, 2, oracle.INVERSE_TIMESPAN, seed=4)
    one = oracle.sample_hop(g, h[0]["nbr"].ravel(), h[0]["ts"].ravel(), 5, oracle.INVERSE_TIMESPAN, 4, 1)
    for f in ("nbr", "eid", "ts", "count"):
        assert np.array_equal(h[1][f], one[f])
    valid = h[0]["eid"] >= 0
    assert (h[0]["ts"][valid] < np.repeat(times, 5).reshape(-1, 5)[valid]).all()
    assert np.array_equal(src[h[0]["eid"][valid]], np.repeat(roots, 5).reshape(-1, 5)[valid])
    v2 = h[1]["eid"] >= 0
    assert (h[1]["ts"][v2] < np.repeat(h[0]["ts"].ravel(), 5).reshape(-1, 5)[v2]).all()


# --------------------------------------------------------------------------- adaptive mini-batch selection
def test_batch_draw_equals_numpy_inverse_cdf():
    """Draw j = first index whose cumulative score exceeds floor(draw * W / 2^64):
    numpy.cumsum + searchsorted(side='right') with the scaling done in Python integers."""
    rng = np.random.default_rng(6)
    for n, b in ((1, 5), (7, 50), (5000, 600), (100000, 64)):
        score = rng.integers(0, 1 << 17, n).astype(np.uint32)
        score[rng.integers(0, n, n // 3)] = 0
        if n == 1:
            score[:] = 9
        cum = np.cumsum(score.astype(np.uint64))
        W = int(cum[-1])
        got = oracle.batch_draw(score, b, seed=31, iteration=12)
        xs = np.array([(oracle.draw64(31, 0x4253454C, 12, j) * W) >> 64 for j in range(b)], np.uint64)
        assert np.array_equal(got, np.searchsorted(cum, xs, side="right").astype(np.int32))
        assert (score[got] > 0).all()                                  # a zero score is never drawn
        again = oracle.batch_draw(score, b, seed=31, iteration=13)
        assert n == 1 or not np.array_equal(got, again)                # the iteration number matters
    assert oracle.batch_draw(np.zeros(4, np.uint32), 3, 1, 0).tolist() == [-1, -1, -1]
    big = np.full(3, 0xFFFFFFFF, np.uint32)                            # sums beyond 32 bits
    got = oracle.batch_draw(big, 3000, 2, 0)
    assert np.bincount(got, minlength=3).min() > 900


def test_batch_draw_probability_is_proportional_to_the_score():
    rng = np.random.default_rng(10)
    score = np.clip(np.rint((1 / (1 + np.exp(-rng.standard_normal(40))) + 0.1) * 65536), 1, None).astype(np.uint32)
    b = 200000
    got = oracle.batch_draw(score, b, seed=3, iteration=0)
    obs = np.bincount(got, minlength=40)
    exp = score / score.sum() * b
    assert (((obs - exp) ** 2) / exp).sum() < stats.chi2.ppf(1 - 1e-4, 39)
    uniform = np.full(25, 6554, np.uint32)                             # "initialised uniformly"
    obs = np.bincount(oracle.batch_draw(uniform, b, seed=4, iteration=1), minlength=25)
    assert (((obs - b / 25) ** 2) / (b / 25)).sum() < stats.chi2.ppf(1 - 1e-4, 24)


def test_score_update_is_the_sequential_loop():
    rng = np.random.default_rng(14)
    n, b = 300, 1000                                                    # many edges drawn more than once
    score = rng.integers(1, 1000, n).astype(np.uint32)
    idx = rng.integers(-3, n + 3, b).astype(np.int32)
    val = rng.integers(0, 1 << 32, b, dtype=np.uint64).astype(np.uint32)
    want = score.copy().tolist()
    for j in range(b):
        if 0 <= idx[j] < n:
            want[idx[j]] = int(val[j])
    oracle.score_update(score, idx, val)
    assert score.tolist() == want
