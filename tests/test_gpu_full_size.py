"""The largest workload (GDELT-shaped: 191 M events, 382 M T-CSR entries, 73 GB edge
table in device memory) at full size, in the launch configuration bench.py times:
the oracle recomputes every sampled output of a whole batch one by one (all 12 000
roots and their 120 000 second-hop roots, most-recent policy), the uniform, weighted and
inverse-timespan finders on several hundred roots that include the longest list, and
properties that hold at any size are checked on everything."""
import numpy as np
import pytest
import torch

import oracle
import paper_2402_05396_amd as T
from paper_2402_05396_amd import workloads as W

pytestmark = pytest.mark.gpu
THREADS = min(16, oracle.max_threads())


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def test_c5_full_size_whole_batch_parity_and_properties():
    free, _ = torch.cuda.mem_get_info()
    if free < 120 * 2 ** 30:
        pytest.skip("needs ~110 GB of free device memory")
    w = W.make(5, num_batches=2)
    n_entries = w.src.shape[0]
    assert n_entries == 382_000_000
    g = T.tcsr_build(dev(w.src), dev(w.dst), dev(w.ts), dev(w.eid), w.num_nodes)
    print("graph built", flush=True)

    # ---- T-CSR: structure checks on the device + a sample of whole lists against the raw events
    indptr, nbr, ts, eid = T.tcsr_view(g)
    deg = torch.bincount(dev(w.src).long(), minlength=w.num_nodes)
    assert torch.equal(indptr[1:] - indptr[:-1], deg) and int(indptr[0]) == 0 and int(indptr[-1]) == n_entries
    seg = torch.repeat_interleave(torch.arange(w.num_nodes, device="cuda"), deg)        # owner of every entry
    same = seg[1:] == seg[:-1]
    assert bool(((ts[1:] >= ts[:-1]) | ~same).all())                                    # time-sorted inside every list
    ev = dev(w.ts[::2])                                                                 # event time by edge id
    assert torch.equal(ev[eid.long()], ts)                                              # records kept together
    del seg, same, deg
    indptr_h = indptr.cpu().numpy()
    rng = np.random.default_rng(0)
    for v in rng.integers(0, w.num_nodes, 6):
        sel = np.flatnonzero(w.src == v)                                                # input order = (ts, position) order
        lo, hi = indptr_h[v], indptr_h[v + 1]
        assert hi - lo == sel.shape[0]
        assert np.array_equal(nbr[lo:hi].cpu().numpy(), w.dst[sel])
        assert np.array_equal(eid[lo:hi].cpu().numpy(), w.eid[sel])
        assert np.array_equal(ts[lo:hi].cpu().numpy(), w.ts[sel])
    del nbr, ts, eid, indptr
    print("T-CSR checked", flush=True)

    # ---- sampler on a whole batch (12 000 roots, 2 hops x 10, most recent)
    roots, times = w.batches[0]
    k = w.k
    got = T.sample_temporal(g, dev(roots), dev(times), k, 2, T.RECENT, 42)
    torch.cuda.synchronize()
    # properties on every output: strictly earlier than the query, a real event of the root, padding after count
    u_ev, v_ev = dev(w.src[::2]), dev(w.dst[::2])
    q_node = [dev(roots), got[0]["nbr"].reshape(-1)]
    q_time = [dev(times), got[0]["ts"].reshape(-1)]
    for h in range(2):
        o = got[h]
        valid = o["eid"] >= 0
        slot = torch.arange(k, device="cuda")[None, :]
        assert torch.equal(valid, slot < o["count"][:, None])
        assert bool((o["ts"] < q_time[h][:, None])[valid].all())
        e = o["eid"].clamp(min=0).long()
        root = q_node[h][:, None].expand(-1, k)
        fwd = (u_ev[e] == root) & (v_ev[e] == o["nbr"])
        bwd = (v_ev[e] == root) & (u_ev[e] == o["nbr"])
        assert bool(((fwd | bwd) & (ev[e] == o["ts"]))[valid].all())
        assert bool((o["ts"][:, :-1] >= o["ts"][:, 1:])[valid[:, 1:]].all())             # most recent first
        assert bool((o["nbr"][~valid] == -1).all()) and bool((o["ts"][~valid] == 0).all())
    # the oracle, one root at a time (linear scans of the raw lists): the whole batch, both hops, every field
    g_ref = oracle.tcsr_build(w.src, w.dst, w.ts, w.eid, w.num_nodes, THREADS)
    print("oracle graph built", flush=True)
    ref = oracle.sample_temporal(g_ref, roots, times, k, 2, oracle.RECENT, 42, threads=THREADS)
    for h in range(2):
        for f in ("nbr", "eid", "ts", "count"):
            assert np.array_equal(got[h][f].cpu().numpy(), ref[h][f]), (h, f)
    print("most-recent finder: whole batch equals the oracle", flush=True)

    # the other finders on 512 roots: 480 of the second batch plus 32 queries on the longest list
    # (37 M entries), from "nothing is earlier" to "everything is earlier"
    hottest = int(np.argmax(indptr_h[1:] - indptr_h[:-1]))
    assert indptr_h[hottest + 1] - indptr_h[hottest] > 30_000_000
    r2, t2 = w.batches[1]
    t_hot = np.concatenate([[w.ts[0], w.ts[0] + 1, w.ts[-1], w.ts[-1] + 1],
                            rng.integers(w.ts[0], w.ts[-1] + 2, 28)]).astype(np.int64)
    roots_x = np.concatenate([r2[:480], np.full(32, hottest, np.int32)]).astype(np.int32)
    times_x = np.concatenate([t2[:480], t_hot]).astype(np.int64)
    assert (roots_x == hottest).sum() >= 32
    weight = rng.integers(1, 1 << 16, w.num_edges, dtype=np.uint32)                      # seeded uint32 weight per edge id
    d_weight = dev(weight.view(np.int32))
    for policy, name, m, hops, n_x in ((T.UNIFORM, "uniform", 0, 2, 512), (T.WEIGHTED, "weighted", 25, 2, 512),
                                       (T.INVERSE_TIMESPAN, "inverse timespan", 0, 1, 512)):
        lo = 512 - n_x
        got_x = T.sample_temporal(g, dev(roots_x[lo:]), dev(times_x[lo:]), k, hops, policy, 42, m,
                                  d_weight if policy == T.WEIGHTED else None)
        torch.cuda.synchronize()
        ref_x = oracle.sample_temporal(g_ref, roots_x[lo:], times_x[lo:], k, hops, policy, 42, m,
                                       weight if policy == T.WEIGHTED else None, threads=THREADS)
        for h in range(hops):
            for f in ("nbr", "eid", "ts", "count"):
                assert np.array_equal(got_x[h][f].cpu().numpy(), ref_x[h][f]), (name, h, f)
        print(f"{name} finder: {n_x} roots x {hops} hops equal the oracle", flush=True)
    del g_ref, d_weight, weight
    print("sampler checked", flush=True)

    # ---- gathers, as bench.py issues them
    table = W.procedural_table_torch(w.edge_seed, w.num_edges, w.edge_dim, torch.float16, 192, "cuda")[:, :w.edge_dim]
    eids = torch.cat([got[0]["eid"].reshape(-1), got[1]["eid"].reshape(-1)])
    edge_out = T.gather_features(table, eids)
    rows = rng.integers(0, eids.numel(), 20000)
    e_np = eids[rows].cpu().numpy()
    want = W.procedural_rows(w.edge_seed, np.maximum(e_np, 0), w.edge_dim, np.float16)
    want[e_np < 0] = 0
    assert edge_out[rows].cpu().numpy().tobytes() == want.tobytes()

    node_host = torch.from_numpy(w.node_feat).pin_memory()
    cap = int(w.cache_ratio * w.num_nodes)
    hot = torch.from_numpy(np.ascontiguousarray(w.notes["hot_order"][:cap]))
    cache = T.cache_init(node_host, cap, hot, staging_rows=w.num_nodes - cap)
    T.cache_tune(cache, stage_blocks=16, refresh_before_gather=True)
    ids = torch.cat([dev(roots), got[0]["nbr"].reshape(-1), got[1]["nbr"].reshape(-1)])
    # as in bench.py: one counted pass and an epoch end first, which also marks the most requested rows
    # (the gather spreads those over the L2 partitions by position)
    T.cache_count_accesses(cache)
    T.cache_prefetch(cache, ids)
    replaced, overlap = T.cache_epoch_end(cache, min_overlap=0)
    T.cache_count_accesses(cache, False)
    assert not replaced and 0 < overlap <= cap
    hm = torch.zeros(2, dtype=torch.int64, device="cuda")
    main, side = torch.cuda.current_stream(), torch.cuda.Stream()
    ready, staged = torch.cuda.Event(), torch.cuda.Event()
    ready.record(main)
    side.wait_event(ready)
    T.cache_prefetch(cache, ids, hit_miss=hm, stream=side)
    staged.record(side)
    main.wait_event(staged)
    node_out = T.cache_gather(cache, ids, stream=main)
    torch.cuda.synchronize()
    ids_np = ids.cpu().numpy()
    assert node_out.cpu().numpy().tobytes() == oracle.gather(w.node_feat, ids_np, threads=THREADS).tobytes()
    assert tuple(hm.tolist()) == oracle.cache_hits(hot.numpy(), w.num_nodes, ids_np)
