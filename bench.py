#!/usr/bin/env python3
"""Benchmark of the mini-batch generation hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic roots:
temporal sampling over 2 hops -> edge-feature gather of every sampled edge ->
node-feature gather (through the device cache) of every root and sampled
neighbor. Inputs (graph, tables, root arrays) are resident in device memory
before the timed region. The K timed steps run twice: launched one by one (this pass times the
dominant kernel for the roofline), then replayed from one HIP graph, which is what `value` and
`ms_per_step` report (`eager_ms_per_step` beside them). Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 5] [--launch graph|eager]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E peak
EDGE_PITCH_ELEMS = {186: 192}   # rows padded to whole 128-byte lines where the width is awkward

# HBM-side traffic per launch of the dominant kernel, from two rocprofv3 --pmc runs
# (FETCH_SIZE, then WRITE_SIZE). The counters cannot be read from inside this process, so
# the figure is a constant taken from the named summary, not from the run that prints it.
MEASURED_TRAFFIC = {
    # (2 x 136 752.8 + 2 148 911.8) KiB per launch
    ("C5-gdelt-shaped", "cache_gather_rows"): (
        2480555418, "profiles/c5_gdelt_shaped_hbm_traffic_pmc.txt: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of this "
                    "benchmark with --edges 20000000 (the node gather reads the same 17 000-row table and serves "
                    "the same number of requests at any event count); not measured in this run"),
}


def log(*a):
    print("[bench]", *a, file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=5, choices=[2, 3, 4, 5])
    ap.add_argument("--edges", type=int, default=None, help="override the event count (smaller = not the named workload)")
    ap.add_argument("--schedule", default="pipeline_node_first",
                    choices=["serial", "overlap", "pipeline", "pipeline_node_first"])
    ap.add_argument("--lanes", type=int, default=2, help="streams that whole batches alternate between (workloads without a node cache)")
    ap.add_argument("--stage-blocks", type=int, default=24, help="width of the PCIe staging copy when it runs beside other kernels")
    ap.add_argument("--policy", default=None, choices=["recent", "uniform", "weighted", "inverse_timespan"],
                    help="override the workload's selection policy (then it is not the named workload)")
    ap.add_argument("--launch", default="graph", choices=["graph", "eager"],
                    help="graph (default): after the eager timed pass, the same steps are captured into one HIP graph "
                         "(both streams, forked and joined by events inside the capture) and the replay is what "
                         "`value` reports; eager: launches one by one only")
    ap.add_argument("--graph", action="store_true", help="same as --launch graph (the default)")
    ap.add_argument("--edge-rows", default="auto", choices=["auto", "finder", "gather"],
                    help="finder: one call finds the neighbors and slices their edge rows (taser_sample_temporal_rows: short rows "
                         "are written by the hop kernels, long ones by one gather launch after the last hop); gather: "
                         "taser_sample_temporal, then taser_gather_features; auto: finder unless a node cache is in the step "
                         "(its schedule puts the late node gather between the sampling and the edge gather)")
    ap.add_argument("--no-refresh", action="store_true", help="do not re-write the gather's working set before the node gather")
    ap.add_argument("--flat-gather", action="store_true", help="node gather in plain output order instead of by L2 partition")
    ap.add_argument("--cache-ratio", type=float, default=None,
                    help="override the share of node rows resident in the device cache (then it is not the named workload)")
    ap.add_argument("--cpu-roots", type=int, default=6000, help="roots of batch 0 the CPU oracle is timed on (0 = skip)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on exactly one GPU (the path has no cross-GPU part); "
              "run it with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2402_05396_amd as T
    from paper_2402_05396_amd import workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    T.lib()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    t0 = time.time()
    kw = {} if args.edges is None else {"edges": args.edges}
    w = W.make(args.config, **kw)
    policy = w.policies[0]
    if args.policy is not None:
        policy = ["recent", "uniform", "weighted", "inverse_timespan"].index(args.policy)
        if policy == 2 and w.edge_weight is None:
            ap.error("this workload has no edge weights")
    log(f"workload {w.name}: {w.num_nodes} nodes, {w.num_edges} events, generated in {time.time() - t0:.1f}s")

    # ------------------------------------------------------------------ resident inputs
    d_src, d_dst, d_ts, d_eid = (torch.from_numpy(x).to(dev) for x in (w.src, w.dst, w.ts, w.eid))
    # a tiny build first: the first launch of a kernel also loads its code object, which would
    # otherwise be counted in the first timed kernel (about 0.6 ms)
    T.tcsr_free(T.tcsr_build(d_src[:4096].contiguous(), d_dst[:4096].contiguous(), d_ts[:4096].contiguous(),
                             d_eid[:4096].contiguous(), w.num_nodes))
    torch.cuda.synchronize()
    T.profile_begin()
    t0 = time.time()
    g = T.tcsr_build(d_src, d_dst, d_ts, d_eid, w.num_nodes)
    torch.cuda.synchronize()
    build_wall_ms = (time.time() - t0) * 1e3
    build_kernels = T.profile_end()
    build_dev_ms = sum(ms for _, ms in build_kernels.values())
    del d_src, d_dst, d_ts, d_eid
    log(f"tcsr_build: {build_wall_ms:.1f} ms wall, {build_dev_ms:.2f} ms in kernels")

    edge_dtype = torch.float16 if w.edge_dtype == "float16" else torch.float32
    pitch = EDGE_PITCH_ELEMS.get(w.edge_dim, w.edge_dim)
    if w.edge_feat is None:
        edge_table = W.procedural_table_torch(w.edge_seed, w.num_edges, w.edge_dim, edge_dtype, pitch, dev)
    else:
        edge_table = torch.zeros((w.num_edges, pitch), dtype=edge_dtype, device=dev)
        edge_table[:, :w.edge_dim] = torch.from_numpy(w.edge_feat).to(dev)
    edge_table = edge_table[:, :w.edge_dim]
    weight = None if w.edge_weight is None else torch.from_numpy(w.edge_weight.view(np.int32)).to(dev)

    cache = None
    if w.node_feat is not None:
        # Alg. 3 as the paper runs it: random residents first; the content the timed steps see is
        # decided further down by one counted pass over the batches and an epoch end.
        node_host = torch.from_numpy(w.node_feat).pin_memory()
        cap = int((w.cache_ratio if args.cache_ratio is None else args.cache_ratio) * w.num_nodes)
        cache = T.cache_init(node_host, cap, None, seed=42, staging_rows=w.num_nodes - cap)
    torch.cuda.synchronize()
    log(f"tables resident after {time.time() - t0:.1f}s")

    k, hops = w.k, w.hops
    R = w.batches[0][0].shape[0]
    n_slots = [R * k ** (h + 1) for h in range(hops)]            # sampled slots per hop
    n_ids = R + sum(n_slots)
    batches = []
    for roots, times in w.batches:
        if roots.shape[0] != R:
            continue                                              # a ragged last batch (chronological workloads) is left out
        ids = torch.empty(n_ids, dtype=torch.int32, device=dev)   # [roots | nbr hop 0 | nbr hop 1]
        ids[:R] = torch.from_numpy(roots).to(dev)
        eids = torch.empty(sum(n_slots), dtype=torch.int32, device=dev)
        out, at_n, at_e, r = [], R, 0, R
        for h in range(hops):
            out.append(dict(nbr=ids[at_n:at_n + n_slots[h]], eid=eids[at_e:at_e + n_slots[h]],
                            ts=torch.empty(n_slots[h], dtype=torch.int64, device=dev),
                            count=torch.empty(r, dtype=torch.int32, device=dev)))
            at_n += n_slots[h]
            at_e += n_slots[h]
            r *= k
        batches.append(dict(roots=ids[:R], times=torch.from_numpy(times).to(dev), ids=ids, eids=eids, out=out))
    # Two sets of output buffers (and two cache handles, i.e. two sets of lookup scratch over
    # the same resident rows) so that consecutive batches can be in flight together.
    n_buf = 2 if w.node_feat is not None else max(2, args.lanes)
    edge_out = [torch.empty((sum(n_slots), w.edge_dim), dtype=edge_dtype, device=dev) for _ in range(n_buf)]
    node_out = [None if cache is None else torch.empty((n_ids, w.node_feat.shape[1]), dtype=torch.float32, device=dev)
                for _ in range(n_buf)]
    caches = [cache]
    warmup_epoch = None
    if cache is not None:
        # One counted pass over all batches with the random content (sampling + classification only),
        # then the epoch end replaces it by the most requested rows.
        def counted_epoch(c):
            hm0 = torch.zeros(2, dtype=torch.int64, device=dev)
            T.cache_count_accesses(c)
            for b in batches:
                T.sample_temporal(g, b["roots"], b["times"], k, hops, policy, 42, w.m, weight, out=b["out"])
                T.cache_prefetch(c, b["ids"], hit_miss=hm0)
            replaced, overlap = T.cache_epoch_end(c, min_overlap=cap)
            T.cache_count_accesses(c, False)
            return hm0.tolist(), replaced, overlap
        (h0, m0), replaced, overlap = counted_epoch(cache)
        residents = T.cache_residents(cache)
        warmup_epoch = {"batches": len(batches), "hit_rate_random_residents": round(h0 / max(h0 + m0, 1), 4),
                        "top_rows_resident_before": overlap, "replaced": replaced}
        log(f"cache warm-up epoch: hit rate {warmup_epoch['hit_rate_random_residents']} with random residents, "
            f"{overlap} of the {cap} most requested rows were resident, replaced = {replaced}")
        # the second handle: the same content, and one counted epoch of its own (the epoch end also
        # records which rows are requested most, which the gather uses to balance its work)
        caches.append(T.cache_init(node_host, cap, residents, staging_rows=w.num_nodes - cap))
        _, replaced2, _ = counted_epoch(caches[1])
        assert not replaced2 and torch.equal(T.cache_residents(caches[1]), residents)
        for c in caches:
            T.cache_tune(c, partitioned_gather=not args.flat_gather)
        if args.schedule != "serial":
            for c in caches:
                T.cache_tune(c, stage_blocks=args.stage_blocks, refresh_before_gather=not args.no_refresh)
    hit_miss = torch.zeros(2, dtype=torch.int64, device=dev)
    main = torch.cuda.current_stream()
    side = torch.cuda.Stream()                       # same (default) priority as the main stream
    ev_sampled = [torch.cuda.Event() for _ in range(n_buf)]
    ev_staged = [torch.cuda.Event() for _ in range(n_buf)]

    rows_call = args.edge_rows == "finder" or (args.edge_rows == "auto" and cache is None)   # one call for neighbors and edge rows
    edge_rows = []                                   # per buffer set: one view of edge_out per hop
    for s in range(n_buf):
        views, at = [], 0
        for h in range(hops):
            views.append(edge_out[s][at:at + n_slots[h]])
            at += n_slots[h]
        edge_rows.append(views)

    def sample(b, s, stream=None):
        stream = main if stream is None else stream
        if rows_call:
            T.sample_temporal_rows(g, b["roots"], b["times"], k, hops, policy, 42, edge_table, m=w.m, edge_weight=weight,
                                   out=b["out"], rows_out=edge_rows[s], stream=stream)
        else:
            T.sample_temporal(g, b["roots"], b["times"], k, hops, policy, 42, w.m, weight, out=b["out"], stream=stream)

    def edge_gather(b, s, stream=None):
        if not rows_call:
            T.gather_features(edge_table, b["eids"], out=edge_out[s], stream=main if stream is None else stream)

    # (not for batches so small that a step is a few microseconds: there the fork and join cost more than they hide)
    two_lanes = cache is None and args.schedule != "serial" and sum(n_slots) >= 100_000
    lanes = [None, side] + [torch.cuda.Stream() for _ in range(n_buf - 2)]     # lane 0 is whatever `main` is at the time
    ev_fork, ev_join = torch.cuda.Event(), [torch.cuda.Event() for _ in range(n_buf - 1)]

    def run(first, count):
        """`count` passes of the whole path over consecutive batches.
        serial:   everything on one stream.
        overlap:  per batch, the PCIe staging of missed node rows runs on a side stream beside
                  the edge gather.
        pipeline: the staging of batch i also runs beside the sampling and edge gather of batch
                  i+1; the node gather of batch i is issued one batch late (two buffer sets).
        pipeline_node_first (default): the same, with the late node gather issued before the
                  edge gather of the current batch.
        Workloads without a node cache have no bus-bound part to hide; for them every schedule but
        `serial` lets whole batches alternate between two streams (each with its own output buffers;
        a batch always goes to the same stream), so that the latency-bound sampling of one batch
        runs beside the bandwidth-bound row copies of the other."""
        if two_lanes:
            ev_fork.record(main)
            for x in lanes[1:]:
                x.wait_event(ev_fork)
            for i in range(count):
                bi = (first + i) % len(batches)
                s = bi % n_buf
                lane = main if s == 0 else lanes[s]
                sample(batches[bi], s, lane)
                edge_gather(batches[bi], s, lane)
            for x, e in zip(lanes[1:], ev_join):
                e.record(x)
                main.wait_event(e)
            return
        pending = None
        for i in range(count):
            b, s = batches[(first + i) % len(batches)], i % n_buf
            sample(b, s)
            if cache is None or args.schedule == "serial":
                edge_gather(b, s)
                if cache is not None:
                    T.cache_lookup(caches[s], b["ids"], out=node_out[s], hit_miss=hit_miss, stream=main)
                continue
            ev_sampled[s].record(main)
            side.wait_event(ev_sampled[s])
            T.cache_prefetch(caches[s], b["ids"], hit_miss=hit_miss, stream=side)
            ev_staged[s].record(side)
            if args.schedule == "pipeline_node_first":
                if pending is not None:
                    pb, ps = pending
                    main.wait_event(ev_staged[ps])
                    T.cache_gather(caches[ps], pb["ids"], out=node_out[ps], stream=main)
                pending = (b, s)
                edge_gather(b, s)
                continue
            edge_gather(b, s)
            if args.schedule == "pipeline":
                if pending is not None:
                    pb, ps = pending
                    main.wait_event(ev_staged[ps])
                    T.cache_gather(caches[ps], pb["ids"], out=node_out[ps], stream=main)
                pending = (b, s)
            else:
                main.wait_event(ev_staged[s])
                T.cache_gather(caches[s], b["ids"], out=node_out[s], stream=main)
        if pending is not None:
            pb, ps = pending
            main.wait_event(ev_staged[ps])
            T.cache_gather(caches[ps], pb["ids"], out=node_out[ps], stream=main)

    # Warm-up, with every library kernel bracketed by events: this names the dominant
    # HBM-bound kernel (the longest of the two gathers; the staging kernel is bound by PCIe
    # and runs beside them on the side stream).
    T.profile_begin()
    run(0, max(args.warmup, 1))
    torch.cuda.synchronize()
    warm = T.profile_end()
    # (with the edge rows written by the hop kernels, those kernels stand for the edge gather)
    finder_names = [n for n in warm if n.startswith("sample_rows_")]
    fused = bool(finder_names)                       # short rows: the hop kernels wrote them; else the call launched the gather
    dominant = max((n for n in warm if n in ("cache_gather_rows", "gather_rows") or n in finder_names), key=lambda n: warm[n][1])
    hit_miss.zero_()
    torch.cuda.synchronize()

    # ------------------------------------------------------------------ timed regions
    # Timed region 1: K steps launched one by one, only the dominant kernel bracketed by HIP events
    # on its own stream (the roofline's time comes from here; 16 event records per step on two
    # streams would cost about 5 % of the step, two cost next to nothing).
    T.profile_begin_only(dominant)
    t0 = time.perf_counter()
    run(0, args.steps)
    torch.cuda.synchronize()
    elapsed_eager = time.perf_counter() - t0
    dominant_time = T.profile_end()[dominant]
    hm = hit_miss.tolist()
    elapsed, launch = elapsed_eager, "eager"
    # Timed region 2 (default): the same K steps captured into one HIP graph (both streams; the side
    # stream is forked from and joined to the capturing stream by the events run() records) and
    # replayed: one untimed replay, then the timed one. `value` is taken from it; if the capture is
    # refused the eager figure stands.
    if args.launch == "graph":
        try:
            capture = torch.cuda.Stream()
            capture.wait_stream(main)
            graph = torch.cuda.CUDAGraph()
            outer_main = main
            try:
                with torch.cuda.stream(capture):
                    with torch.cuda.graph(graph, stream=capture):
                        main = capture                   # run() launches on `main`
                        run(0, args.steps)
            finally:
                main = outer_main
            main.wait_stream(capture)
            graph.replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            graph.replay()
            torch.cuda.synchronize()
            elapsed, launch = time.perf_counter() - t0, "one HIP graph of all timed steps"
            del graph
        except Exception as e:
            log(f"HIP graph capture failed ({type(e).__name__}: {e}); the eager figure stands")
            torch.cuda.synchronize()
    ms_per_step = elapsed * 1e3 / args.steps

    # The same steps once more with every kernel bracketed, for the per-kernel table.
    T.profile_begin()
    run(0, args.steps)
    torch.cuda.synchronize()
    kernels = T.profile_end()

    # ------------------------------------------------------------------ accounting
    # Two byte counts per gather. "Algorithmic": every served row counted as read + written + its
    # id, however often the same source row is asked for. "HBM": what has to cross the memory
    # interface at least once per launch: the dense output, the ids, and every DISTINCT source row
    # requested (a row asked for 100 times is read from HBM once and from L2 after that). The
    # roofline fraction is taken on the second count, so it cannot exceed 1.
    used = [batches[i % len(batches)] for i in range(args.steps)]
    neighbors = sum(int(sum(int(o["count"].sum()) for o in b["out"])) for b in used)
    edge_rb = w.edge_dim * edge_table.element_size()
    node_rb = 0 if cache is None else w.node_feat.shape[1] * 4
    edge_bytes = sum(n_slots) * (2 * edge_rb + 4)                 # row read + row written + id
    node_bytes = n_ids * (2 * node_rb + 4) if cache is not None else 0
    gather_bytes_per_step = edge_bytes + node_bytes
    value = neighbors / elapsed
    gather_gbps = gather_bytes_per_step * args.steps / elapsed / 1e9

    def distinct_valid(t):
        t = t[t >= 0]
        return int(torch.unique(t).numel())
    seen = {id(b): b for b in used}.values()                      # each distinct batch once
    edge_distinct = sum(distinct_valid(b["eids"]) for b in seen) / len(seen)
    node_distinct = sum(distinct_valid(b["ids"]) for b in seen) / len(seen) if cache is not None else 0
    edge_hbm = sum(n_slots) * (edge_rb + 4) + edge_distinct * edge_rb
    node_hbm = n_ids * (node_rb + 4) + node_distinct * node_rb if cache is not None else 0

    per_kernel = {n: {"launches": c, "avg_ms": ms / c} for n, (c, ms) in kernels.items()}
    alg_of = {"cache_gather_rows": node_bytes, "gather_rows": edge_bytes}
    hbm_of = {"cache_gather_rows": node_hbm, "gather_rows": edge_hbm}
    out_bytes = {"cache_gather_rows": n_ids * node_rb, "gather_rows": sum(n_slots) * edge_rb}
    for n in finder_names:          # one launch per hop under one name: bytes per average launch
        alg_of[n], hbm_of[n], out_bytes[n] = edge_bytes / hops, edge_hbm / hops, sum(n_slots) * edge_rb / hops
    roofline = None
    if dominant in hbm_of:
        dom_ms = dominant_time[1] / dominant_time[0]            # measured inside the timed region
        achieved = hbm_of[dominant] / (dom_ms * 1e-3) / 1e9
        traffic, traffic_source = MEASURED_TRAFFIC.get((w.name if args.edges is None else None, dominant), (None, None))
        roofline = {"kernel": dominant, "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
                    "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                    "avg_launch_ms": round(dom_ms, 4), "launches_timed": dominant_time[0],
                    "hbm_bytes": int(hbm_of[dominant]),
                    "bytes_note": "achieved = (dense output + 4 B id per row + every distinct source row once) / "
                                  "average launch time inside the eager timed region (events cannot be read back from a graph)"
                                  + ("; this kernel finds the neighbors and writes their edge rows, one launch per hop: "
                                     "the bytes are the edge rows' alone, averaged over the hops" if dominant in finder_names else ""),
                    "algorithmic_bytes": int(alg_of[dominant]),
                    "algorithmic_GBps": round(alg_of[dominant] / (dom_ms * 1e-3) / 1e9, 1),
                    "algorithmic_note": "rows x (row read + row written + id): repeated source rows are served by "
                                        "L2, so this figure can exceed the HBM peak and is not a roofline fraction",
                    "output_write_GBps": round(out_bytes[dominant] / (dom_ms * 1e-3) / 1e9, 1),
                    "traffic": traffic, "traffic_source": traffic_source}
        if traffic:
            t_gbps = traffic / (dom_ms * 1e-3) / 1e9
            roofline["traffic_GBps"] = round(t_gbps, 1)               # measured HBM-side bytes / measured time
            roofline["traffic_frac"] = round(t_gbps / HBM_PEAK_GBPS, 4)

    # Every row of the path against the roofline that bounds it (per-kernel times of the second pass).
    def hbm_row(hbm, alg, ms, note=None):
        r = {"bound": "hbm", "hbm_bytes": int(hbm), "ms": round(ms, 4),
             "achieved_GBps": round(hbm / (ms * 1e-3) / 1e9, 1), "frac_of_hbm_peak": round(hbm / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
             "algorithmic_bytes": int(alg), "algorithmic_GBps": round(alg / (ms * 1e-3) / 1e9, 1)}
        if note:
            r["note"] = note
        return r
    n_entries = int(w.src.shape[0])
    sample_ms = sum(ms for n, (c, ms) in kernels.items() if n.startswith("sample_")) / args.steps
    roots_per_step = R + sum(n_slots[:-1])
    build_alg = n_entries * (20 + 16) + (w.num_nodes + 1) * 8
    sampler_bytes = roots_per_step * 20 + neighbors / args.steps * 32 + roots_per_step * 56
    rows_report = {
        "a1_tcsr_build": hbm_row(build_alg, build_alg, build_dev_ms,
                                 "once per graph; bytes = 20 in + 16 out per entry; a multi-pass sort moves more"),
        "a2_a6_sampler": dict(hbm_row(sampler_bytes, sampler_bytes, sample_ms,
                                      "bound by dependent-read latency, not bytes: per root 16 B of list bounds + 4 B count + "
                                      "about 7 index/record probes of 8 B; per kept neighbor 16 B read + 16 B written"),
                              neighbors_per_s=round(neighbors / args.steps / (sample_ms * 1e-3), 1)),
    }
    if fused:
        del rows_report["a2_a6_sampler"]
        rows_report["a2_a7_sampler_writing_edge_rows"] = dict(
            hbm_row(sampler_bytes + edge_hbm, sampler_bytes + edge_bytes, sample_ms,
                    "one launch per hop finds the neighbors and copies their edge rows (searching wavefronts run beside copying ones)"),
            neighbors_per_s=round(neighbors / args.steps / (sample_ms * 1e-3), 1))
    else:
        rows_report["a7_edge_gather"] = hbm_row(edge_hbm, edge_bytes, per_kernel["gather_rows"]["avg_ms"])
    step_hbm_bytes = sampler_bytes + edge_hbm
    if cache is not None:
        lookup_ms = sum(per_kernel[n]["avg_ms"] for n in ("cache_classify", "cache_refresh_working_set", "cache_gather_rows")
                        if n in per_kernel)
        rows_report["a8_node_gather_through_cache"] = hbm_row(
            node_hbm + n_ids * 8, node_bytes, lookup_ms,
            "classify (+ working-set re-write) + gather on the HBM side, 8 B per request more for the location array; "
            f"the staging of missed rows ({per_kernel['cache_stage_misses']['avg_ms']:.3f} ms, bus-bound) runs beside it "
            "on the side stream")
        step_hbm_bytes += node_hbm + n_ids * 8
    step_hbm_frac = step_hbm_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS
    gather_hbm_gbps = (edge_hbm + node_hbm) / (ms_per_step * 1e-3) / 1e9

    # ------------------------------------------------------------------ cache maintenance (outside the timed region)
    # Cost of the access counters of Alg. 3 inside the classify kernel, and of one epoch-end
    # top-k + overlap test (no replacement: the residents already are the hottest rows).
    maintenance = None
    if cache is not None:
        T.cache_count_accesses(caches[0])
        torch.cuda.synchronize()
        T.profile_begin()
        for i in range(10):
            T.cache_prefetch(caches[0], batches[i % len(batches)]["ids"], stream=main)
        torch.cuda.synchronize()
        counted = T.profile_end()
        t0 = time.perf_counter()
        replaced, overlap = T.cache_epoch_end(caches[0], min_overlap=0)
        t_epoch = time.perf_counter() - t0
        T.cache_count_accesses(caches[0], False)
        maintenance = {"classify_with_counting_ms": round(counted["cache_classify"][1] / counted["cache_classify"][0], 4),
                       "classify_without_counting_ms": round(per_kernel["cache_classify"]["avg_ms"], 4),
                       "epoch_end_wall_ms": round(t_epoch * 1e3, 3), "epoch_end_overlap": overlap,
                       "rows": w.num_nodes, "capacity": cache.capacity}

    # ------------------------------------------------------------------ further rows (outside the timed region)
    # Candidate-window products of the adaptive sampler on this batch's roots (m = 25 most recent
    # candidates, encodings, 10 of 25 by per-slot weights) and adaptive mini-batch selection over
    # the 10^6 latest events (the training split the paper uses for its largest dataset).
    b0 = batches[0]
    m_c = 25
    cand = T.sample_temporal(g, b0["roots"], b0["times"], m_c, 1, T.RECENT, 42, stream=main)[0]
    slot_w = torch.randint(1, 1 << 16, (R, m_c), dtype=torch.int32, device=dev)
    n_train = min(1_000_000, w.num_edges)
    selector = T.selector_init(n=n_train, initial_score=6554)
    new_scores = torch.randint(1, 1 << 17, (R // 3,), dtype=torch.int32, device=dev)
    for it in range(-2, 20):                     # two untimed passes first
        if it == 0:
            torch.cuda.synchronize()
            T.profile_begin()
        T.candidate_encodings(cand["nbr"], cand["count"], stream=main)
        T.select_weighted(slot_w, cand["count"], k, 42, 0, candidates=cand, stream=main)
        drawn = T.selector_draw(selector, R // 3, 42, it + 2, stream=main)
        T.selector_update(selector, drawn, new_scores, stream=main)
    torch.cuda.synchronize()
    extra = T.profile_end()
    further = {"roots": R, "m": m_c, "k": k, "training_edges": n_train, "batch_edges": R // 3,
               "avg_ms": {n: round(ms / c, 4) for n, (c, ms) in extra.items()}}
    T.selector_free(selector)
    del cand, slot_w, new_scores

    # A plain streaming kernel of known size (out[i] = in[i] + 1 over int32: 1 GiB read +
    # 1 GiB written): under rocprofv3 --pmc its FETCH_SIZE / WRITE_SIZE readings calibrate
    # the counters' unit for the kernels above.
    calib_src = torch.zeros(1 << 28, dtype=torch.int32, device=dev)
    calib_dst = torch.empty_like(calib_src)
    torch.cuda.synchronize()
    torch.add(calib_src, 1, out=calib_dst)
    torch.cuda.synchronize()
    del calib_src, calib_dst

    # ------------------------------------------------------------------ CPU oracle on a bounded sample
    cpu = None
    if args.cpu_roots > 0:
        import oracle
        threads = min(16, oracle.max_threads(), len(os.sched_getaffinity(0)))
        t0 = time.time()
        g_ref = oracle.tcsr_build(w.src, w.dst, w.ts, w.eid, w.num_nodes, threads)
        t_build = time.time() - t0
        roots, times = w.batches[0]
        nr = min(args.cpu_roots, roots.shape[0])
        t0 = time.perf_counter()
        ref = oracle.sample_temporal(g_ref, roots[:nr], times[:nr], k, hops, policy, 42, w.m, w.edge_weight, threads)
        t_sample = time.perf_counter() - t0
        t0 = time.perf_counter()
        node_ref = None
        if w.node_feat is not None:
            node_ref = oracle.gather(w.node_feat, np.concatenate([roots[:nr]] + [o["nbr"].ravel() for o in ref]), threads=threads)
        edge_ref = None
        if w.edge_feat is not None:
            edge_ref = oracle.gather(w.edge_feat, np.concatenate([o["eid"].ravel() for o in ref]), threads=threads)
        t_gather = time.perf_counter() - t0
        cpu_neighbors = sum(int(o["count"].sum()) for o in ref)
        # the oracle must agree with what the device produced for the same roots
        got = batches[0]["out"]
        run(0, 1)
        torch.cuda.synchronize()
        for h in range(hops):
            for f in ("nbr", "eid", "ts"):
                assert np.array_equal(got[h][f][:nr * k ** (h + 1)].cpu().numpy(), ref[h][f].ravel()), f"GPU/oracle mismatch: hop {h} {f}"
            assert np.array_equal(got[h]["count"][:nr * k ** h].cpu().numpy(), ref[h]["count"].ravel()), f"GPU/oracle mismatch: hop {h} count"
        if edge_ref is not None:
            # the edge rows of those roots' slots (run(0, 1) left them in edge_out[0], hop after hop)
            at, parts = 0, []
            for h in range(hops):
                parts.append(edge_out[0][at:at + nr * k ** (h + 1)])
                at += n_slots[h]
            assert torch.cat(parts).cpu().numpy().tobytes() == edge_ref.tobytes(), "GPU/oracle mismatch: edge rows"
        if node_ref is not None:
            # the node rows the device served for those roots and their sampled neighbors (run(0, 1) left them in node_out[0])
            at, parts, r_h = 0, [node_out[0][:nr]], R
            for h in range(hops):
                at += r_h
                r_h *= k
                parts.append(node_out[0][at:at + nr * k ** (h + 1)])
            assert torch.cat(parts).cpu().numpy().tobytes() == node_ref.tobytes(), "GPU/oracle mismatch: node rows"
        sample = (f"first {nr} roots of batch 0, {hops} hops: sampler {t_sample:.2f}s + "
                  f"{'node' if w.edge_feat is None else 'edge'}-feature gather {t_gather:.2f}s; "
                  f"oracle T-CSR build ({t_build:.1f}s) not included")
        if w.edge_feat is None:
            sample += "; edge-feature gather excluded (the table exists only in device memory)"
        # the same oracle on one thread, on a twentieth of those roots
        n1 = max(nr // 20, 1)
        t0 = time.perf_counter()
        ref1 = oracle.sample_temporal(g_ref, roots[:n1], times[:n1], k, hops, policy, 42, w.m, w.edge_weight, 1)
        t_one = time.perf_counter() - t0
        one_thread = round(sum(int(o["count"].sum()) for o in ref1) / t_one, 1)
        cpu = {"value": round(cpu_neighbors / (t_sample + t_gather), 1), "unit": "neighbors/s", "cores": threads,
               "one_thread_sampler_neighbors_per_s": one_thread,
               "kind": "oracle", "sample": sample}

    # Bytes a step pulls over the bus: every distinct non-resident row of a batch crosses it once
    # (counted on the host for batch 0 from the ids the device produced).
    pcie_bytes = None
    if cache is not None:
        ids0 = batches[0]["ids"].cpu().numpy()
        missing = np.setdiff1d(np.unique(ids0[ids0 >= 0]), residents.numpy())
        pcie_bytes = int(missing.shape[0]) * node_rb
    result = {
        "metric": "sampled temporal neighbors/sec + gather GB/s (% of HBM peak), 2-hop 10x10",
        "value": round(value, 1), "unit": "neighbors/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "eager_ms_per_step": round(elapsed_eager * 1e3 / args.steps, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int64", "data": "synthetic",
        "config": {"workload": w.name + ("" if args.edges is None else f" (reduced to {w.num_edges} events)"),
                   "events": w.num_edges, "nodes": w.num_nodes, "roots_per_batch": R, "fanout": [k] * hops,
                   "policy": ["recent", "uniform", "weighted", "inverse_timespan"][policy] + ("" if args.policy is None else " (override)"), "edge_row_bytes": edge_rb,
                   "node_row_bytes": node_rb, "distinct_batches": len(batches),
                   "cache_rows": (0 if cache is None else cache.capacity) if args.cache_ratio is None
                   else f"{cache.capacity} (override)",
                   "schedule": f"batches alternate between {n_buf} streams" if two_lanes else ("serial" if cache is None else args.schedule),
                   "edge_rows": ("taser_sample_temporal_rows: " if rows_call else "taser_sample_temporal, taser_gather_features: ")
                   + ("written by the hop kernels" if fused else "one gather launch after the last hop"),
                   "launch": launch},
        "sampler_neighbors_per_s": round(neighbors / args.steps / (sum(ms for n, (c, ms) in kernels.items()
                                                                       if n.startswith("sample_")) / args.steps * 1e-3), 1),
        "gather_GBps": round(gather_gbps, 1), "gather_bytes_per_step": gather_bytes_per_step,
        "gather_hbm_GBps": round(gather_hbm_gbps, 1), "gather_hbm_frac_of_peak": round(gather_hbm_gbps / HBM_PEAK_GBPS, 4),
        "gather_hbm_bytes_per_step": int(edge_hbm + node_hbm),
        "gather_note": "gather_GBps counts algorithmic bytes (every served row read + written + id) over the whole step time: "
                       "repeated rows are served by L2, so it is no fraction of the HBM peak. gather_hbm_* count what the two "
                       "gathers must move through HBM at least once (outputs, ids, distinct source rows) over the same time, "
                       "step_hbm_* the same plus the sampler's traffic: those are fractions of the roofline",
        "step_hbm_bytes": int(step_hbm_bytes), "step_hbm_frac": round(step_hbm_frac, 4),
        "neighbors_per_step": neighbors / args.steps,
        "cache_hit_rate": None if cache is None or sum(hm) == 0 else round(hm[0] / sum(hm), 4),
        "cache_warmup_epoch": warmup_epoch,
        "pcie_bytes_per_step": pcie_bytes,
        "tcsr_build": {"entries": int(w.src.shape[0]), "wall_ms": round(build_wall_ms, 2),
                       "kernel_ms": round(build_dev_ms, 3),
                       "kernels": {n: round(ms, 3) for n, (_, ms) in build_kernels.items()}},
        "kernels": {n: {"launches": v["launches"], "avg_ms": round(v["avg_ms"], 4)} for n, v in per_kernel.items()},
        "kernels_note": "per-kernel times from a second pass of the same steps with every kernel bracketed by events; "
                        "the roofline kernel's time is from the timed region itself",
        "cache_maintenance": maintenance, "further_rows": further, "rows": rows_report, "roofline": roofline, "cpu_baseline": cpu,
    }
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
