"""Replay of the cache-replacement policy on a synthetic drifting access stream
(TASER, arXiv 2402.05396, Alg. 3 and the experiment of Fig. 3(b): hit rate per
epoch of the policy "cache last epoch's most requested rows", next to a cache
that knows each epoch's frequencies in advance, at 10 / 20 / 30 % of the rows).

Everything the policy does runs in the library (access counting inside the
lookups, epoch-end top-k, overlap test, replacement); this script only draws the
requests, asks for the hit/miss counters and computes the reference hit rate of
the all-knowing cache with numpy. The stream is synthetic: Zipf-distributed
requests over the rows through a rank -> row permutation of which a share is
re-drawn every epoch (popularity drifts).

    python -m paper_2402_05396_amd.cache_policy_replay [--rows 17000] [--dim 413] [--epochs 10]
"""
import argparse
import json

import numpy as np
import torch

import paper_2402_05396_amd as T


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--rows", type=int, default=17000)
    ap.add_argument("--dim", type=int, default=413)
    ap.add_argument("--epochs", type=int, default=10)
    ap.add_argument("--batches", type=int, default=8, help="lookups per epoch")
    ap.add_argument("--requests", type=int, default=400_000, help="requests per lookup")
    ap.add_argument("--zipf", type=float, default=1.0)
    ap.add_argument("--drift", type=float, default=0.02, help="share of the ranks whose row is re-drawn every epoch")
    ap.add_argument("--seed", type=int, default=7)
    args = ap.parse_args(argv)

    rng = np.random.default_rng(args.seed)
    host = torch.from_numpy(rng.standard_normal((args.rows, args.dim)).astype(np.float32)).pin_memory()
    p = 1.0 / np.arange(1, args.rows + 1) ** args.zipf
    p /= p.sum()
    result = {"rows": args.rows, "epochs": args.epochs, "requests_per_epoch": args.batches * args.requests, "ratios": {}}
    for ratio in (0.1, 0.2, 0.3):
        cap = int(ratio * args.rows)
        stream_rng = np.random.default_rng(args.seed + 1)             # the same stream for every ratio
        perm = stream_rng.permutation(args.rows)
        cache = T.cache_init(host, cap, None, seed=args.seed, staging_rows=args.rows - cap)   # "randomly cache k features"
        T.cache_count_accesses(cache)
        hit_miss = torch.zeros(2, dtype=torch.int64, device="cuda")
        out = torch.empty((args.requests, args.dim), dtype=torch.float32, device="cuda")
        rows = []
        for epoch in range(args.epochs):
            moved = stream_rng.choice(args.rows, int(args.drift * args.rows), replace=False)
            perm[moved] = perm[stream_rng.permutation(moved)]
            hit_miss.zero_()
            counts = np.zeros(args.rows, np.int64)
            for _ in range(args.batches):
                ids = perm[stream_rng.choice(args.rows, args.requests, p=p)].astype(np.int32)
                counts += np.bincount(ids, minlength=args.rows)
                T.cache_lookup(cache, torch.from_numpy(ids).cuda(), out=out, hit_miss=hit_miss)
            torch.cuda.synchronize()
            h, m = hit_miss.tolist()
            best = np.sort(counts)[::-1][:cap].sum() / counts.sum()   # the cache that holds this epoch's top rows
            replaced, overlap = T.cache_epoch_end(cache, min_overlap=int(0.95 * cap))
            rows.append({"epoch": epoch, "hit_rate": round(h / (h + m), 4), "all_knowing": round(float(best), 4),
                         "overlap": overlap, "replaced": replaced})
        T.cache_free(cache)
        result["ratios"][f"{int(ratio * 100)}%"] = rows
    print(f"{'epoch':>5s} " + " ".join(f"{r:>8s} {'(best)':>8s}" for r in result["ratios"]))
    for e in range(args.epochs):
        print(f"{e:5d} " + " ".join(f"{v[e]['hit_rate']:8.4f} {v[e]['all_knowing']:8.4f}" for v in result["ratios"].values()))
    print(json.dumps(result))
    return result


if __name__ == "__main__":
    main()
