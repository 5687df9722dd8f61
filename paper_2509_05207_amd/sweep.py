"""Remote fetches per epoch against cache size (the quantity of the cache-size figure in Sec. 5 "Training Time
and Network Efficiency", here on a synthetic graph): for a grid of n_hot, the misses sum |M_i^e| over several epochs

  * with the cache built from the epoch it serves (the steady cache C_s, swapped in by the double buffer), and
  * with the previous epoch's cache still in place (no swap), which is what the secondary cache is there to avoid.

    python -m paper_2509_05207_amd.sweep --workload medium --epochs 4

Runs on the GPU through the C ABI (schedule, cache build, per-batch classification); prints a table and one JSON line."""
import argparse
import json
import sys
import time

import torch

from . import synth


def sweep(rg, W, epochs, fractions, log=print):
    cfg = W.cfg
    feat = rg.make_features(W.is_local, W.row_of, W.local_rows, W.remote_rows, W.row_bytes)
    scheds = [rg.rg_build_schedule(W.indptr, W.indices, W.train, cfg.batch_size, cfg.fanout, cfg.s0, cfg.worker, cfg.epoch + e)
              for e in range(epochs)]
    # |N_remote| of the first epoch and the fetch count without a cache
    base = [sum(rg.rg_classify_batch(s, None, feat, b)["n_miss"] for b in range(s.n_batches)) for s in scheds]
    full = rg.rg_build_cache([scheds[0]], feat, W.n_nodes)
    n_remote = rg.rg_cache_view(full, W.n_nodes)["K_eff"]
    del full
    rows = []
    for frac in fractions:
        K = int(round(frac * n_remote))
        caches = [rg.rg_build_cache([s], feat, K) for s in scheds]
        fresh = [sum(rg.rg_classify_batch(s, c, feat, b)["n_miss"] for b in range(s.n_batches)) for s, c in zip(scheds, caches)]
        stale = [sum(rg.rg_classify_batch(scheds[e], caches[e - 1], feat, b)["n_miss"] for b in range(scheds[e].n_batches))
                 for e in range(1, epochs)]
        rows.append(dict(K=K, frac_of_remote=frac, fetches_per_epoch=sum(fresh) / epochs,
                         fetches_per_epoch_stale_cache=(sum(stale) / len(stale)) if stale else None,
                         cache_bytes=K * ((W.row_bytes + 15) // 16 * 16)))
        del caches
    return dict(workload=cfg.name, epochs=epochs, n_remote_first_epoch=int(n_remote), fetches_per_epoch_no_cache=sum(base) / epochs, rows=rows)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="medium", choices=sorted(synth.CONFIGS))
    ap.add_argument("--epochs", type=int, default=4)
    ap.add_argument("--fractions", default="0,0.01,0.02,0.05,0.1,0.2,0.3,0.5,0.75,1.0")
    args = ap.parse_args()
    if not torch.cuda.is_available():
        sys.exit("sweep: no GPU visible; the HIP path has no CPU fallback")
    from . import binding as rg
    rg.lib()
    W = synth.make_workload(synth.CONFIGS[args.workload], device="cuda", feature_device="cuda", remote_device="cuda")
    t0 = time.perf_counter()
    res = sweep(rg, W, args.epochs, [float(x) for x in args.fractions.split(",")])
    res["seconds"] = time.perf_counter() - t0
    print(f"# {res['workload']}: {res['epochs']} epochs, |N_remote| = {res['n_remote_first_epoch']}, "
          f"{res['fetches_per_epoch_no_cache']:.0f} remote fetches/epoch without a cache")
    print("| n_hot | share of N_remote | fetches/epoch, cache of the same epoch | fetches/epoch, cache of the epoch before | cache MB |")
    print("|---|---|---|---|---|")
    for r in res["rows"]:
        stale = "-" if r["fetches_per_epoch_stale_cache"] is None else f"{r['fetches_per_epoch_stale_cache']:.0f}"
        print(f"| {r['K']} | {r['frac_of_remote']:.2f} | {r['fetches_per_epoch']:.0f} | {stale} | {r['cache_bytes'] / 1e6:.1f} |")
    print(json.dumps(res))


if __name__ == "__main__":
    main()
