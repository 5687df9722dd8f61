"""Benchmark of the RapidGNN data path on one MI355X.

One step = one pass of the whole hot path over one epoch of one synthetic
workload: rg_build_schedule (seeds, shuffle, every hop's sampling and
frontiers), rg_build_cache (tally, TopHot, VectorPull, plans) and
rg_gather_batch for every batch of the epoch.  Inputs are resident in HBM when
the timed region starts; a second, separately reported pass keeps the remote
feature table in pinned host memory (the stand-in for remote partitions), so
its misses cross the host link.

Prints ONE JSON line.  `value` is sampled edges per second over whole steps;
the gathered-feature rate and the per-kernel roofline figures ride along.
Gathers stage --gather-group batches per launch (default: the feature blocks of
the next eight batches back to back in one staging buffer, rg_gather_batches;
more, up to 64, while that would be less than 512 MB per launch).
"""
import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2509_05207_amd import accounting, synth       # noqa: E402

HBM_PEAK_GBPS = 8000.0
METRIC = "sampled edges/s + gathered feature GB/s (fraction of HBM peak), 1 GPU"


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def algorithmic_bytes(rg, sched, indptr, fanout):
    """Per hop: (frontier nodes, sum of degrees, sampled edges, algorithmic bytes of the sampler launch).
    Per frontier node: 16 B of indptr, 4 B frontier ID, 8 B sample offset, 4 B per row entry read,
    4 B per sampled neighbour written."""
    out = []
    for hop, f in enumerate(fanout):
        ids, _, off = rg.rg_schedule_frontier(sched, hop)
        v = ids.long()
        deg = indptr[v + 1] - indptr[v]
        n, sdeg = int(ids.numel()), int(deg.sum().item())
        samp = int(torch.clamp(deg, max=f).sum().item())
        out.append(dict(nodes=n, sum_deg=sdeg, sampled=samp, bytes=n * (16 + 4 + 8) + 4 * sdeg + 4 * samp))
    return out


def run_step(rg, W, feat, out_buf, out_stride, cap_rows, side, group=1):
    cfg = W.cfg
    s = rg.rg_build_schedule(W.indptr, W.indices, W.train, cfg.batch_size, cfg.fanout, cfg.s0, cfg.worker, cfg.epoch)
    c = rg.rg_build_cache([s], feat, W.K)
    if group <= 1:
        for b in range(s.n_batches):
            rg.rg_gather_batch(s, c, feat, b, out_buf, out_stride=out_stride, out_capacity_rows=cap_rows, side_stream=side,
                               want_stats=False)
    else:
        for b in range(0, s.n_batches, group):
            rg.rg_gather_batches(s, c, feat, b, min(group, s.n_batches - b), out_buf, out_stride=out_stride, out_capacity_rows=cap_rows,
                                 side_stream=side, want_stats=False)
    return s, c


def timed(rg, W, feat, out_buf, out_stride, cap_rows, side, steps, warmup, group=1):
    for _ in range(warmup):
        run_step(rg, W, feat, out_buf, out_stride, cap_rows, side, group)
    torch.cuda.synchronize()
    rg.rg_profile_reset()
    t0 = time.perf_counter()
    for _ in range(steps):
        s, c = run_step(rg, W, feat, out_buf, out_stride, cap_rows, side, group)
        del s, c
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    return dt, rg.rg_profile_read()


def overlapped_leg(rg, W, feat, out_stride, epochs=6, group=1):
    """E epochs end to end with the precompute of epoch e+1 (schedule, tally, TopHot, cache, plan: compute- and
    cache-bound) running on a second host thread and stream beside the gathers of epoch e (HBM-bound), as Alg. 1
    arranges it.  Every epoch's whole hot path runs inside the timed region."""
    import queue
    import threading
    cfg = W.cfg
    ready = queue.Queue(maxsize=1)            # the builder stays at most one epoch ahead (two schedules alive)
    build_stream = torch.cuda.Stream()
    errors = []

    def builder():
        try:
            torch.cuda.set_device(0)
            for e in range(epochs):
                s = rg.rg_build_schedule(W.indptr, W.indices, W.train, cfg.batch_size, cfg.fanout, cfg.s0, cfg.worker,
                                         cfg.epoch + e, stream=build_stream)
                c = rg.rg_build_cache([s], feat, W.K, stream=build_stream)
                ready.put((s, c))
        except Exception as ex:           # noqa: BLE001 -- handed to the main thread
            errors.append(ex)
            ready.put(None)

    m_cap = None
    outs = None
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    th = threading.Thread(target=builder)
    th.start()
    edges = 0
    for e in range(epochs):
        item = ready.get()
        if item is None:
            th.join()
            raise errors[0]
        s, c = item
        off_L = rg.rg_schedule_frontier(s, s.L)[2]
        need = max(int(off_L[min(b + group, s.n_batches)] - off_L[b]) for b in range(0, s.n_batches, group))
        if m_cap is None or need > m_cap:
            m_cap = need + need // 8
            outs = [torch.empty(m_cap * out_stride, dtype=torch.uint8, device="cuda") for _ in range(2)]
        for i, b in enumerate(range(0, s.n_batches, group)):
            rg.rg_gather_batches(s, c, feat, b, min(group, s.n_batches - b), outs[i & 1], out_stride=out_stride, out_capacity_rows=m_cap,
                                 want_stats=False)
        edges += sum(rg.rg_schedule_samples(s, h)[1].numel() for h in range(s.L))
        torch.cuda.current_stream().synchronize()      # the epoch's gathers are done before its handles go
        del s, c
    th.join()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    return {"epochs": epochs, "ms_per_epoch": dt / epochs * 1e3, "value": edges / dt, "unit": "sampled edges/s",
            "note": "precompute of epoch e+1 on a second host thread and stream beside the gathers of epoch e"}


def runtime_leg(rg, W, feat, epochs=3, Q=4):
    """The rows after the three calls: E epochs with the double-buffered cache and the depth-Q prefetch queue,
    and the computation blocks of one epoch.  Reported beside the headline figure, never part of it."""
    cfg = W.cfg
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    scheds = [rg.rg_build_schedule(W.indptr, W.indices, W.train, cfg.batch_size, cfg.fanout, cfg.s0, cfg.worker, cfg.epoch + e)
              for e in range(epochs)]
    t_sched = time.perf_counter() - t0
    m_cap = max(int(np.diff(rg.rg_schedule_frontier(s, s.L)[2]).max()) for s in scheds)
    slots = [torch.empty(m_cap * W.stride_bytes, dtype=torch.uint8, device="cuda") for _ in range(Q)]
    pair = rg.rg_cache_pair_create(scheds[0], feat, W.K)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    staged = total = 0
    for e in range(epochs):
        if e + 1 < epochs:
            rg.rg_cache_pair_begin_next(pair, scheds[e + 1])
        pf = rg.rg_prefetcher_create(scheds[e], rg.rg_cache_pair_primary(pair), feat, slots, out_stride=W.stride_bytes,
                                     slot_capacity_rows=m_cap)
        for _ in range(scheds[e].n_batches):
            rg.rg_prefetcher_fill(pf)
            _, _, _, was = rg.rg_prefetcher_acquire(pf)
            rg.rg_prefetcher_release(pf)
            staged += int(was)
            total += 1
        del pf
        if e + 1 < epochs:
            assert rg.rg_cache_pair_swap(pair, wait=True)
    torch.cuda.synchronize()
    t_run = time.perf_counter() - t0
    table_bytes = rg.rg_cache_pair_table_bytes(pair)
    del pair
    rg.rg_profile_reset()
    t0 = time.perf_counter()
    rg.rg_schedule_build_blocks(scheds[0])
    t_blk = time.perf_counter() - t0
    blk = rg.rg_profile_read()["blocks"]
    n_samp = sum(rg.rg_schedule_block(scheds[0], h).numel() for h in range(scheds[0].L))
    # the metadata block through a file and back
    import tempfile
    with tempfile.TemporaryDirectory() as td:
        path = os.path.join(td, "epoch.rgsched")
        t0 = time.perf_counter()
        rg.rg_schedule_save(scheds[0], path)
        t_save = time.perf_counter() - t0
        file_bytes = os.path.getsize(path)
        t0 = time.perf_counter()
        loaded = rg.rg_schedule_load(path)
        t_load = time.perf_counter() - t0
        del loaded
    # the O(f) alternative sampler on the same epoch (a different, equally distributed sample: never the headline figure)
    del scheds
    rg.rg_build_schedule_with(W.indptr, W.indices, W.train, cfg.batch_size, cfg.fanout, cfg.s0, cfg.worker, cfg.epoch,
                              sampler=rg.RG_SAMPLER_POSITIONS)
    torch.cuda.synchronize()
    rg.rg_profile_reset()
    reps = 3
    t0 = time.perf_counter()
    for _ in range(reps):
        sp = rg.rg_build_schedule_with(W.indptr, W.indices, W.train, cfg.batch_size, cfg.fanout, cfg.s0, cfg.worker, cfg.epoch,
                                       sampler=rg.RG_SAMPLER_POSITIONS)
    torch.cuda.synchronize()
    t_pos = (time.perf_counter() - t0) / reps
    pos_kernel_ms = rg.rg_profile_read()["sampler"]["ms"] / reps
    pos_edges = sum(rg.rg_schedule_samples(sp, h)[1].numel() for h in range(sp.L))
    del sp
    return {"epochs": epochs, "Q": Q, "schedule_build_ms_per_epoch": t_sched / epochs * 1e3,
            "schedule_file": {"bytes": file_bytes, "save_ms": t_save * 1e3, "load_ms": t_load * 1e3},
            "position_sampler": {"schedule_build_ms": t_pos * 1e3, "sampler_kernel_ms": pos_kernel_ms, "sampled_edges": pos_edges,
                                 "edges_per_s_kernel": pos_edges / (pos_kernel_ms * 1e-3) if pos_kernel_ms else None},
            "gather_epoch_ms_with_next_cache_built_alongside": t_run / epochs * 1e3, "staged_fraction": staged / max(1, total),
            "cache_table_bytes": table_bytes, "staging_bytes": Q * m_cap * W.stride_bytes,
            "blocks_ms_per_epoch": t_blk * 1e3, "blocks_kernel_ms": blk["ms"], "block_edges": n_samp}


def cpu_baseline(W, indptr_h, indices_h, train_h, budget_s=15.0):
    """The oracle, as it stands, on a bounded prefix of the epoch's batches."""
    import oracle
    cfg = W.cfg
    threads = max(1, min(16, oracle.max_threads(), os.cpu_count() or 1))
    feats = oracle.Features(W.is_local.cpu().numpy(), W.row_of.cpu().numpy(),
                            W.local_rows.contiguous().view(torch.uint8).cpu().numpy(), W.stride_bytes,
                            W.remote_rows.contiguous().view(torch.uint8).cpu().numpy(), W.stride_bytes, W.row_bytes)
    beta = accounting.batches_per_epoch(cfg.n_train, cfg.batch_size)

    def one(nb):
        t0 = time.perf_counter()
        s = oracle.Schedule(indptr_h, indices_h, train_h, cfg.batch_size, cfg.fanout, cfg.s0, cfg.worker, cfg.epoch,
                            batch_lo=0, batch_hi=nb, n_threads=threads)
        t1 = time.perf_counter()
        freq = oracle.frequency([s], W.n_nodes)
        ids, _ = oracle.top_hot(freq, feats.is_local, W.K)
        oracle.cache_fill(ids, feats, table_stride=W.stride_bytes)
        t2 = time.perf_counter()
        for b in range(s.n_batches):
            oracle.gather_batch(s, b, feats, out_stride=W.stride_bytes)
        t3 = time.perf_counter()
        edges = sum(int(s.samples(h)[1].size) for h in range(s.L))
        return t3 - t0, edges, {"schedule": t1 - t0, "cache": t2 - t1, "gather": t3 - t2}
    dt1, _, _ = one(min(threads, beta))
    nb = int(max(threads, min(beta, threads * max(1.0, budget_s / max(dt1, 1e-3)))))
    nb = min(beta, nb // threads * threads if nb >= threads else nb)
    dt, edges, phases = one(nb)
    model = ""
    try:
        with open("/proc/cpuinfo") as fh:
            model = next((ln.split(":", 1)[1].strip() for ln in fh if ln.startswith("model name")), "")
    except OSError:
        pass
    return dict(value=edges / dt, unit="sampled edges/s", cores=threads, kind="oracle",
                sample=f"first {nb} of {beta} batches of the epoch: schedule ({threads} threads, one batch per thread), "
                       f"frequency, TopHot, cache fill and gather of those batches (single thread); {dt:.1f} s",
                seconds={k: round(v, 3) for k, v in phases.items()}, cpu_model=model, host_cpus=os.cpu_count())


def device_copy_gbps(n_bytes=1 << 30, reps=5):
    """Read + write rate of a plain device-to-device copy of n_bytes on this GPU: the yardstick beside the 8 TB/s peak."""
    a = torch.empty(n_bytes, dtype=torch.uint8, device="cuda")
    b = torch.empty_like(a)
    a.fill_(1)
    b.copy_(a)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        b.copy_(a)
    e1.record()
    torch.cuda.synchronize()
    return 2.0 * n_bytes * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9


def measured_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` on `workload` from the committed rocprofv3 --pmc runs
    (profiles/*_traffic.md says how they were taken), or None when there is no such measurement."""
    path = os.path.join(ROOT, "paper_2509_05207_amd", "measured_traffic.json")
    try:
        with open(path) as fh:
            table = json.load(fh)
    except (OSError, ValueError):
        return None
    rec = table.get(f"{workload}:{kernel}")
    return rec.get("hbm_bytes_per_launch") if rec else None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="medium", choices=sorted(synth.CONFIGS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--gather-group", type=int, default=0,
                    help="batches whose feature blocks one gather launch stages back to back (rg_gather_batches, the prefetcher's Q); "
                         "1 = one launch per batch; 0 = eight, doubled up to 64 while a launch would stage less than 512 MB")
    ap.add_argument("--no-pcie-pass", action="store_true")
    ap.add_argument("--no-runtime-leg", action="store_true", help="skip the multi-epoch cache-pair / prefetch-queue / blocks leg")
    ap.add_argument("--pmc-probe", action="store_true",
                    help="also run one plain elementwise kernel of known size (1 GiB read + 1 GiB written), the yardstick "
                         "that rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings of the library's kernels are scaled by")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1")
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the HIP path has no CPU fallback")

    from paper_2509_05207_amd import binding as rg
    rg.lib()
    torch.cuda.set_device(0)
    cfg = synth.CONFIGS[args.workload]
    t0 = time.perf_counter()
    W = synth.make_workload(cfg, device="cuda", feature_device="cuda", remote_device="cuda")
    torch.cuda.synchronize()
    log(f"[bench] workload {cfg.name}: {W.n_nodes} nodes, {W.indices.numel()} edges, K={W.K}, generated in {time.perf_counter() - t0:.1f} s")
    assert rg.rg_graph_validate(W.indptr, W.indices) == 0

    feat_hbm = rg.make_features(W.is_local, W.row_of, W.local_rows, W.remote_rows, W.row_bytes)
    side = torch.cuda.Stream()

    # sizes and algorithmic bytes from one untimed pass
    s = rg.rg_build_schedule(W.indptr, W.indices, W.train, cfg.batch_size, cfg.fanout, cfg.s0, cfg.worker, cfg.epoch)
    hops = algorithmic_bytes(rg, s, W.indptr, cfg.fanout)
    _, _, off_L = rg.rg_schedule_frontier(s, s.L)
    rows_per_epoch = int(off_L[-1])
    m_max = int(np.diff(off_L).max())
    c = rg.rg_build_cache([s], feat_hbm, W.K)
    stats = [rg.rg_gather_batch(s, c, feat_hbm, b, torch.empty(m_max * W.stride_bytes, dtype=torch.uint8, device="cuda"),
                                out_stride=W.stride_bytes, out_capacity_rows=m_max) for b in (0,)]
    view = rg.rg_cache_view(c, W.n_nodes)
    k_eff = view["K_eff"]
    n_batches = s.n_batches
    # how the epoch's accesses to remote features are distributed, and what the cache saves (reported, not timed)
    remote_freq = view["freq"][~W.is_local.bool()]
    touched = remote_freq[remote_freq > 0]
    cls = [rg.rg_classify_batch(s, c, feat_hbm, b) for b in range(n_batches)]
    remote_rows = sum(x["n_hit"] + x["n_miss"] for x in cls)
    fetched_rows = sum(x["n_miss"] for x in cls)
    access_stats = {
        "touched_remote_nodes": int(touched.numel()),
        "share_accessed_once": float((touched == 1).sum().item()) / max(1, touched.numel()),
        "max_frequency": int(touched.max().item()) if touched.numel() else 0,
        "remote_rows_in_input_sets": int(remote_rows), "remote_rows_fetched_with_cache": int(fetched_rows),
        "fetch_reduction": remote_rows / fetched_rows if fetched_rows else None,
        "note": "context, not parity: the paper's Evaluation section reports 45.3 % of nodes accessed exactly once and a maximum "
                "frequency of 66 for an OGBN-Products epoch, and 9.70-15.39x less time in remote fetches (a time ratio on other "
                "graphs and machines; this is a row-count ratio on the synthetic graph)"}
    del view, remote_freq, touched
    del s, c
    sampled_edges = sum(h["sampled"] for h in hops)
    G = args.gather_group
    if G <= 0:      # small batches: more of them per launch, so that a launch is long enough to run at the memory system's rate
        G = 8
        while G < 64 and G < n_batches and rows_per_epoch / n_batches * G * W.stride_bytes < (512 << 20):
            G *= 2
    if G > 1:       # the staging buffer holds the largest group of G consecutive batches
        m_max = max(int(off_L[min(b + G, n_batches)] - off_L[b]) for b in range(0, n_batches, G))
    out_buf = torch.empty(m_max * W.stride_bytes, dtype=torch.uint8, device="cuda")
    log(f"[bench] {n_batches} batches, {sampled_edges} sampled edges/epoch, {rows_per_epoch} gathered rows/epoch, K_eff={k_eff}, batch0 {stats[0]}")

    rg.rg_profile_enable(True)
    dt, prof = timed(rg, W, feat_hbm, out_buf, W.stride_bytes, m_max, side, args.steps, args.warmup, G)
    ms_per_step = dt / args.steps * 1e3
    value = sampled_edges * args.steps / dt
    log(f"[bench] HBM-resident: {ms_per_step:.2f} ms/step; kernel groups: " +
        ", ".join(f"{k}={v['ms'] / args.steps:.2f}ms/{v['launches'] // args.steps}" for k, v in prof.items()))

    # roofline of the dominant kernel (by device time)
    samp_ms = prof["sampler"]["ms"] / args.steps
    gath_ms = (prof["gather"]["ms"] + prof["gather_miss"]["ms"]) / args.steps
    samp_bytes = sum(h["bytes"] for h in hops)
    gath_bytes = accounting.gather_traffic_bytes(rows_per_epoch, W.row_bytes)
    samp_gbps = samp_bytes / (samp_ms * 1e-3) / 1e9 if samp_ms > 0 else 0.0
    gath_gbps = gath_bytes / (gath_ms * 1e-3) / 1e9 if gath_ms > 0 else 0.0
    dominant = max(prof.items(), key=lambda kv: kv[1]["ms"])[0]
    if dominant in ("gather", "gather_miss"):
        roof = dict(kernel="gather_rows_kernel", bound="hbm", achieved=gath_gbps, peak=HBM_PEAK_GBPS, unit="GB/s",
                    frac=gath_gbps / HBM_PEAK_GBPS, traffic=None,
                    launches_per_step=(prof["gather"]["launches"] + prof["gather_miss"]["launches"]) // args.steps,
                    avg_launch_ms=gath_ms / max(1, (prof["gather"]["launches"] + prof["gather_miss"]["launches"]) // args.steps),
                    algorithmic_bytes_per_step=gath_bytes)
    else:
        roof = dict(kernel="sample_kernel", bound="hbm", achieved=samp_gbps, peak=HBM_PEAK_GBPS, unit="GB/s",
                    frac=samp_gbps / HBM_PEAK_GBPS, traffic=None,
                    launches_per_step=prof["sampler"]["launches"] // args.steps,
                    avg_launch_ms=samp_ms / max(1, prof["sampler"]["launches"] // args.steps),
                    algorithmic_bytes_per_step=samp_bytes)
    roof["dominant_group_by_time"] = dominant
    roof["traffic"] = measured_traffic(cfg.name, roof["kernel"])
    copy_gbps = device_copy_gbps()
    roof["device_copy_GBps"] = copy_gbps                       # a 1 GiB device-to-device copy on this machine, read + write
    roof["achieved_over_device_copy"] = roof["achieved"] / copy_gbps
    log(f"[bench] plain device-to-device copy of 1 GiB: {copy_gbps:.0f} GB/s read+write; {roof['kernel']} reaches {roof['achieved']:.0f} GB/s")

    result = {
        "metric": METRIC, "value": value, "unit": "sampled edges/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u32",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {W.n_nodes} nodes, {W.indices.numel()} edges (Chung-Lu, exponent {cfg.gamma}), "
                               f"{cfg.feat_dtype} features dim {cfg.feat_dim}, fanout {cfg.fanout}, batch {cfg.batch_size}, "
                               f"{cfg.n_train} train nodes, K={W.K}, remote table in HBM, {G} batch(es) per gather launch",
                   "n_batches": n_batches, "sampled_edges_per_epoch": sampled_edges, "gathered_rows_per_epoch": rows_per_epoch,
                   "K_eff": int(k_eff)},
        "roofline": roof,
        "access_stats": access_stats,
        "sampler": {"edges_per_s_kernel": sampled_edges / (samp_ms * 1e-3) if samp_ms else None, "GBps": samp_gbps,
                    "frac_hbm": samp_gbps / HBM_PEAK_GBPS, "ms_per_step": samp_ms, "scanned_row_entries": sum(h["sum_deg"] for h in hops)},
        "gather": {"GBps": gath_gbps, "frac_hbm": gath_gbps / HBM_PEAK_GBPS, "ms_per_step": gath_ms,
                   "delivered_GBps": rows_per_epoch * W.row_bytes / (gath_ms * 1e-3) / 1e9 if gath_ms else None},
        "kernel_ms_per_step": {k: v["ms"] / args.steps for k, v in prof.items()},
    }

    if not args.no_pcie_pass:
        remote_pinned = synth.pinned_copy(W.remote_rows)
        feat_pin = rg.make_features(W.is_local, W.row_of, W.local_rows, remote_pinned, W.row_bytes)
        steps2 = max(1, min(args.steps, 2))
        dt2, prof2 = timed(rg, W, feat_pin, out_buf, W.stride_bytes, m_max, side, steps2, 1, G)
        miss_ms = prof2["gather_miss"]["ms"] / steps2
        fill_ms = prof2["cache_fill"]["ms"] / steps2
        result["pcie_inclusive"] = {"value": sampled_edges * steps2 / dt2, "unit": "sampled edges/s", "ms_per_step": dt2 / steps2 * 1e3,
                                    "steps": steps2, "miss_pull_ms_per_step": miss_ms, "cache_fill_ms_per_step": fill_ms,
                                    "note": "remote feature table in pinned host memory; misses and the cache fill cross the host link"}
        log(f"[bench] pinned-host remote table: {dt2 / steps2 * 1e3:.2f} ms/step (miss pull {miss_ms:.2f} ms, cache fill {fill_ms:.2f} ms)")
    if not args.no_runtime_leg:
        result["runtime"] = runtime_leg(rg, W, feat_hbm)
        log(f"[bench] runtime leg: {result['runtime']}")
    rg.rg_profile_enable(False)
    if not args.no_runtime_leg:
        result["overlapped"] = overlapped_leg(rg, W, feat_hbm, W.stride_bytes, group=G)
        log(f"[bench] overlapped epochs: {result['overlapped']}")

    if args.pmc_probe:
        a = torch.ones(1 << 28, dtype=torch.int32, device="cuda")
        b = torch.empty_like(a)
        torch.add(a, 1, out=b)
        torch.cuda.synchronize()
        log("[bench] pmc probe: one elementwise kernel read 1 GiB and wrote 1 GiB")

    if not args.no_cpu_baseline:
        t0 = time.perf_counter()
        result["cpu_baseline"] = cpu_baseline(W, W.indptr.cpu().numpy(), W.indices.cpu().numpy(), W.train.cpu().numpy())
        log(f"[bench] cpu baseline took {time.perf_counter() - t0:.1f} s: {result['cpu_baseline']}")
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
