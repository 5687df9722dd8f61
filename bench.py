"""Benchmark of the RapidGNN data path on one MI355X.

One step = one pass of the whole hot path over one epoch of one synthetic
workload: rg_build_schedule (seeds, shuffle, every hop's sampling and
frontiers), rg_build_cache (tally, TopHot, VectorPull, plans) and the feature
block of every batch of the epoch (rg_gather_batches).  The default workload is
the largest configuration, partition_share: one worker's share of the
OGBN-Papers100M-shaped graph.

Prints ONE JSON line.
  value           sampled edges per second over whole steps, every input resident in HBM when the timed region
                  starts, the library's event timers OFF
  roofline        the kernel group with the most device time, from a second pass of the same steps with the
                  library's per-launch HIP event timers ON (they cost a little, so they stay out of `value`); for the
                  sampler the bound it sits closer to: HBM by the bytes that moved, or the vector unit's integer rate
  pcie_inclusive  the same steps with the remote feature table in pinned host memory -- the configuration's own
                  placement: VectorPull and every miss cross the host link (reported, never `value`)
  cpu_baseline    the CPU oracle on a bounded prefix of the epoch, per call, on one thread and on all cores
  other_workloads the remaining configurations, briefly (value, step time, sampler and gather rates)
Gathers stage --gather-group batches per launch (default, accounting.gather_group: the whole epoch if its feature
blocks together stay under 4 GiB, else the next eight batches back to back in one staging buffer, more, up to 64,
while that would be less than 512 MiB per launch).
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
HEADLINE = "partition_share"


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
    """W warm-up steps, then exactly `steps` steps between two device-wide synchronisations."""
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
    """E epochs end to end with the precompute of epoch e+1 (schedule, tally, TopHot, cache, plan) running on a
    second host thread and stream beside the gathers of epoch e, as Alg. 1 arranges it.  Every epoch's whole hot
    path runs inside the timed region."""
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
        del s, c                                        # (released behind the epoch's gathers; nothing waits here)
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


def cpu_model_string():
    """The first processor's entry of /proc/cpuinfo: model name with vendor, family, model and stepping numbers."""
    want = ("vendor_id", "model name", "cpu family", "model", "stepping")
    got = {}
    try:
        with open("/proc/cpuinfo") as fh:
            for ln in fh:
                if ":" not in ln:
                    if got:
                        break
                    continue
                k, v = (x.strip() for x in ln.split(":", 1))
                if k in want and k not in got:
                    got[k] = v
    except OSError:
        pass
    if not got:
        return ""
    return (f"{got.get('model name', '?')} ({got.get('vendor_id', '?')}, family {got.get('cpu family', '?')}, model {got.get('model', '?')}, "
            f"stepping {got.get('stepping', '?')})")


def cpu_baseline(W, remote_host, budget_s=10.0):
    """The oracle, as it stands, timed per call on a bounded prefix of the epoch's batches: once on one thread and
    once on all cores the process may use (the schedule: one batch per thread; the gathers: one batch per thread;
    the tally, TopHot and cache fill between them are serial code in the oracle and take the same time in both).
    remote_host: a host copy of the remote feature table as a numpy byte array."""
    import concurrent.futures as cf
    import oracle
    cfg = W.cfg
    try:
        nproc = len(os.sched_getaffinity(0))
    except AttributeError:
        nproc = os.cpu_count() or 1
    cores = max(1, min(nproc, oracle.max_threads(), 16))      # (the GPU machine gives a job 16 CPUs, whatever nproc says)
    indptr_h, indices_h, train_h = W.indptr.cpu().numpy(), W.indices.cpu().numpy(), W.train.cpu().numpy()
    feats = oracle.Features(W.is_local.cpu().numpy(), W.row_of.cpu().numpy(),
                            W.local_rows.contiguous().view(torch.uint8).cpu().numpy(), W.stride_bytes,
                            remote_host, W.stride_bytes, W.row_bytes)
    beta = accounting.batches_per_epoch(cfg.n_train, cfg.batch_size)

    def one(nb, threads):
        t0 = time.perf_counter()
        s = oracle.Schedule(indptr_h, indices_h, train_h, cfg.batch_size, cfg.fanout, cfg.s0, cfg.worker, cfg.epoch,
                            batch_lo=0, batch_hi=nb, n_threads=threads)
        t1 = time.perf_counter()
        freq = oracle.frequency([s], W.n_nodes)
        ids, _ = oracle.top_hot(freq, feats.is_local, W.K)
        oracle.cache_fill(ids, feats, table_stride=W.stride_bytes)
        t2 = time.perf_counter()
        if threads == 1:
            for b in range(s.n_batches):
                oracle.gather_batch(s, b, feats, out_stride=W.stride_bytes)
        else:                              # the same call, one batch per thread (the library call releases the interpreter lock)
            with cf.ThreadPoolExecutor(max_workers=threads) as pool:
                list(pool.map(lambda b: oracle.gather_batch(s, b, feats, out_stride=W.stride_bytes).shape, range(s.n_batches)))
        t3 = time.perf_counter()
        edges = sum(int(s.samples(h)[1].size) for h in range(s.L))
        return dict(batches=nb, threads=threads, sampled_edges=edges, seconds=round(t3 - t0, 3),
                    build_schedule_s=round(t1 - t0, 3), build_cache_s=round(t2 - t1, 3), gather_epoch_s=round(t3 - t2, 3),
                    edges_per_s=edges / (t3 - t0))

    probe = one(1, 1)                                            # one batch on one thread sizes both samples
    per_batch = max(probe["seconds"], 1e-3)
    nb1 = int(max(1, min(beta, budget_s / per_batch)))
    single = one(nb1, 1)
    nb_all = int(max(cores, min(beta, cores * budget_s / per_batch)))
    nb_all = min(beta, nb_all // cores * cores if nb_all >= cores else nb_all)
    allc = one(nb_all, cores)
    return dict(value=allc["edges_per_s"], unit="sampled edges/s", cores=cores, kind="oracle",
                sample=f"first {nb_all} of {beta} batches of the {cfg.name} epoch on {cores} threads ({allc['seconds']} s): build_schedule "
                       f"(one batch per thread), build_cache (tally, TopHot, cache fill: serial code), every batch's gather (one batch per "
                       f"thread); beside it the first {nb1} batches on one thread ({single['seconds']} s)",
                all_cores=allc, single_thread=single, nproc=nproc, host_cpus=os.cpu_count(), cpu_model=cpu_model_string())


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


def stored_traffic(workload, kernel):
    """HBM bytes per step of `kernel` on `workload` as counted by separate rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of
    this script (profiles/measured_traffic.json; the profiles/*_traffic.md files give the commands and the calibration).
    A stored measurement, not one of this run: a process cannot read those counters for itself.  None if never taken."""
    try:
        with open(os.path.join(ROOT, "profiles", "measured_traffic.json")) as fh:
            return json.load(fh).get(f"{workload}:{kernel}")
    except (OSError, ValueError):
        return None


def group_rate(ms, n_bytes):
    gbps = n_bytes / (ms * 1e-3) / 1e9 if ms > 0 else 0.0
    return gbps, gbps / HBM_PEAK_GBPS


def measure(rg, name, args, full):
    """One workload: generation, one untimed pass for sizes, the timed steps with the event timers off (`value`) and a
    second pass with them on (per-kernel-group device time).  full: also the access statistics, the pinned-host
    pass, the runtime legs and the CPU baseline."""
    cfg = synth.CONFIGS[name]
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
    view = rg.rg_cache_view(c, W.n_nodes)
    k_eff = view["K_eff"]
    n_batches = s.n_batches
    access_stats = None
    if full:     # how the epoch's accesses to remote features are distributed, and what the cache saves (reported, not timed)
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
        del remote_freq, touched
    del view, s, c
    sampled_edges = sum(h["sampled"] for h in hops)
    G = args.gather_group
    if G <= 0:      # small batches: more of them per launch, so that a launch is long enough to run at the memory system's rate
        G = accounting.gather_group(n_batches, rows_per_epoch, W.stride_bytes)
    if G > 1:       # the staging buffer holds the largest group of G consecutive batches
        m_max = max(int(off_L[min(b + G, n_batches)] - off_L[b]) for b in range(0, n_batches, G))
    out_buf = torch.empty(m_max * W.stride_bytes, dtype=torch.uint8, device="cuda")
    log(f"[bench] {n_batches} batches, {sampled_edges} sampled edges/epoch, {rows_per_epoch} gathered rows/epoch, K_eff={k_eff}, "
        f"{G} batch(es) per gather launch")

    steps, warmup = (args.steps, args.warmup) if full else (min(args.steps, 3), 1)
    # ---- the headline: event timers off
    rg.rg_profile_enable(False)
    dt, _ = timed(rg, W, feat_hbm, out_buf, W.stride_bytes, m_max, side, steps, warmup, G)
    ms_per_step = dt / steps * 1e3
    value = sampled_edges * steps / dt
    # ---- the same steps again with the per-launch event timers on: device time per kernel group
    rg.rg_profile_enable(True)
    dt_prof, prof = timed(rg, W, feat_hbm, out_buf, W.stride_bytes, m_max, side, steps, 1, G)
    rg.rg_profile_enable(False)
    log(f"[bench] {cfg.name}, HBM-resident: {ms_per_step:.2f} ms/step with the event timers off, {dt_prof / steps * 1e3:.2f} with them on; kernel groups: " +
        ", ".join(f"{k}={v['ms'] / steps:.2f}ms/{v['launches'] // steps}" for k, v in prof.items() if v["launches"]))

    samp_ms = prof["sampler"]["ms"] / steps
    gath_ms = (prof["gather"]["ms"] + prof["gather_miss"]["ms"]) / steps
    samp_bytes = sum(h["bytes"] for h in hops)
    gath_bytes = accounting.gather_traffic_bytes(rows_per_epoch, W.row_bytes)
    samp_gbps, samp_frac = group_rate(samp_ms, samp_bytes)
    gath_gbps, gath_frac = group_rate(gath_ms, gath_bytes)
    samp_launches = max(1, prof["sampler"]["launches"] // steps)
    gath_launches = max(1, (prof["gather"]["launches"] + prof["gather_miss"]["launches"]) // steps)
    scanned = sum(h["sum_deg"] for h in hops)
    result = {
        "value": value, "unit": "sampled edges/s", "steps": steps, "warmup": warmup, "ms_per_step": ms_per_step,
        "ms_per_step_with_event_timers": dt_prof / steps * 1e3,
        "config": {"workload": f"{cfg.name}: {W.n_nodes} nodes, {W.indices.numel()} edges (Chung-Lu, exponent {cfg.gamma}), "
                               f"{cfg.feat_dtype} features dim {cfg.feat_dim}, fanout {cfg.fanout}, batch {cfg.batch_size}, "
                               f"{cfg.n_train} train nodes, K={W.K}, every input in HBM for `value` (remote table in pinned host memory: "
                               f"see pcie_inclusive), {G} batch(es) per gather launch",
                   "n_batches": n_batches, "sampled_edges_per_epoch": sampled_edges, "gathered_rows_per_epoch": rows_per_epoch,
                   "K_eff": int(k_eff)},
        "sampler": {"kernel": "sample_kernel", "edges_per_s_kernel": sampled_edges / (samp_ms * 1e-3) if samp_ms else None, "GBps": samp_gbps,
                    "frac_hbm": samp_frac, "ms_per_step": samp_ms, "launches_per_step": samp_launches,
                    "algorithmic_bytes_per_step": samp_bytes, "scanned_row_entries": scanned,
                    "int_ops_per_step": accounting.sampler_int_ops(scanned),
                    "TOPps": accounting.sampler_int_ops(scanned) / (samp_ms * 1e-3) / 1e12 if samp_ms else None,
                    "frac_alu": accounting.sampler_int_ops(scanned) / (samp_ms * 1e-3) / 1e12 / accounting.INT32_VECTOR_PEAK_TOPS if samp_ms else None},
        "gather": {"kernel": "gather_rows_kernel", "GBps": gath_gbps, "frac_hbm": gath_frac, "ms_per_step": gath_ms,
                   "launches_per_step": gath_launches, "algorithmic_bytes_per_step": gath_bytes,
                   "delivered_GBps": rows_per_epoch * W.row_bytes / (gath_ms * 1e-3) / 1e9 if gath_ms else None},
        "kernel_ms_per_step": {k: v["ms"] / steps for k, v in prof.items()},
    }
    for key in ("sampler", "gather"):            # HBM bytes as the counters saw them, where they have been taken
        rec = stored_traffic(cfg.name, result[key]["kernel"])
        if rec:
            result[key]["traffic_per_step"] = rec["hbm_bytes_per_step"]
            result[key]["traffic_over_algorithmic"] = rec["hbm_bytes_per_step"] / result[key]["algorithmic_bytes_per_step"]
    if not full:
        del out_buf, feat_hbm, W
        torch.cuda.empty_cache()
        return result

    # ---- roofline of the dominant kernel group (by device time)
    dominant = max(prof.items(), key=lambda kv: kv[1]["ms"])[0]
    key = "gather" if dominant in ("gather", "gather_miss") else "sampler"
    g = result[key]
    launches = g["launches_per_step"]
    roof = dict(kernel=g["kernel"], bound="hbm", achieved=g["GBps"], peak=HBM_PEAK_GBPS, unit="GB/s", frac=g["frac_hbm"],
                traffic=None, launches_per_step=launches, avg_launch_ms=g["ms_per_step"] / launches,
                algorithmic_bytes_per_launch=g["algorithmic_bytes_per_step"] / launches,
                algorithmic_bytes_per_step=g["algorithmic_bytes_per_step"], dominant_group_by_time=dominant)
    if "traffic_per_step" in g:
        roof["traffic"] = g["traffic_per_step"] / launches                      # per launch, like `achieved`
        roof["traffic_per_step"] = g["traffic_per_step"]
        roof["traffic_over_algorithmic"] = g["traffic_over_algorithmic"]
        roof["traffic_source"] = ("stored: separate rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command "
                                  "(profiles/measured_traffic.json), not read in this run")
    if key == "sampler":
        # The sampler reads a hub's row once per batch that holds the hub, and hands those reads out so that they meet in
        # the caches: its HBM traffic can then be a fraction of its algorithmic bytes, and its algorithmic bytes per
        # second can pass the HBM peak.  Whichever of its two bounds it sits closer to is the one reported: HBM by the
        # bytes that really moved (the stored counter figure; the algorithmic bytes where none is stored), or the vector
        # unit's integer rate by the operations the keys need.
        hbm_bytes = g.get("traffic_per_step", g["algorithmic_bytes_per_step"])
        frac_hbm_moved = hbm_bytes / (g["ms_per_step"] * 1e-3) / 1e9 / HBM_PEAK_GBPS
        roof["hbm"] = {"algorithmic_GBps": g["GBps"], "algorithmic_frac": g["frac_hbm"], "moved_GBps": frac_hbm_moved * HBM_PEAK_GBPS,
                       "moved_frac": frac_hbm_moved}
        if g["frac_alu"] > frac_hbm_moved:
            roof.update(bound="alu", achieved=g["TOPps"], peak=accounting.INT32_VECTOR_PEAK_TOPS, unit="TOP/s", frac=g["frac_alu"],
                        int_ops_per_launch=g["int_ops_per_step"] / launches, int_ops_per_step=g["int_ops_per_step"],
                        int_ops_per_scanned_row_entry=accounting.SAMPLER_INT_OPS_PER_ENTRY)
    copy_gbps = device_copy_gbps()
    roof["device_copy_GBps"] = copy_gbps                       # a 1 GiB device-to-device copy on this machine, read + write
    roof["algorithmic_GBps_over_device_copy"] = g["GBps"] / copy_gbps
    log(f"[bench] plain device-to-device copy of 1 GiB: {copy_gbps:.0f} GB/s read+write; {roof['kernel']} reaches {g['GBps']:.0f} GB/s of algorithmic bytes"
        + (f", {roof['achieved']:.1f} of {roof['peak']:.1f} TOP/s of integer arithmetic" if roof["bound"] == "alu" else ""))
    result["roofline"] = roof
    result["access_stats"] = access_stats

    remote_pinned = None
    if not args.no_pcie_pass:
        t0 = time.perf_counter()
        remote_pinned = synth.pinned_copy(W.remote_rows)
        log(f"[bench] remote table ({remote_pinned.numel() * remote_pinned.element_size() / 1e9:.1f} GB) copied to pinned host memory in "
            f"{time.perf_counter() - t0:.1f} s")
        feat_pin = rg.make_features(W.is_local, W.row_of, W.local_rows, remote_pinned, W.row_bytes)
        steps2 = max(1, min(args.steps, 2))
        rg.rg_profile_enable(True)
        dt2, prof2 = timed(rg, W, feat_pin, out_buf, W.stride_bytes, m_max, side, steps2, 1, G)
        rg.rg_profile_enable(False)
        miss_ms = prof2["gather_miss"]["ms"] / steps2
        fill_ms = prof2["cache_fill"]["ms"] / steps2
        result["pcie_inclusive"] = {"value": sampled_edges * steps2 / dt2, "unit": "sampled edges/s", "ms_per_step": dt2 / steps2 * 1e3,
                                    "steps": steps2, "miss_pull_ms_per_step": miss_ms, "cache_fill_ms_per_step": fill_ms,
                                    "cache_fill_bytes": int(k_eff) * W.row_bytes,
                                    "cache_fill_GBps": int(k_eff) * W.row_bytes / (fill_ms * 1e-3) / 1e9 if fill_ms else None,
                                    "note": "remote feature table in pinned host memory (the configuration's own placement); the cache fill "
                                            "(VectorPull) and every miss (SyncPull) cross the host link"}
        log(f"[bench] pinned-host remote table: {dt2 / steps2 * 1e3:.2f} ms/step (miss pull {miss_ms:.2f} ms, cache fill {fill_ms:.2f} ms)")
        del feat_pin
    if not args.no_runtime_leg:
        rg.rg_profile_enable(True)
        result["runtime"] = runtime_leg(rg, W, feat_hbm)
        rg.rg_profile_enable(False)
        log(f"[bench] runtime leg: {result['runtime']}")
        result["overlapped"] = overlapped_leg(rg, W, feat_hbm, W.stride_bytes, group=G)
        log(f"[bench] overlapped epochs: {result['overlapped']}")

    if args.pmc_probe:
        a = torch.ones(1 << 28, dtype=torch.int32, device="cuda")
        b = torch.empty_like(a)
        torch.add(a, 1, out=b)
        torch.cuda.synchronize()
        del a, b
        log("[bench] pmc probe: one elementwise kernel read 1 GiB and wrote 1 GiB")

    if not args.no_cpu_baseline:
        t0 = time.perf_counter()
        if remote_pinned is not None:
            remote_host = remote_pinned.view(torch.uint8).numpy().reshape(-1)
        else:
            remote_host = W.remote_rows.contiguous().view(torch.uint8).cpu().numpy().reshape(-1)
        result["cpu_baseline"] = cpu_baseline(W, remote_host)
        log(f"[bench] cpu baseline took {time.perf_counter() - t0:.1f} s: {result['cpu_baseline']}")
    del out_buf, feat_hbm, W, remote_pinned
    torch.cuda.empty_cache()
    return result


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default=HEADLINE, choices=sorted(synth.CONFIGS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--gather-group", type=int, default=0,
                    help="batches whose feature blocks one gather launch stages back to back (rg_gather_batches, the prefetcher's Q); "
                         "1 = one launch per batch; 0 = the whole epoch if it stages under 4 GiB, else eight, doubled up to 64 while a launch would stage less than 512 MiB")
    ap.add_argument("--no-pcie-pass", action="store_true")
    ap.add_argument("--no-runtime-leg", action="store_true", help="skip the multi-epoch cache-pair / prefetch-queue / blocks leg")
    ap.add_argument("--no-other-workloads", action="store_true", help="skip the brief passes over the other configurations")
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
    main_result = measure(rg, args.workload, args, full=True)
    result = {"metric": METRIC, "value": main_result.pop("value"), "unit": main_result.pop("unit"), "n_gpus": 1,
              "steps": main_result.pop("steps"), "warmup": main_result.pop("warmup"), "ms_per_step": main_result.pop("ms_per_step"),
              "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u32", "data": "synthetic"}
    result.update(main_result)
    if not args.no_other_workloads:
        others = {}
        for name in ("tiny", "medium", "large_sparse", "fanout_stress", "partition_share"):
            if name == args.workload:
                continue
            rg.rg_trim_memory()
            r = measure(rg, name, args, full=False)
            others[name] = {"value": r["value"], "unit": r["unit"], "steps": r["steps"], "ms_per_step": r["ms_per_step"],
                            "workload": r["config"]["workload"], "sampler": r["sampler"], "gather": r["gather"]}
        result["other_workloads"] = others
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
