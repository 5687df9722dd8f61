"""GPU tests of the runtime around the three calls: the double-buffered cache (C_s / C_sec) and the
rolling prefetch queue of depth Q (Alg. 1, Sec. 3 "Rolling prefetch and execution"), against the oracle.

Every gathered byte must equal the oracle's whatever the pipeline state: staged or not, swapped or not."""
import numpy as np
import pytest
import torch

from paper_2509_05207_amd import synth
from test_gpu_parity import Case, assert_schedules_equal

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rg():
    from paper_2509_05207_amd import binding
    binding.lib()
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return binding


@pytest.fixture(scope="module", params=["small", "mid_bf16"])
def case(request, orc, rg):
    return Case(request.param, orc, rg, s0=11, worker=1, epoch=0, pinned_remote=(request.param == "small"))


def oracle_cache(orc, case, osched):
    w = case.w
    freq = orc.frequency([osched], w.n_nodes)
    ids, slot = orc.top_hot(freq, w.is_local.numpy(), w.K)
    return ids, slot


def slots_for(case, Q, out_stride):
    _, off = case.osched.input_nodes()
    m_max = int(np.diff(off).max())
    return [torch.full(((m_max + 1) * out_stride,), 0xCD, dtype=torch.uint8, device="cuda") for _ in range(Q)], m_max


@pytest.mark.parametrize("Q", [1, 3, 64])
def test_prefetch_queue_delivers_every_batch_in_order(case, rg, orc, Q):
    w = case.w
    out_stride = (w.row_bytes + 15) // 16 * 16
    cache = rg.rg_build_cache([case.gsched], case.gfeat, w.K)
    _, slot = oracle_cache(orc, case, case.osched)
    slots, m_max = slots_for(case, Q, out_stride)
    pf = rg.rg_prefetcher_create(case.gsched, cache, case.gfeat, slots, out_stride=out_stride, slot_capacity_rows=m_max + 1)
    nb = case.gsched.n_batches
    consumer = torch.cuda.Stream()
    for b in range(nb):
        issued = rg.rg_prefetcher_fill(pf)
        staged, held = rg.rg_prefetcher_depth(pf)
        assert held == 0 and staged == min(Q, nb - b), "back-pressure: the queue holds min(Q, remaining) batches"
        assert issued == (min(Q, nb) if b == 0 else (1 if b + Q <= nb else 0))
        got_b, buf, st, was_staged = rg.rg_prefetcher_acquire(pf, stream=consumer)
        assert got_b == b and was_staged
        with torch.cuda.stream(consumer):
            block = buf.clone()                  # the consumer's use of the slot, ordered on its own stream
        rg.rg_prefetcher_release(pf, stream=consumer)
        consumer.synchronize()
        ref = orc.gather_batch(case.osched, b, case.ofeat, out_stride=out_stride, fill=0xCD)
        m = ref.shape[0]
        assert np.array_equal(block.cpu().numpy().reshape(-1, out_stride)[:m, :w.row_bytes], ref[:, :w.row_bytes]), f"batch {b}"
        assert st == orc.batch_stats(case.osched, b, w.is_local.numpy(), slot)
    with pytest.raises(rg.RgError) as e:
        rg.rg_prefetcher_acquire(pf)
    assert e.value.status == rg.RG_ERANGE


def test_unstaged_batches_take_the_default_path(case, rg, orc):
    """The consumer overtakes the prefetcher: the batch is gathered on the spot, same bytes (Sec. 3, race)."""
    w = case.w
    out_stride = w.row_bytes
    cache = rg.rg_build_cache([case.gsched], case.gfeat, w.K)
    slots, m_max = slots_for(case, 2, out_stride)
    pf = rg.rg_prefetcher_create(case.gsched, cache, case.gfeat, slots, out_stride=out_stride, slot_capacity_rows=m_max + 1)
    nb = case.gsched.n_batches
    flags = []
    for b in range(nb):
        if b % 3 == 1:
            rg.rg_prefetcher_fill(pf)            # only now and then: some batches arrive staged, others do not
        got_b, buf, st, was_staged = rg.rg_prefetcher_acquire(pf)
        flags.append(was_staged)
        torch.cuda.synchronize()
        ref = orc.gather_batch(case.osched, b, case.ofeat, out_stride=out_stride, fill=0xCD)
        m = ref.shape[0]
        assert got_b == b
        assert np.array_equal(buf.cpu().numpy().reshape(-1, out_stride)[:m], ref), f"batch {b}"
        rg.rg_prefetcher_release(pf)
    assert not flags[0] and any(flags) and not all(flags)


def test_holding_more_than_q_slots_is_refused(case, rg):
    w = case.w
    slots, m_max = slots_for(case, 2, w.row_bytes)
    pf = rg.rg_prefetcher_create(case.gsched, None, case.gfeat, slots, out_stride=w.row_bytes, slot_capacity_rows=m_max + 1)
    if case.gsched.n_batches < 3:
        pytest.skip("needs three batches")
    rg.rg_prefetcher_acquire(pf)
    rg.rg_prefetcher_acquire(pf)
    with pytest.raises(rg.RgError) as e:
        rg.rg_prefetcher_acquire(pf)
    assert e.value.status == rg.RG_EINVAL
    assert rg.rg_prefetcher_fill(pf) == 0                      # nothing can be staged while both slots are held
    rg.rg_prefetcher_release(pf)
    assert rg.rg_prefetcher_fill(pf) == 1
    torch.cuda.synchronize()
    rg.rg_prefetcher_release(pf)
    with pytest.raises(rg.RgError):
        rg.rg_prefetcher_release(pf)                           # nothing is held any more


def test_slots_smaller_than_the_largest_batch_are_refused(case, rg):
    w = case.w
    slots, m_max = slots_for(case, 2, w.row_bytes)
    with pytest.raises(rg.RgError) as e:
        rg.rg_prefetcher_create(case.gsched, None, case.gfeat, slots, out_stride=w.row_bytes, slot_capacity_rows=m_max - 1)
    assert e.value.status == rg.RG_ERANGE


def test_double_buffered_cache_follows_the_epochs(case, rg, orc):
    """C_sec built from B_{e+1} while epoch e gathers; after the swap it equals the oracle's cache of epoch e+1."""
    w = case.w
    n_epochs = 3
    osch = [case.osched] + [orc.Schedule(w.indptr.numpy(), w.indices.numpy(), w.train.numpy(), w.cfg.batch_size, w.cfg.fanout,
                                         case.s0, case.worker, e, n_threads=8) for e in range(1, n_epochs)]
    gsch = [case.gsched] + [rg.rg_build_schedule(case.indptr, case.indices, case.train, w.cfg.batch_size, w.cfg.fanout,
                                                 case.s0, case.worker, e) for e in range(1, n_epochs)]
    out_stride = w.row_bytes
    _, off = case.osched.input_nodes()
    m_cap = max(int(np.diff(o.input_nodes()[1]).max()) for o in osch)
    out = torch.empty(m_cap * out_stride, dtype=torch.uint8, device="cuda")
    pair = rg.rg_cache_pair_create(gsch[0], case.gfeat, w.K)
    table_stride = (w.row_bytes + 15) // 16 * 16
    for e in range(n_epochs):
        ids, slot = oracle_cache(orc, case, osch[e])
        cur = rg.rg_cache_pair_primary(pair)
        v = rg.rg_cache_view(cur, w.n_nodes)
        assert np.array_equal(v["cache_ids"].cpu().numpy(), ids), f"epoch {e}: C_s is not the top-K of this epoch's schedule"
        if e + 1 < n_epochs:
            rg.rg_cache_pair_begin_next(pair, gsch[e + 1])     # runs beside the gathers below
        for b in range(gsch[e].n_batches):
            out.fill_(0xCD)
            st = rg.rg_gather_batch(gsch[e], cur, case.gfeat, b, out, out_stride=out_stride, out_capacity_rows=m_cap)
            torch.cuda.synchronize()
            ref = orc.gather_batch(osch[e], b, case.ofeat, out_stride=out_stride, fill=0xCD)
            assert np.array_equal(out.cpu().numpy().reshape(m_cap, out_stride)[:ref.shape[0]], ref), f"epoch {e} batch {b}"
            assert st == orc.batch_stats(osch[e], b, w.is_local.numpy(), slot)
            assert rg.rg_cache_pair_table_bytes(pair) <= 2 * w.K * table_stride, "memory bound 2 * n_hot * d"
        if e + 1 < n_epochs:
            assert rg.rg_cache_pair_swap(pair, wait=True)
    assert not rg.rg_cache_pair_swap(pair, wait=True)          # nothing pending: C_s stays


def test_swap_while_staged_gathers_are_in_flight(case, rg, orc):
    """The swap at the epoch boundary releases the old C_s without draining the device: blocks that the prefetcher
    staged from it just before -- their kernels possibly still running -- must arrive intact, and the memory bound
    counts the table that is being built."""
    w = case.w
    o1 = orc.Schedule(w.indptr.numpy(), w.indices.numpy(), w.train.numpy(), w.cfg.batch_size, w.cfg.fanout, case.s0, case.worker, 1,
                      n_threads=8)
    g1 = rg.rg_build_schedule(case.indptr, case.indices, case.train, w.cfg.batch_size, w.cfg.fanout, case.s0, case.worker, 1)
    out_stride = (w.row_bytes + 15) // 16 * 16
    Q = min(3, case.gsched.n_batches)
    slots, m_max = slots_for(case, Q, out_stride)
    _, slot0 = oracle_cache(orc, case, case.osched)
    ids1, _ = oracle_cache(orc, case, o1)
    for _ in range(3):                                           # several boundaries in a row, memory reused in between
        pair = rg.rg_cache_pair_create(case.gsched, case.gfeat, w.K)
        pf = rg.rg_prefetcher_create(case.gsched, rg.rg_cache_pair_primary(pair), case.gfeat, slots, out_stride=out_stride,
                                     slot_capacity_rows=m_max + 1)
        rg.rg_cache_pair_begin_next(pair, g1)
        assert rg.rg_prefetcher_fill(pf) == Q                    # Q gathers enqueued from the old C_s ...
        assert rg.rg_cache_pair_swap(pair, wait=True)            # ... and the old C_s is released under them
        assert rg.rg_cache_pair_table_bytes(pair) <= 2 * w.K * out_stride
        junk = rg.rg_build_cache([g1], case.gfeat, w.K)          # a build right behind the swap draws from the same block cache
        for b in range(Q):
            got_b, buf, st, was_staged = rg.rg_prefetcher_acquire(pf)
            assert got_b == b and was_staged
            torch.cuda.current_stream().synchronize()
            ref = orc.gather_batch(case.osched, b, case.ofeat, out_stride=out_stride, fill=0xCD)
            assert np.array_equal(buf.cpu().numpy().reshape(-1, out_stride)[:ref.shape[0], :w.row_bytes], ref[:, :w.row_bytes]), f"batch {b}"
            assert st == orc.batch_stats(case.osched, b, w.is_local.numpy(), slot0)
            rg.rg_prefetcher_release(pf)
        v = rg.rg_cache_view(rg.rg_cache_pair_primary(pair), w.n_nodes)
        assert np.array_equal(v["cache_ids"].cpu().numpy(), ids1)
        del pf, junk, pair, v


def test_an_unswapped_cache_still_serves_the_next_epoch_exactly(case, rg, orc):
    """The secondary cache is not ready at the boundary (Alg. 1's swap is conditional): the old C_s serves epoch e+1;
    hits are those of the old cache, bytes are unchanged."""
    w = case.w
    o1 = orc.Schedule(w.indptr.numpy(), w.indices.numpy(), w.train.numpy(), w.cfg.batch_size, w.cfg.fanout, case.s0, case.worker, 1,
                      n_threads=8)
    g1 = rg.rg_build_schedule(case.indptr, case.indices, case.train, w.cfg.batch_size, w.cfg.fanout, case.s0, case.worker, 1)
    pair = rg.rg_cache_pair_create(case.gsched, case.gfeat, w.K)
    _, slot0 = oracle_cache(orc, case, case.osched)
    cur = rg.rg_cache_pair_primary(pair)                       # no begin_next: nothing to swap
    assert not rg.rg_cache_pair_swap(pair, wait=False)
    m_cap = int(np.diff(o1.input_nodes()[1]).max())
    out = torch.empty(m_cap * w.row_bytes, dtype=torch.uint8, device="cuda")
    for b in range(0, g1.n_batches, max(1, g1.n_batches // 4)):
        st = rg.rg_gather_batch(g1, cur, case.gfeat, b, out, out_stride=w.row_bytes, out_capacity_rows=m_cap)
        torch.cuda.synchronize()
        ref = orc.gather_batch(o1, b, case.ofeat, out_stride=w.row_bytes, fill=0xCD)
        assert np.array_equal(out.cpu().numpy().reshape(m_cap, w.row_bytes)[:ref.shape[0]], ref)
        assert st == orc.batch_stats(o1, b, w.is_local.numpy(), slot0)


def test_begin_next_twice_without_swap_replaces_the_pending_cache(case, rg, orc):
    w = case.w
    g1 = rg.rg_build_schedule(case.indptr, case.indices, case.train, w.cfg.batch_size, w.cfg.fanout, case.s0, case.worker, 1)
    g2 = rg.rg_build_schedule(case.indptr, case.indices, case.train, w.cfg.batch_size, w.cfg.fanout, case.s0, case.worker, 2)
    o2 = orc.Schedule(w.indptr.numpy(), w.indices.numpy(), w.train.numpy(), w.cfg.batch_size, w.cfg.fanout, case.s0, case.worker, 2,
                      n_threads=8)
    pair = rg.rg_cache_pair_create(case.gsched, case.gfeat, w.K)
    rg.rg_cache_pair_begin_next(pair, g1)
    while True:                                                # a second begin is refused while the first build runs
        try:
            rg.rg_cache_pair_begin_next(pair, g2)
            break
        except rg.RgError as e:
            assert e.status == rg.RG_EINVAL
    assert rg.rg_cache_pair_swap(pair, wait=True)
    ids, _ = oracle_cache(orc, case, o2)
    v = rg.rg_cache_view(rg.rg_cache_pair_primary(pair), w.n_nodes)
    assert np.array_equal(v["cache_ids"].cpu().numpy(), ids)


def test_classification_alone_matches_the_oracle_and_the_sweep_law(case, rg, orc):
    """rg_classify_batch: the counts of a gather without the copy, from the plan or on the fly; summed over an epoch
    they equal the oracle's for every cache size, and fall as the cache grows."""
    from paper_2509_05207_amd import sweep
    w = case.w
    is_local = w.is_local.numpy()
    freq = orc.frequency([case.osched], w.n_nodes)
    n_remote = int(((is_local == 0) & (freq > 0)).sum())
    o1 = orc.Schedule(w.indptr.numpy(), w.indices.numpy(), w.train.numpy(), w.cfg.batch_size, w.cfg.fanout, case.s0, case.worker, 1,
                      n_threads=8)
    g1 = rg.rg_build_schedule(case.indptr, case.indices, case.train, w.cfg.batch_size, w.cfg.fanout, case.s0, case.worker, 1)
    last = None
    for K in (0, 3, n_remote // 5, n_remote):
        _, slot = orc.top_hot(freq, is_local, K)
        c = rg.rg_build_cache([case.gsched], case.gfeat, K)
        total = 0
        for b in range(case.gsched.n_batches):
            st = rg.rg_classify_batch(case.gsched, c, case.gfeat, b)            # from the prepared plan
            assert st == orc.batch_stats(case.osched, b, is_local, slot)
            total += st["n_miss"]
        for b in range(g1.n_batches):
            assert rg.rg_classify_batch(g1, c, case.gfeat, b) == orc.batch_stats(o1, b, is_local, slot)   # on the fly
        assert last is None or total <= last
        last = total
    assert last == 0
    for b in range(0, case.gsched.n_batches, 3):
        assert rg.rg_classify_batch(case.gsched, None, case.gfeat, b) == orc.batch_stats(case.osched, b, is_local, None)

    # the sweep script's own figures for this workload, against the oracle
    class W:
        pass
    W.cfg, W.indptr, W.indices, W.train = w.cfg, case.indptr, case.indices, case.train
    W.is_local, W.row_of, W.local_rows, W.remote_rows = case.is_local, case.row_of, case.local_rows, case.remote_rows
    W.row_bytes, W.n_nodes = w.row_bytes, w.n_nodes
    res = sweep.sweep(rg, W, 2, [0.0, 0.25, 1.0], log=lambda *a: None)
    os_ = [orc.Schedule(w.indptr.numpy(), w.indices.numpy(), w.train.numpy(), w.cfg.batch_size, w.cfg.fanout, w.cfg.s0, w.cfg.worker,
                        w.cfg.epoch + e, n_threads=8) for e in range(2)]
    fr = [orc.frequency([o], w.n_nodes) for o in os_]
    nr = int(((is_local == 0) & (fr[0] > 0)).sum())
    assert res["n_remote_first_epoch"] == nr
    for row, frac in zip(res["rows"], (0.0, 0.25, 1.0)):
        K = int(round(frac * nr))
        assert row["K"] == K
        fresh = stale = 0
        slots = [orc.top_hot(f, is_local, K)[1] for f in fr]
        for e, o in enumerate(os_):
            fresh += sum(orc.batch_stats(o, b, is_local, slots[e])["n_miss"] for b in range(o.n_batches))
        stale = sum(orc.batch_stats(os_[1], b, is_local, slots[0])["n_miss"] for b in range(os_[1].n_batches))
        assert row["fetches_per_epoch"] == fresh / 2 and row["fetches_per_epoch_stale_cache"] == stale


@pytest.mark.parametrize("planned", [True, False])
def test_ranges_of_batches_gathered_back_to_back(case, rg, orc, planned):
    """rg_gather_batches: same bytes and stats as one call per batch, blocks packed at the schedule's row offsets."""
    w = case.w
    nb = case.gsched.n_batches
    cache = rg.rg_build_cache([case.gsched], case.gfeat, w.K) if planned else None
    _, slot = oracle_cache(orc, case, case.osched) if planned else (None, None)
    _, off = case.osched.input_nodes()
    out_stride = w.row_bytes + 4
    side = torch.cuda.Stream()
    for first, n in ((0, nb), (1, min(3, nb - 1)), (nb - 1, 1), (2, 0)):
        rows = int(off[first + n] - off[first])
        out = torch.full(((rows + 2) * out_stride,), 0xCD, dtype=torch.uint8, device="cuda")
        stats = rg.rg_gather_batches(case.gsched, cache, case.gfeat, first, n, out, out_stride=out_stride, out_capacity_rows=rows + 2,
                                     side_stream=side)
        torch.cuda.synchronize()
        got = out.cpu().numpy().reshape(rows + 2, out_stride)
        assert len(stats) == n
        for k in range(n):
            b = first + k
            ref = orc.gather_batch(case.osched, b, case.ofeat, out_stride=out_stride, fill=0xCD)
            at = int(off[b] - off[first])
            assert np.array_equal(got[at:at + ref.shape[0]], ref), f"range ({first}, {n}) batch {b}"
            assert stats[k] == orc.batch_stats(case.osched, b, w.is_local.numpy(), slot)
        assert np.all(got[rows:] == 0xCD), "rows beyond the range were written"
    with pytest.raises(rg.RgError) as e:
        rg.rg_gather_batches(case.gsched, cache, case.gfeat, nb - 1, 2, out, out_stride=out_stride, out_capacity_rows=10 ** 9)
    assert e.value.status == rg.RG_ERANGE
    small = torch.empty(8 * out_stride, dtype=torch.uint8, device="cuda")
    with pytest.raises(rg.RgError) as e:
        rg.rg_gather_batches(case.gsched, cache, case.gfeat, 0, nb, small, out_stride=out_stride, out_capacity_rows=8)
    assert e.value.status == rg.RG_ERANGE


def test_schedule_survives_a_round_trip_through_a_file(case, rg, orc, tmp_path, monkeypatch):
    """The metadata block on storage: saved, loaded into a new handle, equal to the oracle's schedule, and as good
    as the original for the cache, the plan, the gathers and the blocks."""
    w = case.w
    path = tmp_path / "epoch0.rgsched"
    rg.rg_schedule_save(case.gsched, path)
    # what the format says the file holds: header 32 bytes, then per hop offsets + ids (+ sample offsets + samples)
    want = 32
    for hop in range(case.osched.L + 1):
        ids, off = case.osched.frontier(hop)
        want += off.size * 8 + ids.size * 4
        if hop < case.osched.L:
            so, nb = case.osched.samples(hop)
            want += so.size * 8 + nb.size * 4
    assert path.stat().st_size == want
    g = rg.rg_schedule_load(path)
    from test_gpu_parity import assert_schedules_equal
    assert_schedules_equal(rg, g, case.osched)
    ids, slot = oracle_cache(orc, case, case.osched)
    freq = orc.frequency([case.osched], w.n_nodes)
    for tally in ("0", "1"):                                   # a loaded schedule carries no frequencies: the cache tallies its input lists, in words or in bytes
        monkeypatch.setenv("RAPIDGNN_NARROW_TALLY", tally)
        c = rg.rg_build_cache([g], case.gfeat, w.K)
        v = rg.rg_cache_view(c, w.n_nodes)
        assert np.array_equal(v["cache_ids"].cpu().numpy(), ids)
        assert np.array_equal(v["freq"].cpu().numpy().view(np.uint32), freq)
        assert np.array_equal(v["slot_of"].cpu().numpy(), slot)
    _, off = case.osched.input_nodes()
    rows = int(off[-1])
    out = torch.empty(rows * w.row_bytes, dtype=torch.uint8, device="cuda")
    stats = rg.rg_gather_batches(g, c, case.gfeat, 0, g.n_batches, out, out_stride=w.row_bytes, out_capacity_rows=rows)
    torch.cuda.synchronize()
    got = out.cpu().numpy().reshape(rows, w.row_bytes)
    for b in range(g.n_batches):
        ref = orc.gather_batch(case.osched, b, case.ofeat, out_stride=w.row_bytes, fill=0)
        assert np.array_equal(got[off[b]:off[b + 1]], ref)
        assert stats[b] == orc.batch_stats(case.osched, b, w.is_local.numpy(), slot)
    rg.rg_schedule_build_blocks(g)
    for hop in range(g.L):
        assert np.array_equal(rg.rg_schedule_block(g, hop).cpu().numpy(), case.osched.block(hop))


def test_an_epoch_streamed_from_its_file_range_by_range(case, rg, orc, tmp_path):
    """The metadata block streamed back piece by piece: every range of batches of the file equals the oracle's
    schedule of those batches alone, serves gathers with a cache of its own, and yields its computation blocks."""
    w = case.w
    path = tmp_path / "epoch.rgsched"
    rg.rg_schedule_save(case.gsched, path)
    nb = case.gsched.n_batches
    step = max(1, nb // 3)
    ranges = [(lo, min(step, nb - lo)) for lo in range(0, nb, step)] + [(nb - 1, 1), (0, nb), (1, 0), (nb, 0)]
    for lo, n in ranges:
        part = rg.rg_schedule_load_range(path, lo, n)
        assert part.n_batches == n and part.L == case.gsched.L
        if n == 0:
            continue
        o = orc.Schedule(w.indptr.numpy(), w.indices.numpy(), w.train.numpy(), w.cfg.batch_size, w.cfg.fanout, case.s0, case.worker, case.epoch,
                         batch_lo=lo, batch_hi=lo + n, n_threads=4)
        assert_schedules_equal(rg, part, o)
        rg.rg_schedule_build_blocks(part)
        for hop in range(o.L):
            assert np.array_equal(rg.rg_schedule_block(part, hop).cpu().numpy(), o.block(hop))
        cache = rg.rg_build_cache([part], case.gfeat, w.K)
        ids, slot = orc.top_hot(orc.frequency([o], w.n_nodes), w.is_local.numpy(), w.K)
        assert np.array_equal(rg.rg_cache_view(cache, w.n_nodes)["cache_ids"].cpu().numpy(), ids)
        _, off = o.input_nodes()
        rows = int(off[-1])
        out = torch.empty(max(rows, 1) * w.row_bytes, dtype=torch.uint8, device="cuda")
        stats = rg.rg_gather_batches(part, cache, case.gfeat, 0, n, out, out_stride=w.row_bytes, out_capacity_rows=rows)
        torch.cuda.synchronize()
        got = out.cpu().numpy()[: rows * w.row_bytes].reshape(rows, w.row_bytes)
        for b in range(n):
            ref = orc.gather_batch(o, b, case.ofeat, out_stride=w.row_bytes)
            assert np.array_equal(got[off[b]:off[b + 1]], ref), f"range ({lo}, {n}) batch {b}"
            assert stats[b] == orc.batch_stats(o, b, w.is_local.numpy(), slot)
    for lo, n in ((nb, 1), (0, nb + 1), (nb + 1, 0)):
        with pytest.raises(rg.RgError) as e:
            rg.rg_schedule_load_range(path, lo, n)
        assert e.value.status == rg.RG_ERANGE
    data = path.read_bytes()
    (tmp_path / "short").write_bytes(data[:-4])
    with pytest.raises(rg.RgError) as e:
        rg.rg_schedule_load_range(tmp_path / "short", 0, 1)
    assert e.value.status == rg.RG_EIO


def test_damaged_schedule_files_are_refused(case, rg, tmp_path):
    path = tmp_path / "epoch0.rgsched"
    rg.rg_schedule_save(case.gsched, path)
    good = path.read_bytes()

    def refused(data, name):
        p = tmp_path / name
        p.write_bytes(data)
        with pytest.raises(rg.RgError) as e:
            rg.rg_schedule_load(p)
        assert e.value.status == rg.RG_EIO, name

    refused(b"", "empty")
    refused(b"NOTASCHD" + good[8:], "magic")
    refused(good[:40], "header_only")
    refused(good[: len(good) // 2], "half")
    refused(good[:-1], "one_byte_short")
    refused(good + b"\\0", "trailing")
    bad = bytearray(good)
    bad[8:16] = (2**31).to_bytes(8, "little")                  # n_nodes out of range
    refused(bytes(bad), "n_nodes")
    bad = bytearray(good)
    bad[24:28] = (2**31 - 1).to_bytes(4, "little")             # far more batches than the file can hold
    refused(bytes(bad), "n_batches")
    bad = bytearray(good)
    first_ids = 32 + (case.gsched.n_batches + 1) * 8           # first seed ID
    bad[first_ids:first_ids + 4] = (case.w.n_nodes).to_bytes(4, "little")
    refused(bytes(bad), "id_out_of_range")
    bad = bytearray(good)
    bad[32 + 8:32 + 16] = (2**62).to_bytes(8, "little")        # a batch offset beyond everything
    refused(bytes(bad), "offset")
    with pytest.raises(rg.RgError) as e:
        rg.rg_schedule_load(tmp_path / "does_not_exist")
    assert e.value.status == rg.RG_EIO
    with pytest.raises(rg.RgError) as e:
        rg.rg_schedule_save(case.gsched, tmp_path / "no_such_dir" / "x")
    assert e.value.status == rg.RG_EIO
    rg.rg_schedule_load(path)                                  # and the good file still loads
