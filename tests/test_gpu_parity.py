"""GPU parity: the HIP library against the CPU oracle, element by element, through the C ABI.

Integer and byte work throughout, so the bar is bit-exact equality."""
import numpy as np
import pytest
import torch

from paper_2509_05207_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rg():
    from paper_2509_05207_amd import binding
    binding.lib()
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return binding


def np_bytes(t):
    return t.contiguous().view(torch.uint8).cpu().numpy()


class Case:
    """One workload, built by the oracle on the host and by the library on the device."""

    def __init__(self, name, orc, rg, s0=0, worker=0, epoch=0, pinned_remote=False):
        w = synth.make_workload(name)
        self.w, self.name = w, name
        self.s0, self.worker, self.epoch = s0, worker, epoch
        self.osched = orc.Schedule(w.indptr.numpy(), w.indices.numpy(), w.train.numpy(), w.cfg.batch_size, w.cfg.fanout,
                                   s0, worker, epoch, n_threads=8)
        self.ofeat = orc.Features(w.is_local.numpy(), w.row_of.numpy(), np_bytes(w.local_rows), w.stride_bytes,
                                  np_bytes(w.remote_rows), w.stride_bytes, w.row_bytes)
        d = "cuda"
        self.indptr, self.indices, self.train = w.indptr.to(d), w.indices.to(d), w.train.to(d)
        self.is_local, self.row_of = w.is_local.to(d), w.row_of.to(d)
        self.local_rows = w.local_rows.to(d)
        self.remote_rows = w.remote_rows.pin_memory() if pinned_remote else w.remote_rows.to(d)
        self.gsched = rg.rg_build_schedule(self.indptr, self.indices, self.train, w.cfg.batch_size, w.cfg.fanout, s0, worker, epoch)
        self.gfeat = rg.make_features(self.is_local, self.row_of, self.local_rows, self.remote_rows, w.row_bytes)


@pytest.fixture(scope="module", params=["small", "tiny", "mid", "mid_bf16"])
def case(request, orc, rg):
    return Case(request.param, orc, rg, s0=request.param_index, worker=request.param_index % 2, epoch=request.param_index % 3,
                pinned_remote=(request.param in ("small", "mid_bf16")))


def assert_schedules_equal(rg, gs, osched):
    assert gs.n_batches == osched.n_batches and gs.L == osched.L
    for hop in range(osched.L + 1):
        ids, off = osched.frontier(hop)
        gids, goff_dev, goff = rg.rg_schedule_frontier(gs, hop)
        assert np.array_equal(goff, off), f"frontier offsets differ at hop {hop}"
        assert np.array_equal(goff_dev.cpu().numpy(), off)
        assert np.array_equal(gids.cpu().numpy(), ids), f"frontier ids differ at hop {hop}"
    for hop in range(osched.L):
        so, nb = osched.samples(hop)
        gso, gnb = rg.rg_schedule_samples(gs, hop)
        assert np.array_equal(gso.cpu().numpy(), so), f"sample offsets differ at hop {hop}"
        assert np.array_equal(gnb.cpu().numpy(), nb), f"sampled neighbours differ at hop {hop}"


def test_schedule_matches_oracle(case, rg):
    assert rg.rg_graph_validate(case.indptr, case.indices) == 0
    assert_schedules_equal(rg, case.gsched, case.osched)


def test_schedule_is_reproducible_and_seed_dependent(case, rg):
    w = case.w
    again = rg.rg_build_schedule(case.indptr, case.indices, case.train, w.cfg.batch_size, w.cfg.fanout, case.s0, case.worker, case.epoch)
    other = rg.rg_build_schedule(case.indptr, case.indices, case.train, w.cfg.batch_size, w.cfg.fanout, case.s0, case.worker, case.epoch + 1)
    for hop in range(case.gsched.L + 1):
        a = rg.rg_schedule_frontier(case.gsched, hop)[0]
        b = rg.rg_schedule_frontier(again, hop)[0]
        assert torch.equal(a, b)
    a = rg.rg_schedule_frontier(case.gsched, 0)[0]
    c = rg.rg_schedule_frontier(other, 0)[0]
    assert not torch.equal(a, c)


@pytest.mark.parametrize("workspace", [0, 1, "two_batches"])
def test_blocks_match_oracle(case, rg, workspace):
    """Computation blocks: block-local source index of every sample, whatever the workspace grouping."""
    w = case.w
    s = rg.rg_build_schedule(case.indptr, case.indices, case.train, w.cfg.batch_size, w.cfg.fanout, case.s0, case.worker, case.epoch)
    with pytest.raises(rg.RgError) as e:
        rg.rg_schedule_block(s, 0)
    assert e.value.status == (rg.RG_EINVAL if s.L > 0 else rg.RG_ERANGE)
    limit = 2 * 4 * w.n_nodes if workspace == "two_batches" else workspace      # 1 byte: one batch at a time
    rg.rg_schedule_build_blocks(s, workspace_limit_bytes=limit)
    rg.rg_schedule_build_blocks(s)                                               # a second call changes nothing
    for hop in range(s.L):
        got = rg.rg_schedule_block(s, hop).cpu().numpy()
        assert np.array_equal(got, case.osched.block(hop)), f"block of hop {hop} differs"
    with pytest.raises(rg.RgError) as e:
        rg.rg_schedule_block(s, s.L)
    assert e.value.status == rg.RG_ERANGE


@pytest.mark.parametrize("tally", ["bytes", "words"])
@pytest.mark.parametrize("kmode", ["config", "zero", "all", "one"])
def test_cache_matches_oracle(case, rg, orc, kmode, tally, monkeypatch):
    """(These epochs have fewer than 256 batches, so the tally counts in bytes unless told not to.)"""
    if tally == "words":
        monkeypatch.setenv("RAPIDGNN_NARROW_TALLY", "0")
    w = case.w
    freq = orc.frequency([case.osched], w.n_nodes)
    n_cand = int(((w.is_local.numpy() == 0) & (freq > 0)).sum())
    K = {"config": w.K, "zero": 0, "all": n_cand + 10, "one": 1}[kmode]
    ids, slot = orc.top_hot(freq, w.is_local.numpy(), K)
    table = orc.cache_fill(ids, case.ofeat, table_stride=(w.row_bytes + 15) // 16 * 16)
    gc = rg.rg_build_cache([case.gsched], case.gfeat, K)
    v = rg.rg_cache_view(gc, w.n_nodes)
    assert v["K_eff"] == ids.size
    assert np.array_equal(v["freq"].cpu().numpy().view(np.uint32), freq)
    assert np.array_equal(v["cache_ids"].cpu().numpy(), ids)
    assert np.array_equal(v["slot_of"].cpu().numpy(), slot)
    assert v["stride"] == (w.row_bytes + 15) // 16 * 16
    got = v["rows"].cpu().numpy().reshape(ids.size, v["stride"])
    assert np.array_equal(got[:, :w.row_bytes], table[:, :w.row_bytes])
    assert v["K_eff"] * w.row_bytes <= max(K, 0) * w.row_bytes             # n_hot * d bound of one buffer


def check_gather(case, rg, orc, cache, slot, batches, out_stride, use_side_stream):
    w = case.w
    ids, off = case.osched.input_nodes()
    m_max = int(np.diff(off).max())
    side = torch.cuda.Stream() if use_side_stream else None
    out = torch.empty((m_max + 3) * out_stride, dtype=torch.uint8, device="cuda")
    for b in batches:
        out.fill_(0xCD)
        st = rg.rg_gather_batch(case.gsched, cache, case.gfeat, b, out, out_stride=out_stride, out_capacity_rows=m_max + 3,
                                side_stream=side)
        torch.cuda.synchronize()
        ref = orc.gather_batch(case.osched, b, case.ofeat, out_stride=out_stride, fill=0xCD)
        m = ref.shape[0]
        got = out.cpu().numpy().reshape(m_max + 3, out_stride)
        assert np.array_equal(got[:m], ref), f"batch {b}: gathered bytes differ"
        assert np.all(got[m:] == 0xCD), f"batch {b}: rows beyond the batch were written"
        assert st == orc.batch_stats(case.osched, b, w.is_local.numpy(), slot), f"batch {b}: stats differ"


@pytest.mark.parametrize("routing", ["no_cache", "k_zero", "k_config", "k_all"])
def test_gather_matches_oracle_under_every_routing(case, rg, orc, routing):
    w = case.w
    freq = orc.frequency([case.osched], w.n_nodes)
    nb = case.osched.n_batches
    batches = sorted({0, nb // 2, nb - 1})
    if routing == "no_cache":
        cache, slot = None, None
    else:
        K = {"k_zero": 0, "k_config": w.K, "k_all": 10 ** 9}[routing]
        cache = rg.rg_build_cache([case.gsched], case.gfeat, K)
        _, slot = orc.top_hot(freq, w.is_local.numpy(), K)
    for out_stride, side in ((w.row_bytes, False), (w.stride_bytes + 16, True)):
        check_gather(case, rg, orc, cache, slot, batches, out_stride, side)


def test_gather_from_a_cache_built_on_another_epoch(case, rg, orc):
    """The cache has no plan for this schedule: rows are classified on the fly against its slot table."""
    w = case.w
    other_o = orc.Schedule(w.indptr.numpy(), w.indices.numpy(), w.train.numpy(), w.cfg.batch_size, w.cfg.fanout,
                           case.s0, case.worker, case.epoch + 1, n_threads=8)
    other_g = rg.rg_build_schedule(case.indptr, case.indices, case.train, w.cfg.batch_size, w.cfg.fanout, case.s0, case.worker, case.epoch + 1)
    cache = rg.rg_build_cache([other_g], case.gfeat, w.K)
    _, slot = orc.top_hot(orc.frequency([other_o], w.n_nodes), w.is_local.numpy(), w.K)
    check_gather(case, rg, orc, cache, slot, [0, case.osched.n_batches - 1], w.stride_bytes, True)


def test_cache_over_two_epochs(rg, orc):
    c = Case("small", orc, rg, s0=5)
    w = c.w
    o2 = orc.Schedule(w.indptr.numpy(), w.indices.numpy(), w.train.numpy(), w.cfg.batch_size, w.cfg.fanout, 5, 0, 1)
    g2 = rg.rg_build_schedule(c.indptr, c.indices, c.train, w.cfg.batch_size, w.cfg.fanout, 5, 0, 1)
    assert_schedules_equal(rg, g2, o2)
    freq = orc.frequency([c.osched, o2], w.n_nodes)
    ids, slot = orc.top_hot(freq, w.is_local.numpy(), w.K)
    cache = rg.rg_build_cache([c.gsched, g2], c.gfeat, w.K)
    v = rg.rg_cache_view(cache, w.n_nodes)
    assert np.array_equal(v["freq"].cpu().numpy().view(np.uint32), freq)
    assert np.array_equal(v["cache_ids"].cpu().numpy(), ids)
    # both epochs have a plan in this cache
    c2 = Case.__new__(Case)
    c2.__dict__.update(c.__dict__)
    c2.osched, c2.gsched = o2, g2
    check_gather(c, rg, orc, cache, slot, [0, 3], w.stride_bytes, True)
    check_gather(c2, rg, orc, cache, slot, [1, o2.n_batches - 1], w.stride_bytes, False)


@pytest.mark.parametrize("frontier", ["0", "1"])
def test_cache_of_an_epoch_with_more_than_255_batches(rg, orc, frontier, monkeypatch):
    """Frequencies can pass 255 only where the epochs have more batches than that: the tally then counts in 32-bit
    words.  Two-node batches of the small graph with fan-outs (20, 20): 365 batches, and hubs that most of them reach.  With the large-graph
    frontier passes forced, the schedule carries no frequencies of its own and the cache tallies the input lists."""
    monkeypatch.setenv("RAPIDGNN_SPARSE_FRONTIER", frontier)
    c = Case("small", orc, rg, s0=11)
    w = c.w
    o = orc.Schedule(w.indptr.numpy(), w.indices.numpy(), w.train.numpy(), 2, [20, 20], 11, 0, 0)
    g = rg.rg_build_schedule(c.indptr, c.indices, c.train, 2, [20, 20], 11, 0, 0)
    assert o.n_batches > 255
    freq = orc.frequency([o], w.n_nodes)
    assert freq.max() > 255, "the case must need more than a byte per counter"
    for K in (w.K, 7):
        ids, slot = orc.top_hot(freq, w.is_local.numpy(), K)
        v = rg.rg_cache_view(rg.rg_build_cache([g], c.gfeat, K), w.n_nodes)
        assert np.array_equal(v["freq"].cpu().numpy().view(np.uint32), freq)
        assert np.array_equal(v["cache_ids"].cpu().numpy(), ids)
        assert np.array_equal(v["slot_of"].cpu().numpy(), slot)


@pytest.mark.parametrize("tally", ["bytes", "words"])
def test_cache_tallied_from_the_input_lists(rg, orc, tally, monkeypatch):
    """A schedule built with the large-graph frontier passes carries no frequencies of its own: the cache tallies the
    epochs' input lists, in bytes (four counters to a word) or in words."""
    monkeypatch.setenv("RAPIDGNN_SPARSE_FRONTIER", "1")
    if tally == "words":
        monkeypatch.setenv("RAPIDGNN_NARROW_TALLY", "0")
    c = Case("mid", orc, rg, s0=3)
    w = c.w
    o2 = orc.Schedule(w.indptr.numpy(), w.indices.numpy(), w.train.numpy(), w.cfg.batch_size, w.cfg.fanout, 3, 0, 1, n_threads=8)
    g2 = rg.rg_build_schedule(c.indptr, c.indices, c.train, w.cfg.batch_size, w.cfg.fanout, 3, 0, 1)
    freq = orc.frequency([c.osched, o2], w.n_nodes)
    for K in (w.K, 1):
        ids, slot = orc.top_hot(freq, w.is_local.numpy(), K)
        v = rg.rg_cache_view(rg.rg_build_cache([c.gsched, g2], c.gfeat, K), w.n_nodes)
        assert np.array_equal(v["freq"].cpu().numpy().view(np.uint32), freq)
        assert np.array_equal(v["cache_ids"].cpu().numpy(), ids)
        assert np.array_equal(v["slot_of"].cpu().numpy(), slot)
        assert rg.rg_cache_view(rg.rg_build_cache([c.gsched, g2], c.gfeat, K), w.n_nodes)["K_eff"] == ids.size


# ---------------------------------------------------------------- edge cases
def small_graph():
    w = synth.make_workload("small")
    return w, w.indptr.cuda(), w.indices.cuda(), w.train.cuda()


def test_degenerate_schedules(rg, orc):
    w, indptr, indices, train = small_graph()
    ip, ix, tr = w.indptr.numpy(), w.indices.numpy(), w.train.numpy()
    for T, B, fan in ((0, 16, [3, 2]), (10, 4, []), (10, 4, [0, 0]), (1, 1000, [2]), (33, 1, [3]), (64, 64, [1, 1, 1, 1, 1, 1, 1, 1])):
        g = rg.rg_build_schedule(indptr, indices, train[:T], B, fan, 9, 1, 1)
        o = orc.Schedule(ip, ix, tr[:T], B, fan, 9, 1, 1)
        assert_schedules_equal(rg, g, o)


def test_wide_fanouts_and_long_rows(rg, orc):
    """Fan-outs on both sides of every candidate-buffer size, rows far longer than the buffer, one hub row."""
    n = 6000
    rng = np.random.default_rng(12)
    deg = rng.integers(0, 700, n)
    deg[:8] = [0, 1, 63, 64, 65, 255, 256, 5999]
    rows = [np.sort(rng.choice(np.delete(np.arange(n), v), size=int(d), replace=False)).astype(np.int32) for v, d in enumerate(deg)]
    indptr = np.zeros(n + 1, np.int64)
    indptr[1:] = np.cumsum(deg)
    indices = np.concatenate(rows)
    train = rng.permutation(n)[:300].astype(np.int32)
    train[:8] = np.arange(8)
    dp, dx, dt = torch.from_numpy(indptr).cuda(), torch.from_numpy(indices).cuda(), torch.from_numpy(train).cuda()
    assert rg.rg_graph_validate(dp, dx) == 0
    for fan in ([1], [63], [64], [65], [191, 2], [192], [193], [448], [449], [960], [1984], [3, 1984]):
        g = rg.rg_build_schedule(dp, dx, dt, 37, fan, 1, 0, 0)
        o = orc.Schedule(indptr, indices, train, 37, fan, 1, 0, 0, n_threads=8)
        assert_schedules_equal(rg, g, o)


def test_rows_longer_than_a_tile(rg, orc):
    """Rows beyond the tile length (16384) are sampled tile by tile and merged: 2, 3 and 5 tiles, a row of
    exactly one tile and one of a tile plus one, as seeds and as neighbours of seeds."""
    n = 90000
    rng = np.random.default_rng(21)
    deg = rng.integers(0, 40, n)
    big = {0: 16384, 1: 16385, 2: 20000, 3: 40001, 4: 70000}
    for v, d in big.items():
        deg[v] = d
    rows = []
    for v in range(n):
        if v in big:
            r = rng.choice(n - 1, size=big[v], replace=False)
        else:
            r = np.unique(np.concatenate([rng.integers(0, n - 1, int(deg[v])), rng.integers(0, 5, 2)]))   # small rows point at the big ones
        r = np.sort(np.where(r >= v, r + 1, r)).astype(np.int32)
        rows.append(r)
    indptr = np.zeros(n + 1, np.int64)
    indptr[1:] = np.cumsum([r.size for r in rows])
    indices = np.concatenate(rows)
    train = np.concatenate([np.arange(5), rng.permutation(np.arange(5, n))[:400]]).astype(np.int32)
    dp, dx, dt = torch.from_numpy(indptr).cuda(), torch.from_numpy(indices).cuda(), torch.from_numpy(train).cuda()
    assert rg.rg_graph_validate(dp, dx) == 0
    for fan in ([3, 7], [64], [100, 5], [1984]):
        g = rg.rg_build_schedule(dp, dx, dt, 50, fan, 4, 1, 2)
        o = orc.Schedule(indptr, indices, train, 50, fan, 4, 1, 2, n_threads=8)
        assert_schedules_equal(rg, g, o)


def test_errors_are_reported_not_crashes(rg):
    w, indptr, indices, train = small_graph()
    with pytest.raises(rg.RgError) as e:
        rg.rg_build_schedule(indptr, indices, train, 16, [2] * 9)
    assert e.value.status == rg.RG_ERANGE
    with pytest.raises(rg.RgError) as e:
        rg.rg_build_schedule(indptr, indices, train, 16, [1985])
    assert e.value.status == rg.RG_ERANGE
    with pytest.raises(rg.RgError) as e:
        rg.rg_build_schedule(indptr, indices, train, 0, [2])
    assert e.value.status == rg.RG_EINVAL
    s = rg.rg_build_schedule(indptr, indices, train, 100, [3, 2])
    f = rg.make_features(w.is_local.cuda(), w.row_of.cuda(), w.local_rows.cuda(), w.remote_rows.cuda(), w.row_bytes)
    out = torch.zeros(4 * w.row_bytes, dtype=torch.uint8, device="cuda")
    with pytest.raises(rg.RgError) as e:
        rg.rg_gather_batch(s, None, f, 0, out, out_stride=w.row_bytes, out_capacity_rows=4)
    assert e.value.status == rg.RG_ERANGE
    assert int(out.sum().item()) == 0                          # nothing written
    with pytest.raises(rg.RgError) as e:
        rg.rg_gather_batch(s, None, f, s.n_batches, out, out_stride=w.row_bytes, out_capacity_rows=4)
    assert e.value.status == rg.RG_ERANGE
    with pytest.raises(rg.RgError) as e:
        rg.rg_gather_batch(s, None, f, 0, out, out_stride=w.row_bytes - 1, out_capacity_rows=10 ** 6)
    assert e.value.status == rg.RG_EINVAL


def test_graph_validate_counts_violations(rg):
    indptr = torch.tensor([0, 3, 5, 5, 8], dtype=torch.int64, device="cuda")
    good = torch.tensor([1, 2, 3, 0, 2, 0, 1, 2], dtype=torch.int32, device="cuda")
    assert rg.rg_graph_validate(indptr, good) == 0
    bad = torch.tensor([2, 1, 3, 0, 0, 0, 1, 9], dtype=torch.int32, device="cuda")     # unsorted, duplicate, out of range
    assert rg.rg_graph_validate(indptr, bad) == 3


def test_torch_backed_allocator(rg, orc):
    w, indptr, indices, train = small_graph()
    alloc = rg.TorchAllocator()
    g = rg.rg_build_schedule(indptr, indices, train, w.cfg.batch_size, w.cfg.fanout, 2, 0, 0, allocator=alloc.struct)
    o = orc.Schedule(w.indptr.numpy(), w.indices.numpy(), w.train.numpy(), w.cfg.batch_size, w.cfg.fanout, 2, 0, 0)
    assert_schedules_equal(rg, g, o)
    assert alloc.n_alloc > 0 and len(alloc.live) > 0
    f = rg.make_features(w.is_local.cuda(), w.row_of.cuda(), w.local_rows.cuda(), w.remote_rows.cuda(), w.row_bytes)
    c = rg.rg_build_cache([g], f, w.K, allocator=alloc.struct)
    ids, _ = orc.top_hot(orc.frequency([o], w.n_nodes), w.is_local.numpy(), w.K)
    assert np.array_equal(rg.rg_cache_view(c, w.n_nodes)["cache_ids"].cpu().numpy(), ids)
    del c, g
    assert len(alloc.live) == 0                                  # everything handed back


def test_a_schedule_keeps_its_allocator_alive(rg, orc):
    """The allocator object is dropped before the schedule: the handle must hold on to it (its memory is the
    allocator's tensors, and destroy calls back into it)."""
    import gc
    w, indptr, indices, train = small_graph()
    alloc = rg.TorchAllocator()
    live = alloc.live
    g = rg.rg_build_schedule(indptr, indices, train, w.cfg.batch_size, w.cfg.fanout, 2, 0, 0, allocator=alloc.struct)
    del alloc
    gc.collect()
    torch.empty(1 << 24, dtype=torch.uint8, device="cuda").fill_(0x5A)      # would land on freed blocks
    torch.cuda.synchronize()
    o = orc.Schedule(w.indptr.numpy(), w.indices.numpy(), w.train.numpy(), w.cfg.batch_size, w.cfg.fanout, 2, 0, 0)
    assert_schedules_equal(rg, g, o)
    rg.rg_schedule_build_blocks(g)                                           # scratch from the same allocator
    assert np.array_equal(rg.rg_schedule_block(g, 0).cpu().numpy(), o.block(0))
    assert len(live) > 0
    del g
    gc.collect()
    assert len(live) == 0


def test_an_allocation_that_fails_is_an_error_not_a_crash(rg, orc):
    """The per-batch maps of a build are n_batches * n_nodes bits each: an allocator that cannot give that much makes
    the build return RG_ENOMEM with everything it had taken handed back; the same goes for the cache's arrays."""
    import gc
    w, indptr, indices, train = small_graph()
    beta = -(-train.numel() // 16)
    words_per_batch = ((w.n_nodes + 31) // 32 + 63) // 64 * 64
    map_bytes = beta * words_per_batch * 4                                   # one bitmap
    alloc = rg.TorchAllocator(limit_bytes=map_bytes // 2)
    with pytest.raises(rg.RgError) as e:
        rg.rg_build_schedule(indptr, indices, train, 16, [3, 2], allocator=alloc.struct)
    assert e.value.status == rg.RG_ENOMEM and alloc.n_refused >= 1
    torch.cuda.synchronize()
    assert len(alloc.live) == 0                                              # nothing kept
    roomy = rg.TorchAllocator()
    g = rg.rg_build_schedule(indptr, indices, train, 16, [3, 2], allocator=roomy.struct)
    o = orc.Schedule(w.indptr.numpy(), w.indices.numpy(), w.train.numpy(), 16, [3, 2])
    assert_schedules_equal(rg, g, o)
    f = rg.make_features(w.is_local.cuda(), w.row_of.cuda(), w.local_rows.cuda(), w.remote_rows.cuda(), w.row_bytes)
    tight = rg.TorchAllocator(limit_bytes=w.n_nodes * 4 - 1)                 # freq and slot_of need n_nodes * 4 bytes each
    with pytest.raises(rg.RgError) as e:
        rg.rg_build_cache([g], f, w.K, allocator=tight.struct)
    assert e.value.status == rg.RG_ENOMEM
    torch.cuda.synchronize()
    assert len(tight.live) == 0
    del g, e                                                                 # (the caught error's traceback holds the schedule too)
    gc.collect()
    assert len(roomy.live) == 0


def test_train_nodes_are_checked(rg):
    w, indptr, indices, train = small_graph()
    n = w.n_nodes
    for bad_value, fanout in ((n, [3, 2]), (-1, [3, 2]), (2**31 - 1, [3]), (n, [])):
        bad = train.clone()
        bad[17] = bad_value
        with pytest.raises(rg.RgError) as e:
            rg.rg_build_schedule(indptr, indices, bad, 100, fanout)
        assert e.value.status == rg.RG_EINVAL and "train nodes" in str(e.value)
    dup = train.clone()
    dup[5] = dup[400]                                                        # the same ID twice, in different batches
    for fanout in ([3, 2], []):
        with pytest.raises(rg.RgError) as e:
            rg.rg_build_schedule(indptr, indices, dup, 100, fanout)
        assert e.value.status == rg.RG_EINVAL
    torch.cuda.synchronize()
    rg.rg_build_schedule(indptr, indices, train, 100, [3, 2])                # and the good input still builds


def test_more_batches_than_the_limit_are_refused(rg):
    w, indptr, indices, train = small_graph()
    T = rg.RG_MAX_BATCHES + 1
    many = torch.arange(T, dtype=torch.int32, device="cuda") % w.n_nodes     # (never looked at: the count is refused first)
    with pytest.raises(rg.RgError) as e:
        rg.rg_build_schedule(indptr, indices, many, 1, [2])
    assert e.value.status == rg.RG_ERANGE and "RG_MAX_BATCHES" in str(e.value)


def test_seeds_view_is_the_first_frontier(case, rg):
    seeds, off = rg.rg_schedule_seeds(case.gsched)
    ids, ooff = case.osched.seeds()
    assert np.array_equal(seeds.cpu().numpy(), ids) and np.array_equal(off.cpu().numpy(), ooff)


def test_rows_of_odd_width_and_alignment(rg, orc):
    """Row widths and strides at 16-, 8-, 4-, 2- and 1-byte alignment: 16-byte vectors at every dword phase, every
    tail length, and the byte path."""
    w, indptr, indices, train = small_graph()
    ip, ix, tr = w.indptr.numpy(), w.indices.numpy(), w.train.numpy()
    o = orc.Schedule(ip, ix, tr, 100, [5, 3], 3, 0, 0)
    g = rg.rg_build_schedule(indptr, indices, train, 100, [5, 3], 3, 0, 0)
    n_local, n_remote = w.extra["n_local"], w.extra["n_remote"]
    rng = np.random.default_rng(5)
    for row_bytes, stride in ((2408, 2416), (2408, 2408), (2404, 2404), (1204, 1204), (100, 100), (7, 7), (33, 36), (1, 1), (24, 32),
                              (30, 30), (12, 12), (20, 20), (44, 52), (63, 64)):
        loc = rng.integers(0, 256, (n_local, stride), dtype=np.uint8)
        rem = rng.integers(0, 256, (n_remote, stride), dtype=np.uint8)
        of = orc.Features(w.is_local.numpy(), w.row_of.numpy(), loc, stride, rem, stride, row_bytes)
        gf = rg.make_features(w.is_local.cuda(), w.row_of.cuda(), torch.from_numpy(loc).cuda(), torch.from_numpy(rem).cuda(), row_bytes,
                              local_stride=stride, remote_stride=stride)
        cache = rg.rg_build_cache([g], gf, 200)
        for out_stride in (stride, stride + 5 if stride % 4 else stride + 8):
            m = int(np.diff(o.input_nodes()[1]).max())
            out = torch.full((m * out_stride,), 0xEE, dtype=torch.uint8, device="cuda")
            rg.rg_gather_batch(g, cache, gf, 1, out, out_stride=out_stride, out_capacity_rows=m)
            torch.cuda.synchronize()
            ref = orc.gather_batch(o, 1, of, out_stride=out_stride, fill=0xEE)
            assert np.array_equal(out.cpu().numpy()[: ref.size].reshape(ref.shape), ref), (row_bytes, stride, out_stride)


# ------------------------------------------------------------------ the O(f) alternative sampler
@pytest.mark.parametrize("fanout", [None, (300, 3), (70, 2), (1, 1), (64, 63)])
def test_position_sampler_matches_oracle(case, rg, orc, fanout):
    """RG_SAMPLER_POSITIONS against the oracle's position sampler: every frontier, sample and block, bit for bit;
    fan-outs on both sides of the workgroup width and of the 64-slot selection branch."""
    w = case.w
    fan = list(fanout) if fanout else list(w.cfg.fanout)
    o = orc.Schedule(w.indptr.numpy(), w.indices.numpy(), w.train.numpy(), w.cfg.batch_size, fan, case.s0, case.worker, case.epoch,
                     n_threads=8, sampler="positions")
    g = rg.rg_build_schedule_with(case.indptr, case.indices, case.train, w.cfg.batch_size, fan, case.s0, case.worker, case.epoch,
                                  sampler=rg.RG_SAMPLER_POSITIONS)
    assert_schedules_equal(rg, g, o)
    rg.rg_schedule_build_blocks(g)
    for hop in range(g.L):
        assert np.array_equal(rg.rg_schedule_block(g, hop).cpu().numpy(), o.block(hop))
    if fanout is None:
        # the cache and the gather do not care which sampler built the schedule
        freq = orc.frequency([o], w.n_nodes)
        ids, slot = orc.top_hot(freq, w.is_local.numpy(), w.K)
        c = rg.rg_build_cache([g], case.gfeat, w.K)
        assert np.array_equal(rg.rg_cache_view(c, w.n_nodes)["cache_ids"].cpu().numpy(), ids)
        _, off = o.input_nodes()
        m_max = int(np.diff(off).max())
        out = torch.empty(m_max * w.row_bytes, dtype=torch.uint8, device="cuda")
        for b in (0, g.n_batches - 1):
            st = rg.rg_gather_batch(g, c, case.gfeat, b, out, out_stride=w.row_bytes, out_capacity_rows=m_max)
            torch.cuda.synchronize()
            ref = orc.gather_batch(o, b, case.ofeat, out_stride=w.row_bytes, fill=0)
            assert np.array_equal(out.cpu().numpy()[:ref.size].reshape(ref.shape), ref)
            assert st == orc.batch_stats(o, b, w.is_local.numpy(), slot)


def test_unknown_sampler_is_refused(case, rg):
    w = case.w
    with pytest.raises(rg.RgError) as e:
        rg.rg_build_schedule_with(case.indptr, case.indices, case.train, w.cfg.batch_size, w.cfg.fanout, 0, 0, 0, sampler=7)
    assert e.value.status == rg.RG_EINVAL


@pytest.mark.parametrize("force", ["1", "0"])
def test_both_frontier_variants_give_the_same_schedule(case, rg, force, monkeypatch):
    """The frontier passes for very large graphs (eight flag groups per thread, two-pass emit) forced onto small ones."""
    monkeypatch.setenv("RAPIDGNN_SPARSE_FRONTIER", force)
    w = case.w
    g = rg.rg_build_schedule(case.indptr, case.indices, case.train, w.cfg.batch_size, w.cfg.fanout, case.s0, case.worker, case.epoch)
    assert_schedules_equal(rg, g, case.osched)
    g2 = rg.rg_build_schedule(case.indptr, case.indices, case.train, w.cfg.batch_size, w.cfg.fanout, case.s0, case.worker, case.epoch)
    assert_schedules_equal(rg, g2, case.osched)          # bitmaps and flags come back clean from the block cache


@pytest.mark.parametrize("force", ["1", "0"])
@pytest.mark.parametrize("sampler", ["keys", "positions"])
@pytest.mark.parametrize("fanout", [None, (300, 3)])
def test_both_forms_of_the_reached_map_give_the_same_schedule(case, rg, orc, force, sampler, fanout, monkeypatch):
    """Marks as plain byte stores into a byte per ID, and as atomic ORs into a bit per ID (what graphs too large for
    the byte form get), each forced; both samplers mark through the same call.  With fan-outs (300, 3) and the byte
    form forced, the key sampler's first hop still marks bits (its byte-marking kernels stop at a fan-out of 192)
    and its second hop bytes: both forms within one build."""
    monkeypatch.setenv("RAPIDGNN_BYTE_MAPS", force)
    w = case.w
    fan = list(fanout) if fanout else list(w.cfg.fanout)
    code = rg.RG_SAMPLER_KEYS if sampler == "keys" else rg.RG_SAMPLER_POSITIONS
    if sampler == "keys" and not fanout:
        o = case.osched
    else:
        o = orc.Schedule(w.indptr.numpy(), w.indices.numpy(), w.train.numpy(), w.cfg.batch_size, fan, case.s0, case.worker, case.epoch,
                         n_threads=8, sampler=sampler)
    for _ in range(2):                                  # the second build finds the maps' memory used before
        g = rg.rg_build_schedule_with(case.indptr, case.indices, case.train, w.cfg.batch_size, fan, case.s0, case.worker, case.epoch,
                                      sampler=code)
        assert_schedules_equal(rg, g, o)


def test_few_listed_nodes_plan_without_the_route_table(case, rg, orc):
    """An epoch that lists far fewer input nodes than the graph has nodes is planned by direct lookups."""
    w = case.w
    if w.n_nodes < 2000:
        pytest.skip("needs a graph much larger than the epoch's input sets")
    train = case.train[:20].contiguous()
    fan = [3, 2]
    o = orc.Schedule(w.indptr.numpy(), w.indices.numpy(), w.train.numpy()[:20], 7, fan, 5, 0, 0)
    g = rg.rg_build_schedule(case.indptr, case.indices, train, 7, fan, 5, 0, 0)
    assert_schedules_equal(rg, g, o)
    _, off = o.input_nodes()
    assert off[-1] < w.n_nodes // 4
    freq = orc.frequency([o], w.n_nodes)
    ids, slot = orc.top_hot(freq, w.is_local.numpy(), 5)
    c = rg.rg_build_cache([g], case.gfeat, 5)
    assert np.array_equal(rg.rg_cache_view(c, w.n_nodes)["cache_ids"].cpu().numpy(), ids)
    m_max = int(np.diff(off).max())
    out = torch.empty(m_max * w.row_bytes, dtype=torch.uint8, device="cuda")
    for b in range(g.n_batches):
        st = rg.rg_gather_batch(g, c, case.gfeat, b, out, out_stride=w.row_bytes, out_capacity_rows=m_max)
        torch.cuda.synchronize()
        ref = orc.gather_batch(o, b, case.ofeat, out_stride=w.row_bytes, fill=0)
        assert np.array_equal(out.cpu().numpy()[:ref.size].reshape(ref.shape), ref)
        assert st == orc.batch_stats(o, b, w.is_local.numpy(), slot)


def test_rows_that_overflow_the_candidate_buffer_under_the_guessed_cut(rg, orc):
    """Under the guessed cut a long row is expected to yield a few dozen candidates.  Rows built from IDs whose keys
    (under the node's own state) lie below that cut by the hundred overflow the candidate buffer instead: at the very
    first block, in the middle of the row, in its last blocks only, and by accumulation one past the buffer's size,
    so the fast block loop is left at each of its three steps and the general path prunes and goes on."""
    n, f, deg = 200000, 10, 1200
    s0, wk, ep = 5, 0, 1
    hs = orc.hop_state(orc.batch_seed(s0, wk, ep, 0), 0)
    lam = f + 4.0 * np.sqrt(np.float32(f)) + 8.0
    cut = int(np.float32(lam) / np.float32(deg) * np.float32(4294967296.0))
    # (seed, number of low keys, ID range the low-key IDs come from)
    plans = [(17, deg, (0, n)), (1234, 200, (150000, n)), (50001, 300, (80000, 120000)), (77777, 129, (0, n)), (99999, 128, (0, n)),
             (31, 600, (0, 60000))]
    rng = np.random.default_rng(5)
    rows = [np.unique(rng.integers(0, n, 4)).astype(np.int32) for _ in range(n)]
    for v, n_low, (a, b) in plans:
        S = orc.node_state(hs, v)
        keys = np.array([orc.key32(S, u) for u in range(n)], dtype=np.uint64)
        cand = np.arange(n)
        cand = cand[cand != v]
        low = cand[(keys[cand] < cut // 2) & (cand >= a) & (cand < b)]
        high = cand[(keys[cand] > (1 << 31)) & ((cand < a) | (cand >= b) | (b - a == n))]
        assert low.size >= n_low and high.size >= deg - n_low, (v, low.size, high.size)
        row = np.concatenate([rng.permutation(low)[:n_low], rng.permutation(high)[:deg - n_low]])
        rows[v] = np.sort(row).astype(np.int32)
        assert rows[v].size == deg
    indptr = np.zeros(n + 1, np.int64)
    indptr[1:] = np.cumsum([r.size for r in rows])
    indices = np.concatenate(rows)
    train = np.array([p[0] for p in plans] + [8, 9], dtype=np.int32)
    dp, dx, dt = torch.from_numpy(indptr).cuda(), torch.from_numpy(indices).cuda(), torch.from_numpy(train).cuda()
    assert rg.rg_graph_validate(dp, dx) == 0
    g = rg.rg_build_schedule(dp, dx, dt, 100, [f], s0, wk, ep)
    o = orc.Schedule(indptr, indices, train, 100, [f], s0, wk, ep)
    assert_schedules_equal(rg, g, o)
    # the rows are what they were built to be: far more keys below the guessed cut than the buffer holds
    for v, n_low, _ in plans:
        S = orc.node_state(hs, v)
        assert sum(orc.key32(S, int(u)) <= cut for u in rows[v]) == n_low


@pytest.mark.parametrize("deg", [1500, 200])
def test_rows_built_to_defeat_the_guessed_cut(rg, orc, deg):
    """Long rows (and rows of 65-256 IDs, which are held in registers) are first taken with a cut guessed from the
    key distribution.  Rows made of IDs whose keys (under the node's own state) all lie above that cut, or with exactly
    f - 1, f and f + 1 keys below it, force the fallback to the exact procedure and both sides of its trigger."""
    n, f = 20000, 10
    s0, wk, ep = 21, 0, 3
    specials = [11, 222, 3333, 4444, 5555]               # seeds, all in batch 0 (one batch)
    below = [0, f - 1, f, f + 1, 100]                    # keys below the guessed cut in each special row (100: more than a wave holds)
    hs = orc.hop_state(orc.batch_seed(s0, wk, ep, 0), 0)
    lam = f + 4.0 * np.sqrt(np.float32(f)) + 8.0
    cut = int(np.float32(lam) / np.float32(deg) * np.float32(4294967296.0))
    rng = np.random.default_rng(77)
    rows = [np.unique(rng.integers(0, n, 6)).astype(np.int32) for _ in range(n)]
    for v, nb in zip(specials, below):
        S = orc.node_state(hs, v)
        keys = np.array([orc.key32(S, u) for u in range(n)], dtype=np.uint64)
        cand = np.arange(n)
        cand = cand[cand != v]
        lo_ids = cand[keys[cand] < cut // 2]             # safely below the cut
        hi_ids = cand[keys[cand] > (1 << 31)]            # far above it
        assert lo_ids.size >= nb and hi_ids.size >= deg
        row = np.concatenate([rng.permutation(lo_ids)[:nb], rng.permutation(hi_ids)[:deg - nb]])
        rows[v] = np.sort(row).astype(np.int32)
    indptr = np.zeros(n + 1, np.int64)
    indptr[1:] = np.cumsum([r.size for r in rows])
    indices = np.concatenate(rows)
    train = np.array(specials + [5, 6, 7], dtype=np.int32)
    dp, dx, dt = torch.from_numpy(indptr).cuda(), torch.from_numpy(indices).cuda(), torch.from_numpy(train).cuda()
    assert rg.rg_graph_validate(dp, dx) == 0
    g = rg.rg_build_schedule(dp, dx, dt, 100, [f], s0, wk, ep)
    o = orc.Schedule(indptr, indices, train, 100, [f], s0, wk, ep)
    assert_schedules_equal(rg, g, o)
    # the construction did what it set out to do: the oracle's sample of each special row has the planned number of
    # keys below the guessed cut
    ids, off = o.frontier(0)
    so, nbr = o.samples(0)
    for v, nb in zip(specials, below):
        j = int(np.nonzero(ids == v)[0][0])
        S = orc.node_state(hs, v)
        got = nbr[so[j]:so[j + 1]]
        assert got.size == f
        assert sum(orc.key32(S, int(u)) <= cut for u in got) == min(nb, f)


@pytest.mark.parametrize("T", [1, 2, 127, 128, 129, 255, 257, 1000, 4097, 50000])
def test_epoch_shuffle_at_the_bucket_bounds(rg, orc, T):
    """The shuffled order of the train nodes alone (no hops), for sizes on both sides of every change in the number
    of buckets the device shuffle uses, against the oracle's sort by (key, position)."""
    rng = np.random.default_rng(T)
    train = rng.permutation(200000)[:T].astype(np.int32)
    indptr = torch.zeros(200001, dtype=torch.int64, device="cuda")
    indices = torch.empty(0, dtype=torch.int32, device="cuda")
    for s0, worker, epoch in ((0, 0, 0), (12345, 3, 7)):
        g = rg.rg_build_schedule(indptr, indices, torch.from_numpy(train).cuda(), 100, [], s0, worker, epoch)
        want = orc.epoch_seeds(train, s0, worker, epoch)
        got, _, off = rg.rg_schedule_frontier(g, 0)
        assert np.array_equal(got.cpu().numpy(), want), f"T = {T}: shuffled order differs"
        assert off[-1] == T and len(off) == (T + 99) // 100 + 1


@pytest.mark.parametrize("tally", ["bytes", "words"])
def test_top_hot_with_an_unaligned_locality_array(case, rg, orc, tally, monkeypatch):
    """TopHot reads is_local with wide loads when its address allows them: the same array at an odd address (the
    one-by-one path) selects the same cache."""
    if tally == "words":
        monkeypatch.setenv("RAPIDGNN_NARROW_TALLY", "0")
    w = case.w
    shifted = torch.empty(w.n_nodes + 1, dtype=torch.uint8, device="cuda")
    shifted[1:] = case.is_local
    odd = shifted[1:]
    assert odd.data_ptr() % 2 == 1
    feat = rg.make_features(odd, case.row_of, case.local_rows, case.remote_rows, w.row_bytes)
    a = rg.rg_cache_view(rg.rg_build_cache([case.gsched], case.gfeat, w.K), w.n_nodes)
    b = rg.rg_cache_view(rg.rg_build_cache([case.gsched], feat, w.K), w.n_nodes)
    ids, slot = orc.top_hot(orc.frequency([case.osched], w.n_nodes), w.is_local.numpy(), w.K)
    for v in (a, b):
        assert v["K_eff"] == ids.size
        assert np.array_equal(v["cache_ids"].cpu().numpy(), ids)
        assert np.array_equal(v["slot_of"].cpu().numpy(), slot)
