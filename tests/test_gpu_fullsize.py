"""GPU parity at the benchmark's full sizes, every stage against the CPU oracle.

For medium, large_sparse, fanout_stress and partition_share the oracle builds the WHOLE epoch (one host thread per
batch) and everything the library produces is compared with it bit for bit: every frontier, batch offset and
sample of every hop; freq of every node; the TopHot set, its slots and the cache table; the counts of every
batch; and the gathered bytes of a spread of batches (first, last = ragged, some in between), one batch per
launch and in the launch shape the benchmark times (several batches staged back to back by rg_gather_batches).
Nothing here is checked against the library's own outputs.

Memory placement: large_sparse and partition_share keep the remote table in pinned host memory, as their
configuration says (VectorPull and SyncPull cross the host link); medium and fanout_stress keep it in HBM.
Every workload also builds a second cache whose K lies below the number of candidates, so that the radix select and
the id-ascending tie-break at the threshold frequency run at full size (partition_share's own K covers every
touched remote row) and so that misses exist to be pulled.

The tiny configuration's whole epoch is covered by test_gpu_parity.py.
"""
import sys
import time

import numpy as np
import pytest
import torch

from paper_2509_05207_amd import synth

pytestmark = pytest.mark.gpu

PINNED_REMOTE = {"medium": False, "large_sparse": True, "fanout_stress": False, "partition_share": True}
ORACLE_THREADS = 16


_capture = None


@pytest.fixture(scope="module")
def rg(request):
    from paper_2509_05207_amd import binding
    binding.lib()
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    global _capture
    _capture = request.config.pluginmanager.getplugin("capturemanager")
    return binding


def note(msg):
    """A progress line past pytest's capture (these tests run for a while, and a silent run looks hung from outside)."""
    line = f"[fullsize {time.strftime('%H:%M:%S')}] {msg}"
    if _capture is not None:
        with _capture.global_and_fixture_disabled():
            print(line, file=sys.stderr, flush=True)
    else:
        print(line, file=sys.stderr, flush=True)


def host(t):
    return t.cpu().numpy()


def np_bytes(t):
    return t.contiguous().view(torch.uint8).cpu().numpy()


class Epoch:
    """One workload at full size: the library's schedule on the device, the oracle's on the host, both feature views."""

    def __init__(self, name, rg, orc):
        t0 = time.perf_counter()
        self.name = name
        cfg = self.cfg = synth.CONFIGS[name]
        W = self.W = synth.make_workload(cfg, device="cuda", feature_device="cuda", remote_device="cuda")
        torch.cuda.synchronize()
        note(f"{name}: inputs generated ({time.perf_counter() - t0:.1f} s)")
        self.s = rg.rg_build_schedule(W.indptr, W.indices, W.train, cfg.batch_size, cfg.fanout, cfg.s0, cfg.worker, cfg.epoch)
        self.o = orc.Schedule(host(W.indptr), host(W.indices), host(W.train), cfg.batch_size, cfg.fanout, cfg.s0, cfg.worker, cfg.epoch,
                              n_threads=ORACLE_THREADS)
        note(f"{name}: oracle schedule of {self.o.n_batches} batches built ({time.perf_counter() - t0:.1f} s)")
        self.is_local = host(W.is_local)
        if PINNED_REMOTE[name]:
            self.remote = synth.pinned_copy(W.remote_rows)        # the other partitions' memory: pinned host
            W.remote_rows = None                                   # (the device copy is not needed any more)
            remote_np = self.remote.view(torch.uint8).numpy()     # the oracle reads the very same host bytes
            note(f"{name}: remote table of {remote_np.nbytes / 1e9:.1f} GB in pinned host memory ({time.perf_counter() - t0:.1f} s)")
        else:
            self.remote = W.remote_rows
            remote_np = np_bytes(W.remote_rows)
        self.feat = rg.make_features(W.is_local, W.row_of, W.local_rows, self.remote, W.row_bytes)
        self.ofeat = orc.Features(self.is_local, host(W.row_of), np_bytes(W.local_rows), W.stride_bytes, remote_np, W.stride_bytes,
                                  W.row_bytes)
        self.freq = orc.frequency([self.o], W.n_nodes)
        self.n_candidates = int(((self.is_local == 0) & (self.freq > 0)).sum())
        _, self.off = self.o.input_nodes()
        note(f"{name}: ready ({time.perf_counter() - t0:.1f} s); {int(self.off[-1])} input nodes, {self.n_candidates} candidates, K = {W.K}")

    def spread(self):
        """First, last (ragged) and a few batches in between."""
        nb = self.o.n_batches
        return sorted({0, 1, nb // 3, nb // 2, (2 * nb) // 3, nb - 2, nb - 1})

    def group_size(self):
        """Batches per gather launch, as bench.py chooses it."""
        from paper_2509_05207_amd import accounting
        return accounting.gather_group(self.o.n_batches, int(self.off[-1]), self.W.stride_bytes)


@pytest.fixture(scope="module", params=["medium", "large_sparse", "fanout_stress", "partition_share"])
def ep(request, rg, orc):
    e = Epoch(request.param, rg, orc)
    yield e
    del e
    rg.rg_trim_memory()
    torch.cuda.empty_cache()


def test_every_frontier_and_sample(ep, rg):
    s, o = ep.s, ep.o
    assert s.n_batches == o.n_batches and s.L == o.L
    for hop in range(o.L + 1):
        ids, off = o.frontier(hop)
        gids, goff_dev, goff = rg.rg_schedule_frontier(s, hop)
        assert np.array_equal(goff, off), f"{ep.name}: batch offsets of hop {hop}"
        assert np.array_equal(host(goff_dev), off)
        assert np.array_equal(host(gids), ids), f"{ep.name}: frontier {hop}"
    for hop in range(o.L):
        so, nb = o.samples(hop)
        gso, gnb = rg.rg_schedule_samples(s, hop)
        assert np.array_equal(host(gso), so), f"{ep.name}: sample offsets of hop {hop}"
        assert np.array_equal(host(gnb), nb), f"{ep.name}: samples of hop {hop}"
        del so, nb, gso, gnb
    note(f"{ep.name}: every frontier and sample equal")
    if ep.name == "medium":        # computation blocks of a whole epoch at full size (test_gpu_parity.py covers the other shapes)
        rg.rg_schedule_build_blocks(s)
        for hop in range(o.L):
            assert np.array_equal(host(rg.rg_schedule_block(s, hop)), o.block(hop)), f"block {hop}"


def test_medium_frontier_forms_give_the_same_frontiers(ep, rg, monkeypatch):
    """The library picks one form of the frontier pass by the graph's size.  At full size, where a batch's map spans
    several cells of either form, the form it did not pick must give the same frontiers.  (The medium graph builds
    fast in either form; the small-graph form would scan 2 GB of maps per hop on the 10^8-node graph.)"""
    if ep.name != "medium":
        return
    cfg, W, o = ep.cfg, ep.W, ep.o
    for force in ("1", "0"):
        monkeypatch.setenv("RAPIDGNN_SPARSE_FRONTIER", force)
        for again in range(2):                             # the second build takes the first one's maps back from the pool
            s = rg.rg_build_schedule(W.indptr, W.indices, W.train, cfg.batch_size, cfg.fanout, cfg.s0, cfg.worker, cfg.epoch)
            for hop in range(o.L + 1):
                ids, off = o.frontier(hop)
                gids, _, goff = rg.rg_schedule_frontier(s, hop)
                assert np.array_equal(goff, off) and np.array_equal(host(gids), ids), f"forced {force}, build {again}: frontier {hop}"
            del s
        note(f"{ep.name}: frontiers equal with RAPIDGNN_SPARSE_FRONTIER={force}")


def check_cache(ep, rg, orc, c, K, batches, tag):
    """Everything a cache holds and serves, against the oracle: freq, TopHot set and slots, table, the counts of EVERY
    batch, the gathered bytes of `batches` one by one and of the groups of batches that contain them."""
    W, o = ep.W, ep.o
    ids, slot = orc.top_hot(ep.freq, ep.is_local, K)
    v = rg.rg_cache_view(c, W.n_nodes)
    assert np.array_equal(host(v["freq"]).view(np.uint32), ep.freq), f"{tag}: freq"
    assert v["K_eff"] == ids.size == min(K, ep.n_candidates), f"{tag}: K_eff"
    assert np.array_equal(host(v["cache_ids"]), ids), f"{tag}: TopHot set"
    assert np.array_equal(host(v["slot_of"]), slot), f"{tag}: slots"
    table = orc.cache_fill(ids, ep.ofeat, table_stride=v["stride"])
    assert np.array_equal(host(v["rows"]).reshape(ids.size, v["stride"])[:, :W.row_bytes], table[:, :W.row_bytes]), f"{tag}: cache table"
    del table
    note(f"{tag}: freq, TopHot ({ids.size} of {ep.n_candidates} candidates) and cache table equal")
    want = [orc.batch_stats(o, b, ep.is_local, slot) for b in range(o.n_batches)]
    got = [rg.rg_classify_batch(ep.s, c, ep.feat, b) for b in range(o.n_batches)]
    assert got == want, f"{tag}: counts of some batch differ"
    assert sum(x["n_miss"] for x in want) == int(ep.freq[(ep.is_local == 0) & (slot < 0)].sum()), "misses = frequency mass left out of the cache"
    off = ep.off
    m_max = int(np.diff(off).max())
    out = torch.empty(m_max * W.stride_bytes, dtype=torch.uint8, device="cuda")
    side = torch.cuda.Stream()
    for b in batches:
        out.fill_(0xCD)
        st = rg.rg_gather_batch(ep.s, c, ep.feat, b, out, out_stride=W.stride_bytes, out_capacity_rows=m_max, side_stream=side)
        torch.cuda.synchronize()
        ref = orc.gather_batch(o, b, ep.ofeat, out_stride=W.stride_bytes, fill=0xCD)
        assert np.array_equal(host(out)[: ref.size].reshape(ref.shape), ref), f"{tag}: gathered rows of batch {b}"
        assert st == want[b]
    del out
    # the launch shape the benchmark times: G consecutive batches staged back to back by one call
    G = ep.group_size()
    firsts = sorted({0, (o.n_batches - 1) // G * G})            # a whole group and the ragged last one
    for first in firsts:
        n = min(G, o.n_batches - first)
        rows = int(off[first + n] - off[first])
        big = torch.full((rows * W.stride_bytes,), 0xCD, dtype=torch.uint8, device="cuda")
        stats = rg.rg_gather_batches(ep.s, c, ep.feat, first, n, big, out_stride=W.stride_bytes, out_capacity_rows=rows, side_stream=side)
        torch.cuda.synchronize()
        got_rows = host(big).reshape(rows, W.stride_bytes)
        del big
        for k in range(n):
            b = first + k
            ref = orc.gather_batch(o, b, ep.ofeat, out_stride=W.stride_bytes, fill=0xCD)
            at = int(off[b] - off[first])
            assert np.array_equal(got_rows[at:at + ref.shape[0]], ref), f"{tag}: group of {n} at {first}, batch {b}"
            assert stats[k] == want[b]
        del got_rows
    note(f"{tag}: counts of all {o.n_batches} batches, rows of batches {batches} and of {len(firsts)} groups of {G} equal")


def test_cache_and_gather_with_the_configured_k(ep, rg, orc):
    c = rg.rg_build_cache([ep.s], ep.feat, ep.W.K)
    check_cache(ep, rg, orc, c, ep.W.K, ep.spread(), f"{ep.name}, K = {ep.W.K}")


def test_cache_and_gather_with_k_below_the_candidates(ep, rg, orc):
    """K in the middle of a run of equal frequencies: the select's threshold pass and the id-ascending tie-break decide."""
    order = np.sort(ep.freq[(ep.is_local == 0) & (ep.freq > 0)].astype(np.int64))[::-1]
    K = ep.n_candidates // 2
    t = order[K]
    run_lo, run_hi = int(np.searchsorted(-order, -t, "left")), int(np.searchsorted(-order, -t, "right"))
    if run_hi - run_lo >= 3:
        K = (run_lo + run_hi) // 2                              # strictly inside the tied run
    assert 0 < K < ep.n_candidates
    c = rg.rg_build_cache([ep.s], ep.feat, K)
    nb = ep.o.n_batches
    check_cache(ep, rg, orc, c, K, [0, nb // 2, nb - 1], f"{ep.name}, K = {K} (threshold frequency {int(t)}, tied run of {run_hi - run_lo})")


def test_medium_whole_epoch_position_sampler(rg, orc):
    """The O(f) sampler at the benchmark's size: the oracle draws positions too, so the whole epoch is compared."""
    cfg = synth.CONFIGS["medium"]
    W = synth.make_workload(cfg, device="cuda", feature_device="cuda")
    s = rg.rg_build_schedule_with(W.indptr, W.indices, W.train, cfg.batch_size, cfg.fanout, cfg.s0, cfg.worker, cfg.epoch,
                                  sampler=rg.RG_SAMPLER_POSITIONS)
    o = orc.Schedule(host(W.indptr), host(W.indices), host(W.train), cfg.batch_size, cfg.fanout, cfg.s0, cfg.worker, cfg.epoch,
                     n_threads=ORACLE_THREADS, sampler="positions")
    assert s.n_batches == o.n_batches
    for hop in range(o.L + 1):
        ids, off = o.frontier(hop)
        gids, _, goff = rg.rg_schedule_frontier(s, hop)
        assert np.array_equal(goff, off) and np.array_equal(host(gids), ids), f"frontier {hop}"
    for hop in range(o.L):
        so, nb = o.samples(hop)
        gso, gnb = rg.rg_schedule_samples(s, hop)
        assert np.array_equal(host(gso), so) and np.array_equal(host(gnb), nb), f"samples {hop}"
