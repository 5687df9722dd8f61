"""Pins for the oracle's frequency tally, TopHot, cache table, gather and stats
(Eq. 2; Alg. 1 steps 2-4 and inner loop; Sec. 3 "Invariants and bounds")."""
from collections import Counter

import numpy as np
import pytest

from paper_2509_05207_amd import synth


@pytest.fixture(scope="module")
def wl(orc):
    out = {}
    for name in ("small", "mid_bf16"):
        w = synth.make_workload(name)
        s = orc.Schedule(w.indptr.numpy(), w.indices.numpy(), w.train.numpy(), w.cfg.batch_size, w.cfg.fanout,
                         s0=1, n_threads=4)
        out[name] = (w, s)
    return out


def np_bytes(t):
    import torch
    return t.contiguous().view(torch.uint8).numpy()


def features(orc, w):
    return orc.Features(w.is_local.numpy(), w.row_of.numpy(), np_bytes(w.local_rows), w.stride_bytes,
                        np_bytes(w.remote_rows), w.stride_bytes, w.row_bytes)


def full_table(w):
    """X as one [N, row_bytes] byte matrix, assembled with numpy only."""
    loc, rem = np_bytes(w.local_rows), np_bytes(w.remote_rows)
    is_local = w.is_local.numpy().astype(bool)
    X = np.empty((w.n_nodes, w.stride_bytes), np.uint8)
    X[is_local] = loc
    X[~is_local] = rem
    return X[:, :w.row_bytes]


@pytest.mark.parametrize("name", ["small", "mid_bf16"])
def test_frequency_counts_batches_containing_the_node(orc, wl, name):
    w, s = wl[name]
    freq = orc.frequency([s], w.n_nodes)
    ids, off = s.input_nodes()
    c = Counter(ids.tolist())
    ref = np.zeros(w.n_nodes, np.uint32)
    for v, k in c.items():
        ref[v] = k
    assert np.array_equal(freq, ref)
    assert int(freq.sum()) == ids.size                       # counts sum to the number of listed IDs
    assert freq.max() <= s.n_batches                          # a node counts once per batch
    assert np.all(freq[w.train.numpy()] >= 1)                 # every train node is in its own batch
    # per-batch sets are duplicate free, which is what makes "occurrences" = "batches"
    for b in range(s.n_batches):
        seg = ids[off[b]:off[b + 1]]
        assert np.unique(seg).size == seg.size


def test_frequency_over_several_epochs_adds_up(orc, wl):
    w, s = wl["small"]
    s2 = orc.Schedule(w.indptr.numpy(), w.indices.numpy(), w.train.numpy(), w.cfg.batch_size, w.cfg.fanout,
                      s0=1, epoch=1)
    f1, f2 = orc.frequency([s], w.n_nodes), orc.frequency([s2], w.n_nodes)
    assert not np.array_equal(f1, f2)
    assert np.array_equal(orc.frequency([s, s2], w.n_nodes), f1 + f2)


def ref_top_hot(freq, is_local, K):
    cand = np.nonzero((is_local == 0) & (freq > 0))[0]
    order = np.lexsort((cand, -freq[cand].astype(np.int64)))          # freq descending, id ascending
    chosen = np.sort(cand[order[:K]])
    slot = np.full(freq.size, -1, np.int32)
    slot[chosen] = np.arange(chosen.size, dtype=np.int32)
    return chosen.astype(np.int32), slot, cand


@pytest.mark.parametrize("name", ["small", "mid_bf16"])
def test_top_hot_equals_a_full_sort(orc, wl, name):
    w, s = wl[name]
    freq = orc.frequency([s], w.n_nodes)
    is_local = w.is_local.numpy()
    n_cand = int(((is_local == 0) & (freq > 0)).sum())
    for K in (0, 1, 7, w.K, n_cand - 1, n_cand, n_cand + 5, 10 ** 9):
        ids, slot = orc.top_hot(freq, is_local, K)
        rid, rslot, cand = ref_top_hot(freq, is_local, K)
        assert np.array_equal(ids, rid) and np.array_equal(slot, rslot)
        assert ids.size == min(K, n_cand)
        assert not is_local[ids].any()                               # never a local node
        excluded = np.setdiff1d(cand, ids)
        if ids.size and excluded.size:
            assert freq[ids].min() >= freq[excluded].max()           # nothing hotter is left out


def test_top_hot_tie_break_is_by_ascending_id(orc):
    freq = np.array([5, 2, 2, 2, 9, 2, 0, 2], np.uint32)
    is_local = np.array([0, 0, 1, 0, 0, 0, 0, 0], np.uint8)
    ids, slot = orc.top_hot(freq, is_local, 4)
    assert ids.tolist() == [0, 1, 3, 4]                              # 9, 5, then the two smallest ids with freq 2
    assert slot.tolist() == [0, 1, -1, 2, 3, -1, -1, -1]
    ids, _ = orc.top_hot(freq, is_local, 100)
    assert ids.tolist() == [0, 1, 3, 4, 5, 7]                        # freq 0 and local never enter


@pytest.mark.parametrize("name", ["small", "mid_bf16"])
def test_cache_table_and_gather_equal_direct_indexing(orc, wl, name):
    w, s = wl[name]
    X = full_table(w)
    f = features(orc, w)
    freq = orc.frequency([s], w.n_nodes)
    cache_ids, _ = orc.top_hot(freq, w.is_local.numpy(), w.K)
    table = orc.cache_fill(cache_ids, f, table_stride=w.stride_bytes)
    assert np.array_equal(table[:, :w.row_bytes], X[cache_ids])
    assert cache_ids.size * w.row_bytes <= w.K * w.row_bytes         # n_hot * d bound, one buffer
    ids, off = s.input_nodes()
    for b in (0, s.n_batches // 2, s.n_batches - 1):
        out = orc.gather_batch(s, b, f, out_stride=w.stride_bytes + 16, fill=0xAB)
        seg = ids[off[b]:off[b + 1]]
        assert out.shape[0] == seg.size
        assert np.array_equal(out[:, :w.row_bytes], X[seg])
        assert np.all(out[:, w.row_bytes:] == 0xAB)                  # padding left alone


@pytest.mark.parametrize("name", ["small", "mid_bf16"])
def test_stats_are_the_set_arithmetic(orc, wl, name):
    w, s = wl[name]
    is_local = w.is_local.numpy()
    freq = orc.frequency([s], w.n_nodes)
    ids, off = s.input_nodes()
    local_set = set(np.nonzero(is_local)[0].tolist())
    for K in (0, w.K, 10 ** 9):
        cache_ids, slot = orc.top_hot(freq, is_local, K)
        cache_set = set(cache_ids.tolist())
        tot_miss = 0
        for b in range(s.n_batches):
            N_i = set(ids[off[b]:off[b + 1]].tolist())
            st = orc.batch_stats(s, b, is_local, slot)
            assert st["n_rows"] == len(N_i)
            assert st["n_local"] == len(N_i & local_set)
            assert st["n_hit"] == len(N_i & cache_set)
            assert st["n_miss"] == len(N_i - local_set - cache_set)       # |M_i| = RPC count of the batch
            tot_miss += st["n_miss"]
            if K == 0:
                assert st == orc.batch_stats(s, b, is_local, None)
                assert st["n_miss"] == len(N_i - local_set)                # on-demand baseline: all remote
        if K == 10 ** 9:
            assert tot_miss == 0                                           # everything touched is cached


def test_fetches_fall_with_cache_size_and_equal_the_uncached_frequency_mass(orc):
    """Remote fetches of an epoch = sum of freq over the remote nodes left out of the cache (a node is fetched once
    per batch that needs it); so they fall monotonically in n_hot, from the whole remote mass to zero, and TopHot's
    choice is the best one for its size (Eq. 2)."""
    w = synth.make_workload("small")
    s = orc.Schedule(w.indptr.numpy(), w.indices.numpy(), w.train.numpy(), w.cfg.batch_size, w.cfg.fanout, 9, 0, 0)
    is_local = w.is_local.numpy()
    freq = orc.frequency([s], w.n_nodes)
    remote = (is_local == 0) & (freq > 0)
    n_remote = int(remote.sum())
    rng = np.random.default_rng(3)
    last = None
    for K in (0, 1, 7, n_remote // 10, n_remote // 3, n_remote - 1, n_remote, n_remote + 50):
        ids, slot = orc.top_hot(freq, is_local, K)
        misses = sum(orc.batch_stats(s, b, is_local, slot)["n_miss"] for b in range(s.n_batches))
        uncached = remote.copy()
        uncached[ids] = False
        assert misses == int(freq[uncached].sum())
        if last is not None:
            assert misses <= last
        last = misses
        if K == 0:
            assert misses == int(freq[remote].sum())
        if K >= n_remote:
            assert misses == 0
        if 0 < K < n_remote:
            other = rng.choice(np.nonzero(remote)[0], size=K, replace=False)
            alt = remote.copy()
            alt[other] = False
            assert int(freq[alt].sum()) >= misses
