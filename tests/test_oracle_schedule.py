"""Pins for the oracle's epoch schedule: shuffle, batching, hops, frontiers
(Sec. 3 "Offline enumeration and cache construction"; Sec. 4 par. (2))."""
import numpy as np
import pytest

from paper_2509_05207_amd import synth


@pytest.fixture(scope="module")
def small():
    w = synth.make_workload("small")
    return w, w.indptr.numpy(), w.indices.numpy(), w.train.numpy()


def build(orc, small, **kw):
    w, indptr, indices, train = small
    args = dict(batch_size=w.cfg.batch_size, fanout=w.cfg.fanout, s0=3, worker=1, epoch=2)
    args.update(kw)
    return orc.Schedule(indptr, indices, train, **args)


def test_epoch_seeds_are_a_shuffle_by_hash_key(orc, small):
    _, _, _, train = small
    seeds = orc.epoch_seeds(train, 3, 1, 2)
    assert np.array_equal(np.sort(seeds), np.sort(train))
    assert not np.array_equal(seeds, train)
    assert np.array_equal(seeds, orc.epoch_seeds(train, 3, 1, 2))
    assert not np.array_equal(seeds, orc.epoch_seeds(train, 3, 1, 3))
    assert not np.array_equal(seeds, orc.epoch_seeds(train, 3, 0, 2))
    assert not np.array_equal(seeds, orc.epoch_seeds(train, 4, 1, 2))
    # the order is "ascending (key, position)", with the key drawn from the epoch stream
    P = orc.epoch_state(3, 1, 2)
    order = sorted(range(train.size), key=lambda t: (orc.combine(P, t), t))
    assert np.array_equal(seeds, train[order])


def test_shuffle_is_close_to_uniform(orc):
    # position of element 0 after the shuffle, over many epochs: uniform on 0..9
    train = np.arange(10, dtype=np.int32)
    counts = np.zeros(10)
    n = 5000
    for e in range(n):
        counts[int(np.nonzero(orc.epoch_seeds(train, 1, 0, e) == 0)[0][0])] += 1
    chi2 = ((counts - n / 10) ** 2 / (n / 10)).sum()
    assert chi2 < 9 + 5 * np.sqrt(18), chi2


def test_batches_are_consecutive_slices_last_one_partial(orc, small):
    w, _, _, train = small
    s = build(orc, small)
    B, T = w.cfg.batch_size, train.size
    assert s.n_batches == -(-T // B)
    ids, off = s.seeds()
    assert np.array_equal(off, np.minimum(np.arange(s.n_batches + 1) * B, T))
    assert off[-1] - off[-2] == T - (s.n_batches - 1) * B and 0 < off[-1] - off[-2] < B
    assert np.array_equal(ids, orc.epoch_seeds(train, 3, 1, 2))


def test_hops_frontiers_and_samples(orc, small):
    w, indptr, indices, _ = small
    s = build(orc, small)
    L = len(w.cfg.fanout)
    assert s.L == L
    for hop in range(L):
        f = w.cfg.fanout[hop]
        U, uoff = s.frontier(hop)
        Un, noff = s.frontier(hop + 1)
        soff, nbr = s.samples(hop)
        deg = indptr[U.astype(np.int64) + 1] - indptr[U]
        assert np.array_equal(np.diff(soff), np.minimum(deg, f))         # |sample| = min(deg, f)
        bs = None
        for b in range(s.n_batches):
            cur = U[uoff[b]:uoff[b + 1]]
            nxt = Un[noff[b]:noff[b + 1]]
            assert np.array_equal(nxt[:cur.size], cur)                   # U_l is a prefix of U_{l+1}
            assert np.unique(nxt).size == nxt.size                       # no duplicates
            new = nxt[cur.size:]
            assert np.all(np.diff(new) > 0)                              # new IDs ascending
            samp = nbr[soff[uoff[b]]:soff[uoff[b + 1]]]
            assert set(nxt.tolist()) == set(cur.tolist()) | set(samp.tolist())
            # every node's sample equals the single-row sampler under that batch's stream
            hs = orc.hop_state(orc.batch_seed(3, 1, 2, b), hop)
            for j in range(uoff[b], min(uoff[b + 1], uoff[b] + 12)):
                v = int(U[j])
                row = indices[indptr[v]:indptr[v + 1]]
                assert np.array_equal(nbr[soff[j]:soff[j + 1]], orc.sample_row(row, f, orc.node_state(hs, v)))
                assert np.isin(nbr[soff[j]:soff[j + 1]], row).all()
    ids, off = s.input_nodes()
    bound = w.cfg.batch_size
    for f in w.cfg.fanout:
        bound += bound * f
    assert np.diff(off).max() <= min(bound, w.n_nodes)


def test_a_batch_built_alone_equals_the_batch_inside_the_epoch(orc, small):
    s = build(orc, small)
    for b in (0, 3, s.n_batches - 1):
        one = build(orc, small, batch_lo=b, batch_hi=b + 1)
        assert one.n_batches == 1
        for hop in range(s.L + 1):
            ids, off = s.frontier(hop)
            i1, o1 = one.frontier(hop)
            assert np.array_equal(i1, ids[off[b]:off[b + 1]])
        for hop in range(s.L):
            _, off = s.frontier(hop)
            so, nb = s.samples(hop)
            so1, nb1 = one.samples(hop)
            assert np.array_equal(nb1, nb[so[off[b]]:so[off[b + 1]]])


def test_thread_count_does_not_change_the_result(orc, small):
    a, b = build(orc, small), build(orc, small, n_threads=4)
    for hop in range(a.L + 1):
        assert all(np.array_equal(x, y) for x, y in zip(a.frontier(hop), b.frontier(hop)))
    for hop in range(a.L):
        assert all(np.array_equal(x, y) for x, y in zip(a.samples(hop), b.samples(hop)))


def test_schedule_depends_on_seed_worker_epoch(orc, small):
    ref = build(orc, small).input_nodes()[0]
    assert np.array_equal(ref, build(orc, small).input_nodes()[0])
    for kw in (dict(s0=4), dict(worker=2), dict(epoch=3)):
        other = build(orc, small, **kw).input_nodes()[0]
        assert other.size != ref.size or not np.array_equal(other, ref)


def test_degenerate_inputs(orc, small):
    w, indptr, indices, train = small
    empty = orc.Schedule(indptr, indices, np.zeros(0, np.int32), 16, [3, 2])
    assert empty.n_batches == 0 and empty.input_nodes()[0].size == 0
    nohop = orc.Schedule(indptr, indices, train[:10], 4, [])
    assert nohop.n_batches == 3 and np.array_equal(nohop.input_nodes()[0], orc.epoch_seeds(train[:10], 0, 0, 0))
    zero = orc.Schedule(indptr, indices, train[:10], 4, [0, 0])
    assert np.array_equal(zero.input_nodes()[0], zero.seeds()[0])       # fan-out 0 adds nothing
    one = orc.Schedule(indptr, indices, train[:1], 1000, [2])
    assert one.n_batches == 1


def test_stored_digest_of_the_oracle_is_unchanged(orc):
    """Regression guard (not a pin): the oracle's outputs on the integer-only graph still
    hash to what tests/golden/make_oracle_digest.py stored."""
    import importlib.util
    import json
    import os
    here = os.path.dirname(os.path.abspath(__file__))
    spec = importlib.util.spec_from_file_location("make_oracle_digest", os.path.join(here, "golden", "make_oracle_digest.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    with open(os.path.join(here, "golden", "oracle_digest.json")) as fh:
        stored = json.load(fh)
    assert stored["params"] == mod.PARAMS
    assert stored["digests"] == mod.digests()
