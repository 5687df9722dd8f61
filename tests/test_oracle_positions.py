"""Pins for the oracle's O(f) alternative sampler: f distinct positions of the row are drawn and only those are
read.  The paper fixes SAMPLE's law (uniform, without replacement; Prop. 1(a)), not its procedure; these tests pin
the procedure chosen here to that law and to what makes it well defined (a keyed permutation, a selection without
replacement)."""
import numpy as np
import pytest

from paper_2509_05207_amd import synth

G = 0x9E3779B97F4A7C15
M64 = 2**64 - 1


def states(orc, n, salt=0):
    return [orc.mix64((i + 1 + salt * 1000003) * G & M64) for i in range(n)]


@pytest.mark.parametrize("n_bits", [1, 2, 3, 4, 5, 7, 8, 11, 12])
def test_feistel_is_a_permutation_of_all_n_bit_values(orc, n_bits):
    for s in states(orc, 5, n_bits):
        images = sorted(orc.feistel(x, n_bits, s) for x in range(1 << n_bits))
        assert images == list(range(1 << n_bits))


def test_feistel_depends_on_the_key(orc):
    a = [orc.feistel(x, 10, 1) for x in range(64)]
    b = [orc.feistel(x, 10, 2) for x in range(64)]
    assert a != b and a != list(range(64))


@pytest.mark.parametrize("deg", [2, 3, 17, 63, 64, 65, 66, 100, 128, 129, 1000, 4097])
def test_positions_are_distinct_in_range_and_exhaust_the_row(orc, deg):
    for s in states(orc, 4, deg):
        pos = orc.draw_positions(deg, deg - 1, s)                  # all but one position: the permutation walked to its end
        assert pos.min() >= 0 and pos.max() < deg
        assert np.unique(pos).size == deg - 1


@pytest.mark.parametrize("deg", [9, 64, 65, 700])
def test_draws_are_a_sequence_smaller_fanout_is_a_prefix(orc, deg):
    s = states(orc, 1, deg)[0]
    full = orc.draw_positions(deg, deg - 1, s)
    for f in (1, 2, 5, deg // 2):
        assert np.array_equal(orc.draw_positions(deg, f, s), full[:f])


@pytest.mark.parametrize("deg", [2, 5, 13, 40, 64])
def test_short_rows_follow_selection_without_replacement(orc, deg):
    """deg <= 64: draw t takes the r_t-th position still free, r_t = floor(u_t * (deg - t)) with u_t the draw's 32-bit
    fraction: written here with an explicit list of free positions."""
    for s in states(orc, 6, deg):
        free = list(range(deg))
        want = []
        for t in range(deg - 1):
            u = orc.mix64((s + (t + 1) * G) & M64) >> 32
            want.append(free.pop((u * (deg - t)) >> 32))
        assert orc.draw_positions(deg, deg - 1, s).tolist() == want


def inclusion_counts(orc, deg, f, n):
    inc = np.zeros((n, deg), bool)
    for i, s in enumerate(states(orc, n, deg * 131 + f)):
        inc[i, orc.draw_positions(deg, f, s)] = True
    return inc


@pytest.mark.parametrize("deg,f", [(5, 1), (5, 2), (6, 5), (13, 5), (23, 10), (64, 12), (65, 12), (100, 25), (257, 10), (1000, 25), (6000, 10)])
def test_every_position_is_included_with_probability_f_over_deg(orc, deg, f):
    """Prop. 1(a): the marginal law of the sample is that of uniform sampling without replacement."""
    n = 12000
    inc = inclusion_counts(orc, deg, f, n)
    cnt = inc.sum(axis=0).astype(float)
    exp = n * f / deg
    chi2 = ((cnt - exp) ** 2 / exp).sum() / (1 - f / deg)           # an inclusion indicator has variance p(1-p)
    z = (chi2 - (deg - 1)) / np.sqrt(2 * (deg - 1))
    assert abs(z) < 4.5, (deg, f, z)


@pytest.mark.parametrize("deg,f", [(5, 2), (8, 3), (13, 5), (33, 7), (64, 12), (65, 12), (100, 25)])
def test_pairs_of_positions_are_included_together_as_often_as_they_should(orc, deg, f):
    """Without replacement: P(p and q both drawn) = f(f-1) / (deg(deg-1)) for every pair."""
    n = 12000
    inc = inclusion_counts(orc, deg, f, n).astype(np.float64)
    co = inc.T @ inc
    iu = np.triu_indices(deg, 1)
    p = f * (f - 1) / (deg * (deg - 1))
    z = (co[iu] - n * p) / np.sqrt(n * p * (1 - p))
    assert np.abs(z).max() < 5.0, (deg, f, np.abs(z).max())
    assert abs(z.mean()) < 0.5


def test_row_sample_reads_the_drawn_positions_or_the_whole_row(orc):
    row = np.arange(1000, 1300, 3, dtype=np.int32)                  # 100 neighbours
    s = states(orc, 1)[0]
    assert np.array_equal(orc.sample_row_positions(row, 100, s), row)      # deg <= f: the row, in order
    assert np.array_equal(orc.sample_row_positions(row, 500, s), row)
    got = orc.sample_row_positions(row, 7, s)
    assert np.array_equal(got, row[orc.draw_positions(100, 7, s)])
    assert orc.sample_row_positions(row, 0, s).size == 0
    assert orc.sample_row_positions(np.empty(0, np.int32), 5, s).size == 0


def test_schedule_built_with_the_position_sampler(orc):
    """Same seeds, hop states, frontier rule and counts as the main reading; only SAMPLE differs."""
    w = synth.make_workload("small")
    indptr, indices, train = w.indptr.numpy(), w.indices.numpy(), w.train.numpy()
    a = orc.Schedule(indptr, indices, train, w.cfg.batch_size, w.cfg.fanout, 4, 1, 2, sampler="positions")
    k = orc.Schedule(indptr, indices, train, w.cfg.batch_size, w.cfg.fanout, 4, 1, 2)
    assert np.array_equal(a.seeds()[0], k.seeds()[0]) and np.array_equal(a.seeds()[1], k.seeds()[1])
    differs = False
    for hop in range(a.L):
        ids, off = a.frontier(hop)
        nxt, noff = a.frontier(hop + 1)
        so, nbr = a.samples(hop)
        for b in range(a.n_batches):
            hs = orc.hop_state(orc.batch_seed(4, 1, 2, b), hop)
            seen = set(ids[off[b]:off[b + 1]].tolist())
            fresh = set()
            for j in range(off[b], off[b + 1]):
                v = int(ids[j])
                row = indices[indptr[v]:indptr[v + 1]]
                got = nbr[so[j]:so[j + 1]]
                want = orc.sample_row_positions(row, w.cfg.fanout[hop], orc.node_state(hs, v))
                assert np.array_equal(got, want)
                assert got.size == min(row.size, w.cfg.fanout[hop]) and np.unique(got).size == got.size
                fresh.update(int(u) for u in got if int(u) not in seen)
            seg = nxt[noff[b]:noff[b + 1]]
            assert np.array_equal(seg[:off[b + 1] - off[b]], ids[off[b]:off[b + 1]])
            assert seg[off[b + 1] - off[b]:].tolist() == sorted(fresh)
        if hop == 0:
            differs = not np.array_equal(nbr, k.samples(0)[1])
    assert differs                                                    # it is a different sample from the main reading's
    assert a.block(0).size == a.samples(0)[1].size                    # blocks work on either schedule
