"""Pins for the oracle's per-node sampler SAMPLE(eta(v), f) (Sec. 2.1 node-wise
sampling; Sec. 4 par. (2); Prop. 1).  Brute force, invariants and the
statistics Prop. 1(a)/(b) state."""
import numpy as np
import pytest


def brute_force(orc, row, f, s):
    """Definition written out: every composite key, one full sort, first f, back to row order."""
    comp = [((orc.key32(s, int(u)) << 32) | int(u), j) for j, u in enumerate(row)]
    comp.sort()
    keep = sorted(j for _, j in comp[:f])
    return np.array([row[j] for j in keep], dtype=np.int32)


def state(orc, s0=0, w=0, e=0, i=0, hop=0, v=0):
    return orc.node_state(orc.hop_state(orc.batch_seed(s0, w, e, i), hop), v)


@pytest.mark.parametrize("deg,f", [(1, 1), (5, 5), (6, 5), (7, 3), (64, 10), (65, 64), (200, 1), (1000, 25),
                                   (4097, 50), (300, 299)])
def test_equals_brute_force(orc, deg, f):
    rng = np.random.default_rng(deg * 131 + f)
    for trial in range(4):
        row = np.sort(rng.choice(1 << 20, size=deg, replace=False)).astype(np.int32)
        s = state(orc, i=trial, v=int(row[0]))
        got = orc.sample_row(row, f, s)
        assert np.array_equal(got, brute_force(orc, row, f, s))


def test_invariants_subset_size_no_duplicates_row_order(orc):
    rng = np.random.default_rng(3)
    for _ in range(50):
        deg = int(rng.integers(0, 400))
        f = int(rng.integers(0, 40))
        row = np.sort(rng.choice(100000, size=deg, replace=False)).astype(np.int32)
        got = orc.sample_row(row, f, state(orc, v=deg, i=f))
        assert got.size == min(deg, f)
        assert np.unique(got).size == got.size
        assert np.isin(got, row).all()
        assert np.all(np.diff(got) > 0)          # row order == ascending for a sorted row


def test_small_rows_and_zero_fanout(orc):
    row = np.array([3, 9, 27], np.int32)
    assert np.array_equal(orc.sample_row(row, 3, 1), row)
    assert np.array_equal(orc.sample_row(row, 10, 1), row)
    assert orc.sample_row(row, 0, 1).size == 0
    assert orc.sample_row(np.zeros(0, np.int32), 5, 1).size == 0


def test_sample_is_a_function_of_the_neighbour_set_not_of_storage_order(orc):
    rng = np.random.default_rng(4)
    row = np.sort(rng.choice(50000, size=300, replace=False)).astype(np.int32)
    s = state(orc, v=5)
    ref = set(orc.sample_row(row, 17, s).tolist())
    for _ in range(5):
        shuffled = rng.permutation(row).astype(np.int32)
        got = orc.sample_row(shuffled, 17, s)
        assert set(got.tolist()) == ref
        pos = {int(u): j for j, u in enumerate(shuffled)}
        assert all(pos[int(a)] < pos[int(b)] for a, b in zip(got[:-1], got[1:]))   # emitted in row order


def test_deterministic_and_stream_dependent(orc):
    row = np.arange(1000, 1400, dtype=np.int32)
    base = dict(s0=5, w=1, e=2, i=3, hop=1, v=77)
    ref = orc.sample_row(row, 20, state(orc, **base))
    assert np.array_equal(ref, orc.sample_row(row, 20, state(orc, **base)))
    for k in base:
        other = dict(base)
        other[k] += 1
        assert not np.array_equal(ref, orc.sample_row(row, 20, state(orc, **other))), k


def test_keys_of_one_node_never_tie(orc):
    """For a fixed node state the key is a bijection of the 32-bit neighbour id (every step is
    invertible), so distinct neighbours have distinct keys and the id half of the composite
    never decides.  The inverse is written here, independently, from the derived constants."""
    from math import isqrt
    G32 = ((isqrt(5 << 128) - (1 << 64)) // 2) >> 32
    A32 = (isqrt(2 << 128) - (1 << 64)) >> 32
    B32 = (isqrt(3 << 128) - (1 << 64)) >> 32
    M = (1 << 32) - 1

    def unkey(s, k):
        lo, hi = s & M, s >> 32
        k ^= k >> 16
        k = (k * pow(B32, -1, 1 << 32)) & M
        k ^= k >> 15
        k ^= k >> 30
        k = (k * pow(A32, -1, 1 << 32)) & M
        k = (k - hi) & M
        k ^= k >> 16
        k = (k * pow(G32, -1, 1 << 32)) & M
        return k ^ lo
    rng = np.random.default_rng(8)
    for _ in range(2000):
        s = int(rng.integers(0, 1 << 63)) * 2 + int(rng.integers(0, 2))
        u = int(rng.integers(0, 1 << 31))
        assert unkey(s, orc.key32(s, u)) == u


def test_prop1a_marginal_is_uniform_without_replacement(orc):
    """Over many batch indices a fixed node with 20 neighbours and fan-out 5 includes each
    neighbour with probability 5/20 and each pair with probability (5*4)/(20*19)."""
    row = (np.arange(20, dtype=np.int32) * 7919 + 13) % 1000003
    row = np.sort(row).astype(np.int32)
    n = 12000
    inc = np.zeros(20)
    pair = np.zeros((20, 20))
    pos = {int(u): j for j, u in enumerate(row)}
    for i in range(n):
        got = orc.sample_row(row, 5, state(orc, s0=11, i=i, v=4242))
        idx = [pos[int(u)] for u in got]
        inc[idx] += 1
        for x in idx:
            for y in idx:
                if x < y:
                    pair[x, y] += 1
    p = inc / n
    sd = np.sqrt(0.25 * 0.75 / n)
    assert np.all(np.abs(p - 0.25) < 4 * sd), p
    # chi-square over neighbours (inclusion counts; variance of a without-replacement draw is smaller,
    # so the plain multinomial bound is conservative)
    chi2 = ((inc - n * 0.25) ** 2 / (n * 0.25)).sum()
    assert chi2 < 19 + 5 * np.sqrt(2 * 19), chi2
    pp = pair[np.triu_indices(20, 1)] / n
    p2 = (5 * 4) / (20 * 19)
    assert np.all(np.abs(pp - p2) < 4.5 * np.sqrt(p2 * (1 - p2) / n)), (pp.min(), pp.max())


def test_prop1b_batches_are_uncorrelated(orc):
    """Inclusion indicators of the same neighbour under two different (e, i, w) tuples are uncorrelated."""
    row = np.arange(500, 540, dtype=np.int32)
    n = 6000
    both = 0
    for t in range(n):
        a = orc.sample_row(row, 10, state(orc, s0=t, i=3, v=9))
        b = orc.sample_row(row, 10, state(orc, s0=t, i=4, v=9))
        both += int(row[0] in a and row[0] in b)
    p = both / n
    assert abs(p - 1 / 16) < 4 * np.sqrt((1 / 16) * (15 / 16) / n), p
