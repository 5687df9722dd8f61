"""Pins for the oracle's computation blocks (Sec. 4 par. (8): the sampled subgraph of every hop, relabelled
to positions in the batch's node list, as a trainer consumes it)."""
import numpy as np
import pytest

from paper_2509_05207_amd import synth


@pytest.fixture(scope="module", params=["small", "tiny"])
def built(request, orc):
    w = synth.make_workload(request.param)
    s = orc.Schedule(w.indptr.numpy(), w.indices.numpy(), w.train.numpy(), w.cfg.batch_size, w.cfg.fanout, 5, 0, 1)
    return w, s


def per_batch(s, hop):
    """Yields (U_hop of the batch, U_{hop+1} of the batch, per-destination sample offsets, sampled IDs, positions)."""
    ids0, off0 = s.frontier(hop)
    ids1, off1 = s.frontier(hop + 1)
    so, nbr = s.samples(hop)
    pos = s.block(hop)
    for b in range(s.n_batches):
        p0, p1 = off0[b], off0[b + 1]
        k0, k1 = so[p0], so[p1]
        yield ids0[p0:p1], ids1[off1[b]:off1[b + 1]], so[p0:p1 + 1] - k0, nbr[k0:k1], pos[k0:k1]


def test_positions_invert_the_batch_node_list(built):
    _, s = built
    for hop in range(s.L):
        for dst, src, indptr, nbr, pos in per_batch(s, hop):
            assert pos.size == nbr.size == indptr[-1]
            assert np.all((pos >= 0) & (pos < src.size))
            assert np.array_equal(src[pos], nbr)                    # the definition, read backwards
            assert np.array_equal(src[:dst.size], dst)              # destination j is source j


def test_positions_match_a_dictionary_lookup(built):
    _, s = built
    for hop in range(s.L):
        for _, src, _, nbr, pos in per_batch(s, hop):
            where = {int(v): j for j, v in enumerate(src)}
            assert len(where) == src.size                           # a node list has no repeats, so positions are unique
            assert [where[int(u)] for u in nbr] == pos.tolist()


def test_block_edges_are_graph_edges_between_the_right_nodes(built):
    w, s = built
    indptr, indices = w.indptr.numpy(), w.indices.numpy()
    for hop in range(s.L):
        for dst, src, bptr, _, pos in per_batch(s, hop):
            for j in range(dst.size):
                row = indices[indptr[dst[j]]:indptr[dst[j] + 1]]
                got = src[pos[bptr[j]:bptr[j + 1]]]
                assert got.size == min(row.size, w.cfg.fanout[hop])
                assert np.all(np.isin(got, row))


def test_aggregation_over_a_block_equals_aggregation_over_global_ids(built):
    """A mean-aggregation layer run on block-local indices sees the same neighbours as one run on graph IDs."""
    w, s = built
    rng = np.random.default_rng(0)
    X = rng.integers(-1000, 1000, size=(w.n_nodes, 3)).astype(np.int64)
    for hop in range(s.L):
        for dst, src, bptr, nbr, pos in per_batch(s, hop):
            H = X[src]                                              # the gathered block, in batch order
            a = np.add.reduceat(np.vstack([H[pos], np.zeros((1, 3), np.int64)]), np.minimum(bptr[:-1], pos.size), axis=0)
            b = np.add.reduceat(np.vstack([X[nbr], np.zeros((1, 3), np.int64)]), np.minimum(bptr[:-1], nbr.size), axis=0)
            empty = bptr[1:] == bptr[:-1]
            a[empty] = 0
            b[empty] = 0
            assert np.array_equal(a, b)


def test_block_of_a_hop_beyond_the_last_is_refused(built):
    _, s = built
    with pytest.raises(RuntimeError):
        s.block(s.L)
