"""GPU parity over many seeded random shapes: graphs whose rows mix every length class of the sampler (empty, shorter
than the fan-out, up to 64, up to 256, a few blocks, many blocks, above the tile size), fan-outs from 1 to several
hundred, one to three hops, ragged last batches -- each schedule against the oracle's, bit for bit, for both samplers."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rg():
    from paper_2509_05207_amd import binding
    binding.lib()
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return binding


def random_graph(rng, n, classes):
    """CSR with rows sorted and duplicate free; a row's length is drawn from one of `classes` (lo, hi, weight)."""
    w = np.array([c[2] for c in classes], dtype=np.float64)
    pick = rng.choice(len(classes), size=n, p=w / w.sum())
    deg = np.array([rng.integers(classes[k][0], classes[k][1] + 1) for k in pick], dtype=np.int64)
    deg = np.minimum(deg, n - 1)
    rows = []
    for v in range(n):
        d = int(deg[v])
        if d == 0:
            rows.append(np.empty(0, np.int32))
            continue
        if d * 3 > n:                                    # dense row: a random subset of all other IDs
            cand = np.delete(np.arange(n, dtype=np.int32), v)
            r = rng.choice(cand, size=d, replace=False)
        else:
            r = np.unique(rng.integers(0, n, size=2 * d + 8))
            r = r[r != v][:d]
        rows.append(np.sort(r).astype(np.int32))
    indptr = np.zeros(n + 1, np.int64)
    indptr[1:] = np.cumsum([r.size for r in rows])
    return indptr, (np.concatenate(rows) if indptr[-1] else np.empty(0, np.int32))


SHAPES = [
    # n, row-length classes (lo, hi, weight), fan-outs, batch size, train nodes
    (600, [(0, 0, 1), (1, 9, 4), (10, 64, 3), (65, 256, 2), (257, 599, 1)], (5, 3), 64, 300),
    (3000, [(1, 30, 5), (31, 200, 3), (201, 1500, 2), (1501, 2999, 0.3)], (10,), 128, 777),
    (3000, [(1, 30, 5), (31, 200, 3), (201, 1500, 2)], (1, 1, 1), 100, 450),
    (5000, [(0, 3, 2), (40, 70, 3), (250, 260, 2), (500, 530, 1), (1000, 1100, 1)], (25, 10), 256, 1000),
    (20000, [(5, 60, 6), (100, 900, 3), (16000, 19999, 0.02)], (15, 10, 5), 512, 2000),          # rows above the tile size
    (2000, [(1, 1999, 1)], (63, 2), 50, 333),
    (2000, [(1, 1999, 1)], (64, 65), 1000, 999),
    (2000, [(1, 1999, 1)], (200, 1), 77, 500),
    (2500, [(300, 2400, 1)], (700,), 40, 100),                                                    # the largest candidate buffers
    (1200, [(0, 0, 5), (1, 2, 1)], (4, 4), 16, 1200),                                             # almost no edges
    (40000, [(2, 12, 8), (13, 40, 2)], (5, 5, 5), 1024, 5000),
    (900, [(64, 64, 1), (65, 65, 1), (256, 256, 1), (257, 257, 1), (63, 63, 1), (255, 255, 1)], (9, 7), 33, 400),   # the class boundaries
    (3000, [(1, 16, 2), (17, 32, 2), (33, 48, 2), (49, 64, 2), (0, 0, 1)], (15, 40, 64), 97, 1500),                 # short rows only: every count of IDs per lane, fan-outs around them
    (1500, [(15, 17, 1), (31, 33, 1), (47, 49, 1), (63, 65, 1)], (16, 1, 63), 64, 1500),                            # the sixteen-lane boundaries
]


@pytest.mark.parametrize("shape", range(len(SHAPES)))
@pytest.mark.parametrize("sampler,maps", [("keys", "auto"), ("keys", "bytes"), ("keys", "bits"), ("keys", "one_row_per_wave"), ("keys", "four_short_rows_per_wave"), ("keys", "four_short_rows_inline"),
                                          ("positions", "auto")])
def test_random_shape(rg, orc, shape, sampler, maps, monkeypatch):
    if maps in ("bytes", "bits"):                        # the form of the reached-ID map, forced (chosen per hop otherwise)
        monkeypatch.setenv("RAPIDGNN_BYTE_MAPS", "1" if maps == "bytes" else "0")
    if maps == "one_row_per_wave":                       # without the kernel that samples four short rows at a time ...
        monkeypatch.setenv("RAPIDGNN_SHORT_ROWS", "0")
    if maps == "four_short_rows_per_wave":               # ... with it in every hop (by default: in hops that mark with byte stores) ...
        monkeypatch.setenv("RAPIDGNN_SHORT_ROWS", "1")
    if maps == "four_short_rows_inline":                 # ... and with the same done inside the other kernel (by default: in hops that mark with atomic ORs)
        monkeypatch.setenv("RAPIDGNN_SHORT_ROWS", "2")
    n, classes, fanout, batch, n_train = SHAPES[shape]
    rng = np.random.default_rng(4000 + shape)
    indptr, indices = random_graph(rng, n, classes)
    train = rng.permutation(n)[:n_train].astype(np.int32)
    s0, worker, epoch = 100 + shape, shape % 3, shape % 5
    o = orc.Schedule(indptr, indices, train, batch, list(fanout), s0, worker, epoch, n_threads=8, sampler=sampler)
    dp, dx, dt = torch.from_numpy(indptr).cuda(), torch.from_numpy(indices).cuda(), torch.from_numpy(train).cuda()
    assert rg.rg_graph_validate(dp, dx) == 0
    code = rg.RG_SAMPLER_KEYS if sampler == "keys" else rg.RG_SAMPLER_POSITIONS
    g = rg.rg_build_schedule_with(dp, dx, dt, batch, list(fanout), s0, worker, epoch, sampler=code)
    assert g.n_batches == o.n_batches and g.L == o.L
    for hop in range(o.L + 1):
        ids, off = o.frontier(hop)
        gids, _, goff = rg.rg_schedule_frontier(g, hop)
        assert np.array_equal(goff, off), f"frontier offsets differ at hop {hop}"
        assert np.array_equal(gids.cpu().numpy(), ids), f"frontier ids differ at hop {hop}"
    for hop in range(o.L):
        so, nb = o.samples(hop)
        gso, gnb = rg.rg_schedule_samples(g, hop)
        assert np.array_equal(gso.cpu().numpy(), so), f"sample offsets differ at hop {hop}"
        assert np.array_equal(gnb.cpu().numpy(), nb), f"sampled neighbours differ at hop {hop}"


@pytest.mark.parametrize("group_tiles", ["1", "0"])
def test_rows_of_several_tiles(rg, orc, group_tiles, monkeypatch):
    """Hub rows on both sides of the tiling threshold and of the tile length, up to three tiles, as seeds and as
    neighbours of many short rows, so that every batch samples them in every hop; with the tile jobs handed out
    grouped by the piece they read, and in frontier order."""
    monkeypatch.setenv("RAPIDGNN_GROUP_TILES", group_tiles)
    rng = np.random.default_rng(77)
    n = 200_000
    hub_deg = [16384, 16385, 40000, 65535, 65536, 65537, 70000, 131072, 131073, 150000, 196608, 199999]
    hubs = rng.permutation(n)[:len(hub_deg)]
    deg = rng.integers(1, 7, size=n)
    rows = [None] * n
    small = rng.integers(0, n, size=(n, 6))
    with_hub = rng.random(n) < 0.3
    for v in range(n):
        r = small[v, :deg[v]]
        if with_hub[v]:
            r = np.append(r, hubs[rng.integers(0, len(hubs))])
        r = np.unique(r)
        rows[v] = r[r != v].astype(np.int32)
    for h, d in zip(hubs, hub_deg):
        cand = np.delete(np.arange(n, dtype=np.int32), h)
        rows[h] = np.sort(rng.choice(cand, size=d, replace=False)).astype(np.int32)
    indptr = np.zeros(n + 1, np.int64)
    indptr[1:] = np.cumsum([r.size for r in rows])
    indices = np.concatenate(rows)
    train = np.concatenate([hubs, rng.permutation(n)[:300]]).astype(np.int32)
    train = train[np.sort(np.unique(train, return_index=True)[1])]
    fanout, batch = [12, 4], 64
    o = orc.Schedule(indptr, indices, train, batch, fanout, 5, 1, 2, n_threads=8)
    dp, dx, dt = torch.from_numpy(indptr).cuda(), torch.from_numpy(indices).cuda(), torch.from_numpy(train).cuda()
    assert rg.rg_graph_validate(dp, dx) == 0
    g = rg.rg_build_schedule(dp, dx, dt, batch, fanout, 5, 1, 2)
    assert g.n_batches == o.n_batches
    for hop in range(o.L + 1):
        ids, off = o.frontier(hop)
        gids, _, goff = rg.rg_schedule_frontier(g, hop)
        assert np.array_equal(goff, off) and np.array_equal(gids.cpu().numpy(), ids), f"frontier {hop}"
    for hop in range(o.L):
        so, nb = o.samples(hop)
        gso, gnb = rg.rg_schedule_samples(g, hop)
        assert np.array_equal(gso.cpu().numpy(), so) and np.array_equal(gnb.cpu().numpy(), nb), f"samples {hop}"
