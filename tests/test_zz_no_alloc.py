"""The entry point that allocates nothing (rg_gather_batch_noalloc) against rg_gather_batch, through the C ABI.

Both classify a batch on the fly; one takes its routing entries and counters from an allocation, the other from the
array built into the library.  Bytes and counts must be identical, call after call, also when a smaller batch
follows a larger one in the same scratch."""
import numpy as np
import pytest
import torch

from paper_2509_05207_amd import synth

pytestmark = pytest.mark.gpu

SENTINEL = 0xA5


@pytest.fixture(scope="module")
def rg():
    from paper_2509_05207_amd import binding
    binding.lib()
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return binding


def np_bytes(t):
    return t.contiguous().view(torch.uint8).cpu().numpy()


@pytest.mark.parametrize("name,pinned", [("mid", False), ("mid_bf16", True)])
def test_noalloc_equals_gather_batch_on_consecutive_calls(rg, orc, name, pinned):
    w = synth.make_workload(name)
    cfg = w.cfg
    d = "cuda"
    indptr, indices, train = w.indptr.to(d), w.indices.to(d), w.train.to(d)
    s = rg.rg_build_schedule(indptr, indices, train, cfg.batch_size, cfg.fanout, 3, 1, 0)
    other = rg.rg_build_schedule(indptr, indices, train, cfg.batch_size, cfg.fanout, 3, 1, 1)
    remote = w.remote_rows.pin_memory() if pinned else w.remote_rows.to(d)
    feat = rg.make_features(w.is_local.to(d), w.row_of.to(d), w.local_rows.to(d), remote, w.row_bytes)
    cache_of_other = rg.rg_build_cache([other], feat, w.K)          # no plan for `s`: both entry points classify on the fly
    o = orc.Schedule(w.indptr.numpy(), w.indices.numpy(), w.train.numpy(), cfg.batch_size, cfg.fanout, 3, 1, 0, n_threads=4)
    ofeat = orc.Features(w.is_local.numpy(), w.row_of.numpy(), np_bytes(w.local_rows), w.stride_bytes, np_bytes(w.remote_rows),
                         w.stride_bytes, w.row_bytes)
    _, off = o.input_nodes()
    sizes = np.diff(off)
    big, small = int(np.argmax(sizes)), s.n_batches - 1            # the largest batch, then the ragged last one
    assert sizes[small] < sizes[big]
    out_stride = w.stride_bytes + 16                                 # padding that must stay untouched
    cap = int(sizes.max()) + 3
    for c in (None, cache_of_other):
        for b in (big, small):                                       # two calls in a row, the second with the smaller input
            ref = torch.full((cap * out_stride,), SENTINEL, dtype=torch.uint8, device=d)
            got = torch.full((cap * out_stride,), SENTINEL, dtype=torch.uint8, device=d)
            st_ref = rg.rg_gather_batch(s, c, feat, b, ref, out_stride=out_stride, out_capacity_rows=cap)
            st_got = rg.rg_gather_batch_noalloc(s, c, feat, b, got, out_stride=out_stride, out_capacity_rows=cap)
            torch.cuda.synchronize()
            assert st_got == st_ref, (name, b)
            assert torch.equal(got, ref), (name, b)
            m = int(sizes[b])
            rows = got.cpu().numpy().reshape(cap, out_stride)
            want = orc.gather_batch(o, b, ofeat, out_stride=out_stride, fill=SENTINEL)
            assert np.array_equal(rows[:m], want)
            assert (rows[m:] == SENTINEL).all()
            # without stats the call only enqueues work: same bytes once the stream has drained
            again = torch.full((cap * out_stride,), SENTINEL, dtype=torch.uint8, device=d)
            assert rg.rg_gather_batch_noalloc(s, c, feat, b, again, out_stride=out_stride, out_capacity_rows=cap, want_stats=False) is None
            torch.cuda.synchronize()
            assert torch.equal(again, ref)


def test_noalloc_refuses_what_does_not_fit(rg):
    d = "cuda"
    # a batch of RG_NOALLOC_MAX_ROWS + 1 seeds and no hops: its input set is one row too many for the built-in scratch
    n = rg.RG_NOALLOC_MAX_ROWS + 1
    indptr = torch.zeros(n + 1, dtype=torch.int64, device=d)
    indices = torch.zeros(0, dtype=torch.int32, device=d)
    train = torch.arange(n, dtype=torch.int32, device=d)
    s = rg.rg_build_schedule(indptr, indices, train, n, [], 0, 0, 0)
    is_local = torch.ones(n, dtype=torch.uint8, device=d)
    row_of = torch.zeros(n, dtype=torch.int32, device=d)
    table = torch.zeros((1, 4), dtype=torch.float32, device=d)
    feat = rg.make_features(is_local, row_of, table, table, 16)
    out = torch.full((64,), SENTINEL, dtype=torch.uint8, device=d)
    with pytest.raises(rg.RgError) as e:
        rg.rg_gather_batch_noalloc(s, None, feat, 0, out, out_stride=16, out_capacity_rows=n)
    assert e.value.status == rg.RG_ERANGE and "RG_NOALLOC_MAX_ROWS" in str(e.value)
    # one seed fewer fits the scratch but not this output buffer
    s2 = rg.rg_build_schedule(indptr, indices, train[:-1], n - 1, [], 0, 0, 0)
    with pytest.raises(rg.RgError) as e:
        rg.rg_gather_batch_noalloc(s2, None, feat, 0, out, out_stride=16, out_capacity_rows=4)
    assert e.value.status == rg.RG_ERANGE
    with pytest.raises(rg.RgError) as e:
        rg.rg_gather_batch_noalloc(s2, None, feat, 1, out, out_stride=16, out_capacity_rows=4)
    assert e.value.status == rg.RG_ERANGE
    torch.cuda.synchronize()
    assert bool((out == SENTINEL).all())


def test_noalloc_at_the_scratch_limit(rg):
    """A batch of exactly RG_NOALLOC_MAX_ROWS rows: the last routing entry is the last 8 bytes of the scratch array."""
    d = "cuda"
    n = rg.RG_NOALLOC_MAX_ROWS
    indptr = torch.zeros(n + 1, dtype=torch.int64, device=d)
    indices = torch.zeros(0, dtype=torch.int32, device=d)
    train = torch.arange(n, dtype=torch.int32, device=d)
    s = rg.rg_build_schedule(indptr, indices, train, n, [], 0, 0, 0)
    is_local = (torch.arange(n, device=d) % 3 == 0).to(torch.uint8)
    loc = is_local.to(torch.int64)
    row_of = torch.where(loc == 1, torch.cumsum(loc, 0) - 1, torch.cumsum(1 - loc, 0) - 1).to(torch.int32)
    n_local = int(loc.sum().item())
    local = torch.arange(n_local * 4, dtype=torch.int32, device=d).reshape(n_local, 4)
    remote = -torch.arange((n - n_local) * 4, dtype=torch.int32, device=d).reshape(n - n_local, 4) - 1
    feat = rg.make_features(is_local, row_of, local, remote, 16)
    out = torch.empty((n, 4), dtype=torch.int32, device=d)
    st = rg.rg_gather_batch_noalloc(s, None, feat, 0, out, out_stride=16, out_capacity_rows=n)
    ids = rg.rg_schedule_frontier(s, 0)[0].long()
    want = torch.where((is_local[ids] == 1)[:, None], local[row_of[ids].long() * (is_local[ids] == 1)],
                       remote[row_of[ids].long() * (is_local[ids] == 0)])
    assert torch.equal(out, want)
    assert st == dict(n_rows=n, n_local=n_local, n_hit=0, n_miss=n - n_local)
