"""ctypes front end of the CPU oracle (rapidgnn_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The product package never imports this module
and this module never imports the product package.

The wrappers only marshal numpy arrays; every piece of arithmetic is in the C
file, where each function cites the passage of the paper it follows.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rapidgnn_oracle.c")
_LIB = os.path.join(_HERE, "librapidgnn_oracle.so")


def build(force=False):
    """Compile the oracle with gcc (-O2, OpenMP only for the threaded timing leg)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp",
                               "-Wall", "-Wextra", "-o", _LIB, _SRC])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        u64, u32, i64, i32, vp = C.c_uint64, C.c_uint32, C.c_int64, C.c_int32, C.c_void_p
        L.orc_mix64.restype = u64; L.orc_mix64.argtypes = [u64]
        L.orc_combine.restype = u64; L.orc_combine.argtypes = [u64, u64]
        L.orc_batch_seed.restype = u64; L.orc_batch_seed.argtypes = [u64, u32, u32, u32]
        L.orc_hop_state.restype = u64; L.orc_hop_state.argtypes = [u64, u32]
        L.orc_node_state.restype = u64; L.orc_node_state.argtypes = [u64, i32]
        L.orc_epoch_state.restype = u64; L.orc_epoch_state.argtypes = [u64, u32, u32]
        L.orc_key32.restype = u32; L.orc_key32.argtypes = [u64, i32]
        L.orc_num_batches.restype = u64; L.orc_num_batches.argtypes = [u64, u64]
        L.orc_epoch_seeds.restype = C.c_int; L.orc_epoch_seeds.argtypes = [vp, u64, u64, u32, u32, vp]
        L.orc_sample_row.restype = u32; L.orc_sample_row.argtypes = [vp, i64, u32, u64, vp, vp]
        L.orc_build_schedule.restype = vp
        L.orc_build_schedule.argtypes = [i64, vp, vp, vp, u64, u32, vp, u32, u64, u32, u32, u32, u32, C.c_int]
        L.orc_build_schedule_with.restype = vp
        L.orc_build_schedule_with.argtypes = [i64, vp, vp, vp, u64, u32, vp, u32, u64, u32, u32, u32, u32, C.c_int, C.c_int]
        L.orc_feistel.restype = u64; L.orc_feistel.argtypes = [u64, u32, u64]
        L.orc_draw_positions.restype = None; L.orc_draw_positions.argtypes = [i64, u32, u64, vp]
        L.orc_sample_row_positions.restype = u32; L.orc_sample_row_positions.argtypes = [vp, i64, u32, u64, vp, vp]
        L.orc_schedule_destroy.restype = None; L.orc_schedule_destroy.argtypes = [vp]
        L.orc_schedule_n_batches.restype = u32; L.orc_schedule_n_batches.argtypes = [vp]
        L.orc_schedule_hops.restype = u32; L.orc_schedule_hops.argtypes = [vp]
        L.orc_schedule_frontier_size.restype = i64; L.orc_schedule_frontier_size.argtypes = [vp, u32]
        L.orc_schedule_samples_size.restype = i64; L.orc_schedule_samples_size.argtypes = [vp, u32]
        L.orc_schedule_get_frontier.restype = None; L.orc_schedule_get_frontier.argtypes = [vp, u32, vp, vp]
        L.orc_schedule_get_samples.restype = None; L.orc_schedule_get_samples.argtypes = [vp, u32, vp, vp]
        L.orc_schedule_get_block.restype = C.c_int; L.orc_schedule_get_block.argtypes = [vp, u32, vp]
        L.orc_frequency.restype = None; L.orc_frequency.argtypes = [vp, u32, i64, vp]
        L.orc_top_hot.restype = i64; L.orc_top_hot.argtypes = [vp, vp, i64, u64, vp, vp]
        L.orc_cache_fill.restype = None
        L.orc_cache_fill.argtypes = [vp, i64, vp, vp, vp, u64, vp, u64, u32, vp, u64]
        L.orc_gather_batch.restype = i64
        L.orc_gather_batch.argtypes = [vp, u32, vp, vp, vp, u64, vp, u64, u32, vp, u64]
        L.orc_batch_stats.restype = None; L.orc_batch_stats.argtypes = [vp, u32, vp, vp, vp]
        L.orc_max_threads.restype = C.c_int; L.orc_max_threads.argtypes = []
        _lib = L
    return _lib


def _p(a):
    return a.ctypes.data_as(C.c_void_p) if a is not None else None


def _arr(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


# ---- hash family -----------------------------------------------------------
def mix64(x): return lib().orc_mix64(int(x) & (2**64 - 1))
def combine(h, x): return lib().orc_combine(int(h) & (2**64 - 1), int(x) & (2**64 - 1))
def batch_seed(s0, w, e, i): return lib().orc_batch_seed(int(s0), int(w), int(e), int(i))
def hop_state(bs, hop): return lib().orc_hop_state(int(bs), int(hop))
def node_state(hs, v): return lib().orc_node_state(int(hs), int(v))
def epoch_state(s0, w, e): return lib().orc_epoch_state(int(s0), int(w), int(e))
def key32(s, u): return lib().orc_key32(int(s), int(u))
def num_batches(T, B): return lib().orc_num_batches(int(T), int(B))
def max_threads(): return lib().orc_max_threads()


def epoch_seeds(train, s0, w, e):
    train = _arr(train, np.int32)
    out = np.empty_like(train)
    rc = lib().orc_epoch_seeds(_p(train), train.size, int(s0), int(w), int(e), _p(out))
    assert rc == 0
    return out


def sample_row(row, f, s):
    row = _arr(row, np.int32)
    heap = np.empty(max(int(f), 1), np.uint64)
    out = np.empty(max(min(int(f), row.size), 1), np.int32)
    m = lib().orc_sample_row(_p(row), row.size, int(f), int(s), _p(heap), _p(out))
    return out[:m].copy()


def feistel(x, n_bits, s): return lib().orc_feistel(int(x), int(n_bits), int(s) & (2**64 - 1))


def draw_positions(deg, f, s):
    """f distinct positions in [0, deg), deg > f, in draw order (the O(f) alternative sampler)."""
    assert deg > f >= 1
    pos = np.empty(f, np.int64)
    lib().orc_draw_positions(int(deg), int(f), int(s) & (2**64 - 1), _p(pos))
    return pos


def sample_row_positions(row, f, s):
    row = _arr(row, np.int32)
    out = np.empty(max(min(row.size, f), 1), np.int32)
    pos = np.empty(max(f, 1), np.int64)
    m = lib().orc_sample_row_positions(_p(row), row.size, int(f), int(s) & (2**64 - 1), _p(pos), _p(out))
    return out[:m].copy()


class Schedule:
    """One epoch's schedule: seeds, frontiers U_0..U_L and per-hop samples."""

    def __init__(self, indptr, indices, train, batch_size, fanout, s0=0, worker=0, epoch=0,
                 batch_lo=0, batch_hi=0, n_threads=1, sampler="keys"):
        self.indptr = _arr(indptr, np.int64)
        self.indices = _arr(indices, np.int32)
        train = _arr(train, np.int32)
        fan = _arr(fanout, np.uint32)
        self.n_nodes = self.indptr.size - 1
        self.h = lib().orc_build_schedule_with(self.n_nodes, _p(self.indptr), _p(self.indices), _p(train),
                                               train.size, int(batch_size), _p(fan), fan.size, int(s0),
                                               int(worker), int(epoch), int(batch_lo), int(batch_hi),
                                               int(n_threads), {"keys": 0, "positions": 1}[sampler])
        if not self.h:
            raise RuntimeError("orc_build_schedule failed")
        self.n_batches = lib().orc_schedule_n_batches(self.h)
        self.L = lib().orc_schedule_hops(self.h)

    def __del__(self):
        if getattr(self, "h", None) and _lib is not None:
            _lib.orc_schedule_destroy(self.h)
            self.h = None

    def frontier(self, hop):
        n = lib().orc_schedule_frontier_size(self.h, hop)
        ids = np.empty(n, np.int32)
        off = np.empty(self.n_batches + 1, np.int64)
        lib().orc_schedule_get_frontier(self.h, hop, _p(ids), _p(off))
        return ids, off

    def samples(self, hop):
        n = lib().orc_schedule_frontier_size(self.h, hop)
        m = lib().orc_schedule_samples_size(self.h, hop)
        off = np.empty(n + 1, np.int64)
        nbr = np.empty(m, np.int32)
        lib().orc_schedule_get_samples(self.h, hop, _p(off), _p(nbr))
        return off, nbr

    def block(self, hop):
        """src_pos: position in the batch's U_{hop+1} of every sampled neighbour of hop `hop`."""
        if not 0 <= hop < self.L:
            raise RuntimeError(f"block of hop {hop}: the schedule has hops 0..{self.L - 1}")
        pos = np.empty(lib().orc_schedule_samples_size(self.h, hop), np.int32)
        if lib().orc_schedule_get_block(self.h, hop, _p(pos)) != 0:
            raise RuntimeError("orc_schedule_get_block failed")
        return pos

    def seeds(self):
        return self.frontier(0)

    def input_nodes(self):
        return self.frontier(self.L)


def frequency(schedules, n_nodes):
    hs = (C.c_void_p * len(schedules))(*[s.h for s in schedules])
    freq = np.empty(n_nodes, np.uint32)
    lib().orc_frequency(hs, len(schedules), n_nodes, _p(freq))
    return freq


def top_hot(freq, is_local, K):
    freq = _arr(freq, np.uint32)
    is_local = _arr(is_local, np.uint8)
    n = freq.size
    ids = np.empty(max(min(int(K), n), 1), np.int32)
    slot_of = np.empty(n, np.int32)
    k_eff = lib().orc_top_hot(_p(freq), _p(is_local), n, int(K), _p(ids), _p(slot_of))
    assert k_eff >= 0
    return ids[:k_eff].copy(), slot_of


class Features:
    """Byte view of the feature tables: X[v] = local[row_of[v]] or remote[row_of[v]]."""

    def __init__(self, is_local, row_of, local_rows, local_stride, remote_rows, remote_stride, row_bytes):
        self.is_local = _arr(is_local, np.uint8)
        self.row_of = _arr(row_of, np.int32)
        self.local_rows = np.ascontiguousarray(local_rows).view(np.uint8).reshape(-1)
        self.remote_rows = np.ascontiguousarray(remote_rows).view(np.uint8).reshape(-1)
        self.local_stride, self.remote_stride, self.row_bytes = int(local_stride), int(remote_stride), int(row_bytes)


def cache_fill(cache_ids, f, table_stride=None):
    cache_ids = _arr(cache_ids, np.int32)
    table_stride = int(table_stride or f.row_bytes)
    table = np.zeros(max(cache_ids.size * table_stride, 1), np.uint8)
    lib().orc_cache_fill(_p(cache_ids), cache_ids.size, _p(f.is_local), _p(f.row_of), _p(f.local_rows),
                         f.local_stride, _p(f.remote_rows), f.remote_stride, f.row_bytes, _p(table), table_stride)
    return table[:cache_ids.size * table_stride].reshape(cache_ids.size, table_stride)


def gather_batch(sched, batch, f, out_stride=None, fill=0):
    ids, off = sched.input_nodes()
    m = int(off[batch + 1] - off[batch])
    out_stride = int(out_stride or f.row_bytes)
    out = np.full(max(m * out_stride, 1), fill, np.uint8)
    got = lib().orc_gather_batch(sched.h, batch, _p(f.is_local), _p(f.row_of), _p(f.local_rows), f.local_stride,
                                 _p(f.remote_rows), f.remote_stride, f.row_bytes, _p(out), out_stride)
    assert got == m
    return out[:m * out_stride].reshape(m, out_stride)


def batch_stats(sched, batch, is_local, slot_of=None):
    is_local = _arr(is_local, np.uint8)
    so = _arr(slot_of, np.int32) if slot_of is not None else None
    st = np.zeros(4, np.uint64)
    lib().orc_batch_stats(sched.h, batch, _p(is_local), _p(so), _p(st))
    return dict(n_rows=int(st[0]), n_local=int(st[1]), n_hit=int(st[2]), n_miss=int(st[3]))
