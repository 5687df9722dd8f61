"""Seeded synthetic workloads: power-law CSR graphs, partitions, train sets, features.

This module only manufactures INPUTS.  It holds none of the method's
arithmetic (no seed derivation, sampling keys, counting, ranking or gathering)
and imports neither the HIP binding nor the CPU oracle; both are fed from it.

The graphs stand in for the datasets the paper trains on (Table 1: Reddit,
OGBN-Products, OGBN-Papers100M), which are not available here: directed
Chung-Lu graphs with a power-law expected-degree sequence of the same node
count, edge count and feature width.  Randomness is a counter-based generator
(the published splitmix64 finaliser over integer counters) evaluated with torch
integer ops, so a workload is a pure function of (config, seed) and can be
produced on the CPU or, for the big ones, on the GPU.
"""
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np
import torch

_M64 = (1 << 64) - 1


def _s64(c):
    c &= _M64
    return c - (1 << 64) if c >= (1 << 63) else c


_SM_GAMMA = _s64(0x9E3779B97F4A7C15)
_SM_M1 = _s64(0xBF58476D1CE4E5B9)
_SM_M2 = _s64(0x94D049BB133111EB)


def _lsr(x, k):
    return (x >> k) & ((1 << (64 - k)) - 1)


def counter_bits(seed: int, stream: int, idx: torch.Tensor) -> torch.Tensor:
    """64 pseudo-random bits per counter value (splitmix64 finaliser), as int64."""
    base = _s64((seed * 0xD1342543DE82EF95 + stream * 0xAF251AF3B0F025B5 + 0x2545F4914F6CDD1D) & _M64)
    z = idx.to(torch.int64) * _SM_GAMMA + base
    z = (z ^ _lsr(z, 30)) * _SM_M1
    z = (z ^ _lsr(z, 27)) * _SM_M2
    z = z ^ _lsr(z, 31)
    return z


def counter_uniform(seed: int, stream: int, idx: torch.Tensor) -> torch.Tensor:
    """float64 uniforms in [0, 1) with 53 random bits."""
    return _lsr(counter_bits(seed, stream, idx), 11).to(torch.float64) * (2.0 ** -53)


@dataclass
class Config:
    name: str
    n_nodes: int
    n_edges: int                 # target number of directed edges after dedup
    gamma: float                 # power-law exponent of the expected-degree sequence
    feat_dtype: str              # "float32" | "bfloat16"
    feat_dim: int
    fanout: List[int]
    batch_size: int
    n_train: int
    cache_frac: Optional[float]  # K as a fraction of the remote node count ...
    cache_k: Optional[int]       # ... or K given directly
    n_parts: int = 4
    local_rows_only: bool = False   # keep adjacency of local rows only (one partition's share)
    gen_seed: int = 1000
    s0: int = 0
    worker: int = 0
    epoch: int = 0


# The five workloads of the benchmark definition (node/edge/feature shapes of
# Table 1's datasets; see the module docstring), plus small ones for tests.
CONFIGS = {
    "tiny": Config("tiny", 10_000, 100_000, 2.1, "float32", 64, [10, 5], 256, 2_000, None, 1_000, gen_seed=1000),
    "medium": Config("medium", 233_000, 114_000_000, 2.1, "float32", 602, [25, 10], 1024, 150_000, 0.10, None,
                     gen_seed=1001),
    "large_sparse": Config("large_sparse", 2_450_000, 124_000_000, 2.3, "float32", 100, [15, 10, 5], 1024,
                           200_000, 0.05, None, gen_seed=1002),
    "fanout_stress": Config("fanout_stress", 2_450_000, 124_000_000, 2.3, "bfloat16", 256, [50, 50], 4096,
                            200_000, 0.20, None, gen_seed=1002),
    "partition_share": Config("partition_share", 111_000_000, 400_000_000, 2.1, "float32", 128, [15, 10], 2048,
                              300_000, None, 40_000_000_000 // 512, local_rows_only=True, gen_seed=1004),
    # test-sized shapes
    "small": Config("small", 3_000, 24_000, 2.1, "float32", 24, [6, 4], 100, 730, None, 300, gen_seed=7),
    "mid": Config("mid", 60_000, 3_000_000, 2.1, "float32", 50, [12, 7, 3], 512, 9_000, 0.10, None, gen_seed=8),
    "mid_bf16": Config("mid_bf16", 40_000, 1_200_000, 2.3, "bfloat16", 77, [20, 20], 1000, 5_500, 0.25, None,
                       gen_seed=9),
}


@dataclass
class Workload:
    cfg: Config
    indptr: torch.Tensor        # int64 [N+1]
    indices: torch.Tensor       # int32 [E], each row ascending, duplicate-free
    train: torch.Tensor         # int32 [T], distinct
    is_local: torch.Tensor      # uint8 [N]
    row_of: torch.Tensor        # int32 [N]
    local_rows: torch.Tensor    # [n_local, stride_elems] feature dtype
    remote_rows: torch.Tensor   # [n_remote, stride_elems]
    row_bytes: int
    stride_bytes: int
    K: int
    extra: dict = field(default_factory=dict)

    @property
    def n_nodes(self):
        return self.cfg.n_nodes


def powerlaw_weights(n: int, gamma: float, n_edges: int) -> np.ndarray:
    """Expected-degree weights w_r ~ (r+1)^(-1/(gamma-1)), capped so that no
    expected degree exceeds n/2 at the target edge count."""
    alpha = 1.0 / (gamma - 1.0)
    w = np.arange(1, n + 1, dtype=np.float64) ** (-alpha)
    for _ in range(8):
        cap = (n / 2.0) * w.sum() / max(n_edges, 1)
        if w[0] <= cap:
            break
        w = np.minimum(w, cap)
    return w


def _draw_edges(cfg: Config, n_draw: int, cdf_row, cdf_col, perm, device, chunk=1 << 26):
    n = cfg.n_nodes
    keys = []
    for lo in range(0, n_draw, chunk):
        idx = torch.arange(lo, min(lo + chunk, n_draw), dtype=torch.int64, device=device)
        rv = torch.searchsorted(cdf_row, counter_uniform(cfg.gen_seed, 11, idx)).clamp_(max=n - 1)
        ru = torch.searchsorted(cdf_col, counter_uniform(cfg.gen_seed, 12, idx)).clamp_(max=n - 1)
        v, u = perm[rv], perm[ru]
        keep = v != u
        keys.append((v * n + u)[keep])
        del idx, rv, ru, v, u, keep
    key = torch.unique(torch.cat(keys))      # sorted: rows ascending, neighbours ascending within a row
    return key


def make_graph(cfg: Config, device="cpu"):
    """Directed Chung-Lu graph; returns (indptr int64, indices int32, is_local uint8)."""
    n = cfg.n_nodes
    dev = torch.device(device)
    ids = torch.arange(n, dtype=torch.int64, device=dev)
    # rank -> node ID: a fixed pseudo-random relabelling, so degree is not monotone in ID
    perm = torch.sort(counter_bits(cfg.gen_seed, 1, ids), stable=True).indices
    # partition: hash to n_parts, part 0 is the local one
    part = _lsr(counter_bits(cfg.gen_seed, 2, ids), 33) % cfg.n_parts
    is_local = (part == 0).to(torch.uint8)
    del part

    w = powerlaw_weights(n, cfg.gamma, cfg.n_edges)
    cdf_col = torch.from_numpy(np.cumsum(w) / w.sum()).to(dev)
    if cfg.local_rows_only:
        w_row = w * is_local[perm].cpu().numpy().astype(np.float64)
        cdf_row = torch.from_numpy(np.cumsum(w_row) / w_row.sum()).to(dev)
    else:
        cdf_row = cdf_col

    n_draw = int(cfg.n_edges * 1.02)
    key = None
    for _ in range(4):      # hubs saturate: redraw with more edges until the distinct count is near the target
        key = _draw_edges(cfg, n_draw, cdf_row, cdf_col, perm, dev)
        got = key.numel()
        if abs(got - cfg.n_edges) <= 0.02 * cfg.n_edges or n_draw > 40 * cfg.n_edges:
            break
        n_draw = int(n_draw * min(4.0, (cfg.n_edges / max(got, 1)) ** 1.15)) + 1
        del key
    rows = key // n
    indices = (key - rows * n).to(torch.int32)
    del key
    counts = torch.bincount(rows, minlength=n)
    indptr = torch.zeros(n + 1, dtype=torch.int64, device=dev)
    indptr[1:] = torch.cumsum(counts, 0)
    return indptr, indices, is_local


def make_workload(name_or_cfg, device="cpu", feature_device=None, pin_remote=False, remote_device=None) -> Workload:
    """Build every input of one configuration.

    device: where the graph arrays are produced and left.  feature_device:
    where the local table is left (default: same).  remote_device: where the
    remote table is produced and left; by default the host (pinned if
    pin_remote) when feature_device is a GPU, standing in for the other
    partitions' memory.  pinned_copy() moves a table made on the GPU there.
    """
    cfg = CONFIGS[name_or_cfg] if isinstance(name_or_cfg, str) else name_or_cfg
    dev = torch.device(device)
    fdev = torch.device(feature_device) if feature_device is not None else dev
    indptr, indices, is_local = make_graph(cfg, dev)
    n = cfg.n_nodes
    ids = torch.arange(n, dtype=torch.int64, device=dev)

    loc = is_local.to(torch.int64)
    n_local = int(loc.sum().item())
    n_remote = n - n_local
    row_of = torch.where(loc == 1, torch.cumsum(loc, 0) - 1, torch.cumsum(1 - loc, 0) - 1).to(torch.int32)

    # train nodes: T distinct IDs, uniform among the nodes whose adjacency this share holds
    tkey = counter_bits(cfg.gen_seed, 3, ids)
    if cfg.local_rows_only:
        elig = ids[is_local == 1]
        tkey = tkey[is_local == 1]
    else:
        elig = ids
    order = torch.sort(tkey, stable=True).indices[: cfg.n_train]
    train = elig[order].to(torch.int32)
    del tkey, order, elig, ids

    dt = {"float32": torch.float32, "bfloat16": torch.bfloat16}[cfg.feat_dtype]
    esz = 4 if dt == torch.float32 else 2
    row_bytes = cfg.feat_dim * esz
    stride_bytes = (row_bytes + 15) // 16 * 16
    se = stride_bytes // esz

    def table(rows, seed, where, pin):
        g = torch.Generator(device=where)
        g.manual_seed(cfg.gen_seed * 7919 + seed)
        if where.type == "cpu":
            t = torch.empty((rows, se), dtype=dt, pin_memory=pin)
            step = max(1, (1 << 28) // max(se, 1))
            for lo in range(0, rows, step):
                hi = min(rows, lo + step)
                t[lo:hi] = torch.randn((hi - lo, se), generator=g, dtype=torch.float32).to(dt)
            return t
        t = torch.empty((rows, se), dtype=dt, device=where)
        step = max(1, (1 << 30) // max(se, 1))
        for lo in range(0, rows, step):
            hi = min(rows, lo + step)
            t[lo:hi] = torch.randn((hi - lo, se), generator=g, device=where, dtype=torch.float32).to(dt)
        return t

    local_rows = table(n_local, 1, fdev, False)
    if remote_device is not None:
        remote_rows = table(n_remote, 2, torch.device(remote_device), False)
    elif fdev.type == "cpu":
        remote_rows = table(n_remote, 2, fdev, False)
    else:
        remote_rows = table(n_remote, 2, torch.device("cpu"), pin_remote)

    K = cfg.cache_k if cfg.cache_k is not None else int(cfg.cache_frac * n_remote)
    return Workload(cfg, indptr, indices, train, is_local, row_of, local_rows, remote_rows,
                    row_bytes, stride_bytes, K, dict(n_local=n_local, n_remote=n_remote))


_hip = None


def pinned_empty(shape, dtype) -> torch.Tensor:
    """An uninitialised tensor in pinned host memory of exactly the size asked for, straight from hipHostMalloc.
    (torch's pinned allocator rounds a request up to the next power of two, which for a table of tens of GB goes
    past what a box lets a process pin.)  The memory is freed when the last tensor or array over it is gone."""
    import ctypes
    import weakref
    global _hip
    if _hip is None:
        torch.cuda.init()
        _hip = ctypes.CDLL("libamdhip64.so")
        _hip.hipHostMalloc.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_size_t, ctypes.c_uint]
        _hip.hipHostFree.argtypes = [ctypes.c_void_p]
    n = 1
    for d in shape:
        n *= int(d)
    nbytes = n * torch.empty(0, dtype=dtype).element_size()
    if nbytes == 0:
        return torch.empty(shape, dtype=dtype, pin_memory=True)
    p = ctypes.c_void_p()
    rc = _hip.hipHostMalloc(ctypes.byref(p), nbytes, 0)
    if rc != 0 or not p.value:
        raise MemoryError(f"hipHostMalloc of {nbytes} bytes failed with status {rc}")
    buf = (ctypes.c_uint8 * nbytes).from_address(p.value)
    weakref.finalize(buf, _hip.hipHostFree, p)
    return torch.frombuffer(buf, dtype=dtype).view(*shape)


def pinned_copy(t: torch.Tensor, chunk_rows: int = 1 << 22) -> torch.Tensor:
    """A pinned host copy of a (device) table, made in chunks."""
    out = pinned_empty(tuple(t.shape), t.dtype)
    for lo in range(0, t.shape[0], chunk_rows):
        out[lo:lo + chunk_rows].copy_(t[lo:lo + chunk_rows])
    return out


def integer_graph(n: int, deg_lo: int, deg_hi: int, seed: int):
    """A small graph made with integer arithmetic only (no floating point), so
    that it is identical on every machine: stored expected values refer to it.
    Row v gets deg_lo + hash % (deg_hi - deg_lo + 1) distinct pseudo-random
    neighbours.  Returns numpy (indptr int64, indices int32)."""
    rows = []
    indptr = np.zeros(n + 1, np.int64)
    for v in range(n):
        hv = int(counter_bits(seed, 21, torch.tensor([v]))[0].item()) & _M64
        d = deg_lo + hv % (deg_hi - deg_lo + 1)
        cand = _lsr(counter_bits(seed, 22, torch.arange(v * 4096, v * 4096 + 3 * d + 8)), 20) % n
        cand = np.unique(cand.numpy())
        cand = cand[cand != v]
        # drop a pseudo-random subset down to d (or keep all if fewer)
        if cand.size > d:
            sel = _lsr(counter_bits(seed, 23, torch.from_numpy(cand) + v * n), 7).numpy()
            cand = np.sort(cand[np.argsort(sel, kind="stable")[:d]])
        rows.append(cand.astype(np.int32))
        indptr[v + 1] = indptr[v] + cand.size
    return indptr, (np.concatenate(rows) if rows else np.zeros(0, np.int32))
