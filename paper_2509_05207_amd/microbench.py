"""Micro-benchmarks of the access patterns alone (csrc_micro/micro.hip), the yardsticks quoted beside the kernels:

  * a plain streaming copy, the runtime's own device-to-device copy, and stores alone / loads alone;
  * the sampler's marking traffic alone: atomic ORs into bitmaps against byte stores into byte maps;
  * the sampler's row reads alone on a workload's real frontiers: every row streamed once, keys computed, minimum kept.

    python -m paper_2509_05207_amd.microbench --workload medium

Prints markdown.  Builds libmicro.so beside the package's library on first use."""
import argparse
import ctypes as C
import os
import subprocess
import sys

import torch

from . import synth

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(HERE, "csrc_micro", "micro.hip")
LIB = os.path.join(HERE, "libmicro.so")


def build():
    deps = [SRC, os.path.join(HERE, "csrc", "rg_device.h")]
    if os.path.exists(LIB) and all(os.path.getmtime(LIB) >= os.path.getmtime(p) for p in deps):
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
                           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
                           "-I", os.path.join(ROOT, "include"), "-o", LIB, SRC])
    return LIB


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="medium", choices=sorted(synth.CONFIGS))
    args = ap.parse_args()
    build()
    if not torch.cuda.is_available():
        sys.exit("microbench: built " + LIB + "; no GPU visible to run it on")
    mb = C.CDLL(LIB)
    vp, u64, u32, i64 = C.c_void_p, C.c_uint64, C.c_uint32, C.c_int64
    mb.mb_copy.restype = mb.mb_marks.restype = mb.mb_stream.restype = mb.mb_fill.restype = mb.mb_read.restype = C.c_float
    mb.mb_fill.argtypes = [vp, u64, C.c_int, C.c_int, C.c_int]
    mb.mb_read.argtypes = [vp, u64, vp, C.c_int, C.c_int]
    mb.mb_copy.argtypes = [vp, vp, u64, C.c_int, C.c_int, C.c_int]
    mb.mb_marks.argtypes = [vp, vp, vp, u64, u32, u32, u64, C.c_int, C.c_int]
    mb.mb_stream.argtypes = [vp, vp, vp, i64, vp, C.c_int, C.c_int, C.c_int]

    print("## Plain copies (read + write counted)\n")
    print("| copy | bytes | us | GB/s |\n|---|---|---|---|")
    for nbytes in (193_300_000 // 16 * 16, 1 << 30):
        a = torch.ones(nbytes, dtype=torch.uint8, device="cuda")
        b = torch.empty_like(a)
        best = None
        for unroll in (4, 8):
            for grid in (4096, 8192, 16384):
                ms = mb.mb_copy(a.data_ptr(), b.data_ptr(), nbytes, unroll, grid, 10)
                assert ms > 0, ms
                if best is None or ms < best[0]:
                    best = (ms, unroll, grid)
        print(f"| 16-byte loads and stores, {best[1]} per thread in flight, {best[2]} workgroups (best of six shapes) | {nbytes} | {best[0] * 1e3:.1f} | {2 * nbytes / best[0] / 1e6:.0f} |")
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        b.copy_(a)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(10):
            b.copy_(a)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 10
        print(f"| the runtime's device-to-device copy (torch `copy_`) | {nbytes} | {ms * 1e3:.1f} | {2 * nbytes / ms / 1e6:.0f} |")
        one = torch.zeros(1, dtype=torch.int32, device="cuda")
        for name, call in (("stores alone, plain", lambda g: mb.mb_fill(b.data_ptr(), nbytes, 0, g, 10)),
                           ("stores alone, nontemporal", lambda g: mb.mb_fill(b.data_ptr(), nbytes, 1, g, 10)),
                           ("loads alone", lambda g: mb.mb_read(a.data_ptr(), nbytes, one.data_ptr(), g, 10))):
            best = None
            for grid in (4096, 8192, 16384):
                ms = call(grid)
                assert ms > 0, ms
                best = ms if best is None else min(best, ms)
            print(f"| {name} (16 bytes per lane, best of three grids; one direction, bytes counted once) | {nbytes} | {best * 1e3:.1f} | {nbytes / best / 1e6:.0f} |")
        del a, b

    print("\n## Marks alone (IDs with a power-law bias, consecutive marks share a batch)\n")
    print("| nodes | batches | marks | form | ms | G marks/s |\n|---|---|---|---|---|---|")
    for n_nodes, n_batches, n_marks in ((233_000, 147, 29_000_000), (2_450_000, 49, 167_000_000), (2_450_000, 196, 140_000_000)):
        wpb = ((n_nodes + 31) // 32 + 63) // 64 * 64
        words = torch.zeros(wpb * n_batches, dtype=torch.int32, device="cuda")
        flags = torch.zeros(wpb // 8 * n_batches, dtype=torch.uint8, device="cuda")
        bts = torch.zeros(wpb * 32 * n_batches, dtype=torch.uint8, device="cuda")
        for mode, name in ((0, "atomic OR into a bit per ID + flag byte"), (1, "store into a byte per ID + flag byte")):
            ms = mb.mb_marks(words.data_ptr(), flags.data_ptr(), bts.data_ptr(), wpb, n_nodes, n_batches, n_marks, mode, 3)
            assert ms > 0, ms
            print(f"| {n_nodes} | {n_batches} | {n_marks} | {name} | {ms:.3f} | {n_marks / ms / 1e6:.1f} |")
        del words, flags, bts

    from . import binding as rg
    rg.lib()
    cfg = synth.CONFIGS[args.workload]
    W = synth.make_workload(cfg, device="cuda", feature_device="cuda")
    s = rg.rg_build_schedule(W.indptr, W.indices, W.train, cfg.batch_size, cfg.fanout, cfg.s0, cfg.worker, cfg.epoch)
    print(f"\n## Row reads alone: {cfg.name}, every row of a hop's frontier streamed once (rows above 16,384 IDs in pieces of that size, as the sampler's tiles are)\n")
    print("| hop | rows and pieces | IDs read | kernel | ms | GB/s |\n|---|---|---|---|---|---|")
    for hop in range(len(cfg.fanout)):
        ids = rg.rg_schedule_frontier(s, hop)[0].long()
        rb0 = W.indptr[ids]
        deg0 = W.indptr[ids + 1] - rb0
        pieces = torch.clamp((deg0 + 16383) // 16384, min=1)                  # a row above 16,384 IDs is read in pieces, like the sampler's tiles
        owner = torch.repeat_interleave(torch.arange(ids.numel(), device="cuda"), pieces)
        k = torch.arange(owner.numel(), device="cuda") - torch.repeat_interleave(torch.cumsum(pieces, 0) - pieces, pieces)
        rb = (rb0[owner] + k * 16384).contiguous()
        deg = torch.clamp(deg0[owner] - k * 16384, max=16384).to(torch.int32).contiguous()
        n = rb.numel()
        out = torch.empty(n, dtype=torch.int32, device="cuda")
        total = int(deg.sum().item())
        for hash_, name in ((0, "loads and an XOR"), (1, "loads, key of every ID, minimum")):
            best = None
            for grid in (8192, 16384, 32768):
                ms = mb.mb_stream(W.indices.data_ptr(), rb.data_ptr(), deg.data_ptr(), n, out.data_ptr(), hash_, grid, 3)
                assert ms > 0, ms
                best = ms if best is None else min(best, ms)
            print(f"| {hop} | {n} | {total} | {name} | {best:.3f} | {total * 4 / best / 1e6:.0f} |")


if __name__ == "__main__":
    main()
