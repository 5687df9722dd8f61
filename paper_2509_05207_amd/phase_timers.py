"""Where the sampling kernel's waves spend their time: the library built with -DRG_PHASE_TIMERS (cycle counter read
around each phase of the kernel, summed over all waves) run on one epoch's schedule build.

    python -m paper_2509_05207_amd.phase_timers --workload medium

The profiling build goes to librapidgnn_hip_phases.so beside the ordinary library, which it does not touch; the
timers themselves cost a few per cent, so the shares matter, not the total."""
import argparse
import ctypes as C
import os
import sys

import torch

from . import build as hip_build
from . import synth

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "librapidgnn_hip_phases.so")
PHASES = ("wave total", "tiles of rows above 16,384 IDs", "group set-up", "rows of up to 64 IDs", "rows of 65-256 IDs", "long rows, all of it",
          "long row: entry up to the loop", "long row: streaming loop", "long row: final cut to f", "long row: output and marks",
          "#long rows", "#blocks of 256 IDs", "#candidates at the final cut", "#rows of up to 64 IDs", "#rows of 65-256 IDs",
          "per-node loop overhead", "rows copied whole", "#rows copied whole", "#nodes", "work counter")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="medium", choices=sorted(synth.CONFIGS))
    ap.add_argument("--rebuild", action="store_true")
    args = ap.parse_args()
    if args.rebuild or not os.path.exists(LIB) or hip_build.stale_against(LIB):
        hip_build.build(out=LIB, defines=("RG_PHASE_TIMERS",))
    if not torch.cuda.is_available():
        sys.exit("phase_timers: built " + LIB + "; no GPU visible to run it on")
    from . import binding as rg
    rg.use_library(LIB)
    lib = rg.lib()
    lib.rg_phase_timers_read.restype = C.c_int
    cfg = synth.CONFIGS[args.workload]
    W = synth.make_workload(cfg, device="cuda", feature_device="cuda")
    vals = (C.c_ulonglong * len(PHASES))()
    for _ in range(2):                      # the first build warms the allocator; the second is read
        s = rg.rg_build_schedule(W.indptr, W.indices, W.train, cfg.batch_size, cfg.fanout, cfg.s0, cfg.worker, cfg.epoch)
        torch.cuda.synchronize()
        rc = lib.rg_phase_timers_read(vals, len(PHASES), 1)
        assert rc == 0, rc
        del s
    v = list(vals)
    total = v[0] or 1
    print(f"# {cfg.name}: cycles summed over all waves of the sampling launches of one schedule build")
    print("| phase | cycles or count | share of wave time |")
    print("|---|---|---|")
    for name, x in zip(PHASES, v):
        share = "" if name.startswith("#") else f"{100.0 * x / total:.1f} %"
        print(f"| {name} | {x} | {share} |")
    if v[10]:
        print(f"per long row: {v[5] / v[10]:.0f} cycles, {v[11] / v[10]:.1f} blocks, {v[7] / max(1, v[11]):.0f} loop cycles per block, "
              f"{v[12] / v[10]:.1f} candidates at the final cut")
    if v[13]:
        print(f"per row of up to 64 IDs: {v[3] / v[13]:.0f} cycles")
    if v[14]:
        print(f"per row of 65-256 IDs: {v[4] / v[14]:.0f} cycles")
    if v[18]:
        print(f"per node: {v[15] / v[18]:.0f} cycles of loop overhead")


if __name__ == "__main__":
    main()
