"""Where a tile's time goes inside the persistent grouped-GEMM kernels: runs bench.py's step on the profiling build of
the library (libflexmoe_phases.so: build.build_phases_library(), the kernels compiled with -DFLEXMOE_TILE_PHASES) and
prints, per kind of product, the mean time per output tile from the tile's start to its first barrier, in the K loop
and in the epilogue, and how the workgroups' totals spread over the eight XCDs.

    python -m paper_2304_03946_amd.tile_phases gpt_xl [gpt_m ...]          (on a GPU machine, from the repository root)
"""
from __future__ import annotations

import contextlib
import ctypes
import io
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
from paper_2304_03946_amd import binding  # noqa: E402

KINDS = ["forward GEMM1", "forward GEMM2", "backward dH", "backward dXp", "weight gradient (last launch: dW1)"]


def main(workloads):
    binding.LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libflexmoe_phases.so")
    if not os.path.exists(binding.LIB_PATH):
        sys.exit("tile_phases: build the profiling library first (paper_2304_03946_amd.build.build_phases_library())")
    import bench
    lib = ctypes.CDLL(binding.LIB_PATH)
    for w in workloads:
        sys.argv = ["bench.py", "--workload", w, "--no-cpu-baseline", "--no-others", "--no-variants", "--no-stages",
                    "--steps", "5", "--warmup", "2"]
        buf = io.StringIO()
        with contextlib.redirect_stdout(buf):
            bench.main()
        line = json.loads(buf.getvalue().strip().splitlines()[-1])
        out = np.zeros((5, 256, 4), dtype=np.uint64)
        rc = lib.flexmoe_debug_tile_phases(out.ctypes.data_as(ctypes.c_void_p))
        if rc != 0:
            sys.exit(f"tile_phases: hipMemcpyFromSymbol failed ({rc})")
        print(f"{w}: {line['ms_per_step']} ms per step with the timers in, grouped-GEMM calls {line['roofline']['launch_ms_by_call']} ms")
        print("  (last step's launches; 100 MHz clock, us; a workgroup = one compute unit)")
        forward_only = line["config"].get("passes") == "forward"
        for k, name in enumerate(KINDS):
            if forward_only and k >= 2:      # the device array still holds the previous workload's backward launches
                continue
            a = out[k].astype(np.float64) / 100.0
            n = out[k][:, 3].astype(np.float64)
            m = n > 0
            if not m.any():
                continue
            top, kl, ep = (a[m, 0] / n[m]).mean(), (a[m, 1] / n[m]).mean(), (a[m, 2] / n[m]).mean()
            tot = a[:, 0] + a[:, 1] + a[:, 2]
            xcd = [round(float(tot[x::8][n[x::8] > 0].mean()), 1) if (n[x::8] > 0).any() else 0.0 for x in range(8)]
            print(f"  {name:36s} tiles/workgroup {n[m].mean():5.1f}   per tile: to first barrier {top:5.2f}  K loop {kl:7.2f}  "
                  f"epilogue {ep:5.2f}")
            print(f"  {'':36s} workgroup totals by XCD {xcd}   max/mean {tot[m].max() / tot[m].mean():.3f}")


if __name__ == "__main__":
    main(sys.argv[1:] or ["gpt_xl"])
