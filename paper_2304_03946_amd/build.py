"""Build libflexmoe.so (HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libflexmoe.so")
SOURCES = ["api.hip", "gate.hip", "route.hip", "route_static.hip", "permute_combine.hip", "ffn_f32.hip", "ffn_bf16.hip", "gate_bwd.hip",
           "scheduler.cpp"]     # .cpp = host-only code

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _compile(src: str) -> str:
    obj = os.path.join(CSRC, os.path.splitext(src)[0] + ".o")
    cmd = [HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def generate_tables() -> str:
    """Constant data compiled into the library: the GELU residual tables (csrc/gen_act_lut.py)."""
    out = os.path.join(CSRC, "act_lut_data.inc")
    r = subprocess.run([sys.executable, os.path.join(CSRC, "gen_act_lut.py"), out], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("gen_act_lut.py failed:\n" + r.stderr)
    return out


def build_probe(verbose: bool = True) -> str:
    """The K-loop microbenchmark behind the ceilings quoted for the grouped GEMMs (csrc/probe/kloop_probe.hip):
    a stand-alone executable next to the library; run it on the GPU machine as paper_2304_03946_amd/kloop_probe."""
    out = os.path.join(PKG, "kloop_probe")
    cmd = [HIPCC, "-O3", "-std=c++17", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           os.path.join(CSRC, "probe", "kloop_probe.hip"), "-o", out]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for kloop_probe.hip:\n" + r.stderr)
    if verbose:
        print(f"built {out}")
    return out


def build_phases_library(verbose: bool = True) -> str:
    """A second library with per-tile phase timers in the persistent GEMM kernels (-DFLEXMOE_TILE_PHASES), for
    paper_2304_03946_amd/tile_phases.py; not loaded by anything else.  Needs the objects of build_library()."""
    out = os.path.join(PKG, "libflexmoe_phases.so")
    obj = os.path.join(CSRC, "ffn_bf16_phases.o")
    r = subprocess.run([HIPCC, *FLAGS, "-DFLEXMOE_TILE_PHASES", "-c", os.path.join(CSRC, "ffn_bf16.hip"), "-o", obj],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for ffn_bf16.hip (phases):\n" + r.stderr)
    objs = [obj if s == "ffn_bf16.hip" else os.path.join(CSRC, os.path.splitext(s)[0] + ".o") for s in SOURCES]
    r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", out, *objs], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print(f"built {out}")
    return out


def build_library(verbose: bool = True) -> str:
    """Compile every source and link the shared library; always rebuilds."""
    generate_tables()
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print(f"built {LIB}")
    return LIB


if __name__ == "__main__":
    build_library()
    build_probe()
    build_phases_library()
