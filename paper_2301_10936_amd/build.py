"""Build the HIP library in-tree:  python -m paper_2301_10936_amd.build

hipcc cross-compiles for gfx950 without a GPU.  The result, libpit_hip.so, sits next to this file
and is what the ctypes binding loads.
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpit_hip.so")
SOURCES = ["pit_api.hip", "pit_index.hip", "pit_gemm.hip", "pit_gemm_m.hip", "pit_moe.hip", "pit_attn.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-Wno-inline-asm", "-Wno-pass-failed",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


PROBE_LIB = os.path.join(HERE, "libpit_probe.so")     # measurement probes (bench_micro.py --probe), not the product


def _compile(srcs, lib, verbose):
    cmd = ["hipcc", *FLAGS, "-o", lib, *srcs]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    noise = "is not a recognized feature for this target"
    out = "\n".join(l for l in proc.stdout.splitlines() if noise not in l)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)


def build(verbose: bool = False) -> str:
    srcs = [os.path.join(CSRC, s) for s in SOURCES if os.path.exists(os.path.join(CSRC, s))]
    _compile(srcs, LIB, verbose)
    _compile([os.path.join(CSRC, "pit_probe.hip")], PROBE_LIB, verbose)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
    sys.exit(0)
