"""Offline profiling for kernel selection (paper Section 3.2: the tile cost is profiled once per
operator and GPU type, independent of model, shape and sparsity pattern).

Measures, on the GPU this runs on, the running time per covered micro-tile of every (dense tile,
PIT-axis) pair the library offers for C[M, N] = A[M, K] . B[K, N] with a sparse A, and prints the
table as JSON -- the ``tile_cost`` values of pit_select_kernel's candidates.

    python -m paper_2301_10936_amd.tile_cost [--n 2048] [--out tile_cost.json]

Candidates (micro-tile shape on A as stored [M, K]):
    gather_k     128 x 1   k is the PIT-axis (A supplied K-major), pit_sread_gemm(GATHER_K, mt=128)
    gather_k_64  64 x 1    the same with the 64-row tile, mt=64;   gather_k_32  32 x 1, mt=32
    dense_k      128 x 1   the dense kernel (PIT_GEMM_DENSE_K, identity addressing, no index): cost per
                           micro-tile of the whole grid
    gather_m_S   1 x S     m is the PIT-axis, k-slabs of S in {32, 64, 128}, pit_sread_gemm(GATHER_M, mt=S)
    gather_m_row 1 x K     m is the PIT-axis, whole rows, pit_sread_gemm(GATHER_M, mt=K)
"sparse_ns_per_tile" is measured at the stated cover (keep), "dense_ns_per_tile" at full cover through the
index.  For the gather_k family and the dense kernel, a whole step (pit_build_index at the candidate's
micro-tile + the product; the dense kernel builds no index) is also fitted as
    step time = "step_fixed_ns" + covered micro-tiles x "step_ns_per_tile"
from two covers (0.1 and 0.6) of a 4096^3 product (the dense kernel: from two extents of k): these two numbers
are the fixed_cost and tile_cost of pit_select_kernel's candidates.  (The step time is not quite affine in the
cover: steeper below 0.1 and, for the low tiles, above 0.5.  A fit through covers 0.02 and 0.4 instead ranked the
three tile heights no better at 95-99 % sparsity, where they are within 5 us of each other, and worse between.)
"""
import argparse
import json
import sys
import time

import numpy as np
import torch

from . import pit, workloads as wl


def _dev(bits):
    return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).cuda()


def _time(fn, reps=20):
    # the clocks of sustained load are reached only after tens of milliseconds of uninterrupted work (the first
    # few hundred launches after an idle spell run 10-20 % slower): what is timed is preceded by 50 ms of itself
    fn()                          # (one-time set-up behind a first call is not sustained work)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < 0.05:
        for _ in range(16):
            fn()
        torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps * 1e-3


def measure(M=2048, K=4096, N=2048, keep=0.5, seed=0):
    g = np.random.default_rng(seed)
    B = _dev(wl.to_bf16_bits(g.standard_normal((K, N)).astype(np.float32)))
    table = {}

    def gather_k(frac, mt=128):
        live = g.random((K, M // mt)) < frac
        At = np.repeat(live, mt, axis=1).astype(np.float32) * g.standard_normal((K, M)).astype(np.float32)
        tA = _dev(wl.to_bf16_bits(At))
        ix = pit.pit_build_index(tA, 1, mt, 0)
        C = torch.empty((M, N), dtype=torch.float32, device="cuda")
        t = _time(lambda: pit.pit_sread_gemm(pit.PIT_GEMM_GATHER_K, tA, B, ix, mt, M, N, K, out=C))
        return t / max(int(live.sum()), 1)

    def gather_m(slab, frac):
        live = g.random((M, K // slab)) < frac
        A = np.repeat(live, slab, axis=1).astype(np.float32) * g.standard_normal((M, K)).astype(np.float32)
        tA = _dev(wl.to_bf16_bits(A))
        ix = pit.pit_build_index(tA, 1, slab, 0)
        C = torch.empty((M, N), dtype=torch.float32, device="cuda")
        t = _time(lambda: pit.pit_sread_gemm(pit.PIT_GEMM_GATHER_M, tA, B, ix, slab, M, N, K, out=C))
        return t / max(int(live.sum()), 1)

    for name, fn in [("gather_k", gather_k), ("gather_k_64", lambda fr: gather_k(fr, 64)), ("gather_k_32", lambda fr: gather_k(fr, 32))] + \
                    [(f"gather_m_{s}", (lambda fr, s=s: gather_m(s, fr))) for s in (32, 64, 128, K)]:
        key = name if not name.endswith("_" + str(K)) else "gather_m_row"
        table[key] = {"sparse_ns_per_tile": fn(keep) * 1e9, "dense_ns_per_tile": fn(1.0) * 1e9}
    for k, v in step_costs().items():
        table.setdefault(k, {}).update(v)
    shapes = {"gather_k": [128, 1], "gather_k_64": [64, 1], "gather_k_32": [32, 1], "dense_k": [128, 1],
              "gather_m_32": [1, 32], "gather_m_64": [1, 64], "gather_m_128": [1, 128], "gather_m_row": [1, K]}
    return {"device": torch.cuda.get_device_name(0), "M": M, "K": K, "N": N, "keep": keep,
            "candidates": {k: {"micro_tile": shapes[k], **v} for k, v in table.items()}}


def step_costs(n=4096, seed=1):
    """Affine fit of a whole step (index build + product) over the number of covered micro-tiles, per tile height
    of the GATHER_K kernel, and the dense kernel's time per micro-tile of the grid, on an n^3 product."""
    g = np.random.default_rng(seed)
    B = _dev(wl.to_bf16_bits(g.standard_normal((n, n)).astype(np.float32)))
    vals = g.standard_normal((n, n)).astype(np.float32)
    C = torch.empty((n, n), dtype=torch.float32, device="cuda")
    out = {}
    for name, mt in (("gather_k", 128), ("gather_k_64", 64), ("gather_k_32", 32)):
        pts = []
        for frac in (0.1, 0.6):
            live = g.random((n, n // mt)) < frac
            tA = _dev(wl.to_bf16_bits(np.repeat(live, mt, axis=1) * vals))
            ix = pit.PitIndex.empty(n // mt, (n // mt) * n)
            ws = torch.empty(pit.pit_build_index_workspace(n, n, 1, mt, 0), dtype=torch.uint8, device="cuda")

            def step():
                pit.pit_build_index(tA, 1, mt, 0, out=ix, ws=ws)
                pit.pit_sread_gemm(pit.PIT_GEMM_GATHER_K, tA, B, ix, mt, n, n, n, out=C)

            pts.append((int(live.sum()), _time(step) * 1e9))
        slope = (pts[1][1] - pts[0][1]) / (pts[1][0] - pts[0][0])
        out[name] = {"step_ns_per_tile": slope, "step_fixed_ns": max(pts[0][1] - slope * pts[0][0], 0.0)}
    # the dense kernel: the same fit over the micro-tiles of the whole grid, from two extents of k
    tA = _dev(wl.to_bf16_bits(vals))
    pts = []
    for k in (n // 2, n):
        t = _time(lambda: pit.pit_sread_gemm(pit.PIT_GEMM_DENSE_K, tA[:k], B[:k], None, 128, n, n, k, out=C)) * 1e9
        pts.append((k * (n // 128), t))
    slope = (pts[1][1] - pts[0][1]) / (pts[1][0] - pts[0][0])
    out["dense_k"] = {"step_ns_per_tile": slope, "step_fixed_ns": max(pts[0][1] - slope * pts[0][0], 0.0),
                      "dense_ns_per_tile": pts[1][1] / pts[1][0]}
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--n", type=int, default=2048)
    ap.add_argument("--out", default=None)
    a = ap.parse_args()
    if not torch.cuda.is_available():
        print("tile_cost: no GPU visible", file=sys.stderr)
        sys.exit(1)
    t0 = time.time()
    res = measure(N=a.n)
    res["seconds"] = round(time.time() - t0, 1)
    txt = json.dumps(res, indent=1)
    print(txt)
    if a.out:
        open(a.out, "w").write(txt + "\n")


if __name__ == "__main__":
    main()
