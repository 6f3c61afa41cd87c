#!/usr/bin/env python3
"""Synthetic versions of the paper's micro-benchmarks (Section 5.4): a 4096^3 product under block
sparsity of several granularities and ratios, the index build alone on 4096 x 4096 masks, and the
overhead at 0 % sparsity.  Prints one JSON object; not part of the bench.py contract.

    python bench_micro.py [--reps 20]
"""
import argparse
import json
import sys

import numpy as np
import torch


def _time(fn, reps):
    for _ in range(3):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps * 1e-3


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--reps", type=int, default=20)
    a = ap.parse_args()
    if not torch.cuda.is_available():
        print("bench_micro.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    from paper_2301_10936_amd import pit, workloads as wl
    n = 4096
    g = np.random.default_rng(0)

    def bf16(x):
        return torch.from_numpy(wl.to_bf16_bits(x).view(np.int16)).view(torch.bfloat16).cuda()

    B = bf16(g.standard_normal((n, n)).astype(np.float32))
    dense_A = bf16(g.standard_normal((n, n)).astype(np.float32))
    t_dense = _time(lambda: torch.matmul(dense_A, B), a.reps)
    out = {"shape": [n, n, n], "dense_hipblaslt_ms": round(t_dense * 1e3, 4), "gemm": [], "index_build": []}

    # A stored K-major (At[k][m]); sparsity in blocks of gm tokens x gk channels, i.e. At blocks of gk x gm
    vals = g.standard_normal((n, n)).astype(np.float32)
    # (64, 32) is also the case of weights pruned in blocks of 32 k x 64 outputs, with the operand roles swapped
    for gm, gk in ((32, 1), (32, 64), (128, 1), (64, 32)):
        for s in (0.0, 0.5, 0.9, 0.95, 0.99):
            keep = wl.iid_block_mask(n, n, gk, gm, s, seed=int(s * 100) + gm + gk)
            At = bf16(vals * keep)
            ix = pit.PitIndex.empty(n // 128, (n // 128) * n)
            ws = torch.empty(pit.pit_build_index_workspace(n, n, 1, 128, 0), dtype=torch.uint8, device="cuda")
            C = torch.empty((n, n), dtype=torch.float32, device="cuda")

            def step():
                pit.pit_build_index(At, 1, 128, 0, out=ix, ws=ws)
                pit.pit_sread_gemm(pit.PIT_GEMM_GATHER_K, At, B, ix, 128, n, n, n, out=C)

            t = _time(step, a.reps)
            t_idx = _time(lambda: pit.pit_build_index(At, 1, 128, 0, out=ix, ws=ws), a.reps)
            torch.cuda.synchronize()
            want = C.clone()
            # the same step replayed from a HIP graph: the GPU's time without the host's launch calls
            # (every replay is checked against the eager result)
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                step()
            torch.cuda.current_stream().wait_stream(side)
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                step()
            ok = True
            for _ in range(3):
                C.fill_(-1.0)
                graph.replay()
                torch.cuda.synchronize()
                ok = ok and bool(torch.equal(C, want))
            t_graph = _time(graph.replay, a.reps)
            cover = int(ix.seg_ptr[-1].item()) / float((n // 128) * n)
            out["gemm"].append({"granularity_tokens_x_channels": [gm, gk], "sparsity": s, "cover_128x1": round(cover, 4),
                                "step_ms": round(t * 1e3, 4), "index_ms": round(t_idx * 1e3, 4),
                                "step_graph_ms": round(t_graph * 1e3, 4), "graph_matches_eager": ok,
                                "speedup_vs_dense": round(t_dense / min(t, t_graph), 3)})

    # A row-major [m][k], zeros in blocks of 1 token x 64 channels: PIT-axis m inside k-slabs of 64
    # (GATHER_M, the slabs' partial products are added in strips of C held in LDS)
    out["gemm_row_major_1x64"] = []
    for s in (0.5, 0.9, 0.95, 0.99):
        keep = wl.iid_block_mask(n, n, 1, 64, s, seed=int(s * 100) + 7)
        A = bf16(vals * keep)
        ix = pit.PitIndex.empty(n // 64, (n // 64) * n)
        ws = torch.empty(pit.pit_build_index_workspace(n, n, 1, 64, 0), dtype=torch.uint8, device="cuda")
        C = torch.empty((n, n), dtype=torch.float32, device="cuda")

        def step_m():
            pit.pit_build_index(A, 1, 64, 0, out=ix, ws=ws)
            pit.pit_sread_gemm(pit.PIT_GEMM_GATHER_M, A, B, ix, 64, n, n, n, out=C)

        t = _time(step_m, a.reps)
        torch.cuda.synchronize()
        cover = int(ix.seg_ptr[-1].item()) / float((n // 64) * n)
        out["gemm_row_major_1x64"].append({"sparsity": s, "cover_1x64": round(cover, 4), "step_ms": round(t * 1e3, 4),
                                           "speedup_vs_dense": round(t_dense / t, 3)})

    # index build alone on byte masks (Section 5.4, "Sparsity detection"), 99 % sparsity
    for gr in (1, 16, 32):
        m = torch.from_numpy(wl.iid_block_mask(n, n, gr, gr, 0.99, seed=gr)).cuda()
        ix = pit.PitIndex.empty(n // gr, (n // gr) * (n // gr))
        ws = torch.empty(pit.pit_build_index_workspace(n, n, gr, gr, 1), dtype=torch.uint8, device="cuda")
        t = _time(lambda: pit.pit_build_index(m, gr, gr, 1, out=ix, ws=ws), a.reps)
        out["index_build"].append({"mask": [n, n], "micro_tile": [gr, gr], "ms": round(t * 1e3, 4),
                                   "GB_per_s": round(n * n / t / 1e9, 1)})
    print(json.dumps(out))


if __name__ == "__main__":
    main()
