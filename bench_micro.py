#!/usr/bin/env python3
"""Synthetic versions of the paper's micro-benchmarks on one MI355X (not part of the bench.py contract).

  * Section 5.3 ("Effectiveness of PIT transformation"): a 4096^3 product whose sparse operand has zeros in
    blocks of several granularities at 0 - 99 % sparsity, 0 % being the overhead check against the dense kernel.
    Every kernel the library offers for a K-major operand is timed at every point -- GATHER_K at tile heights
    128, 64 and 32 (index rebuilt in every step) and the dense kernel -- next to hipBLASLt's dense GEMM, and
    Algorithm 1 (Section 3.2) is run on the point with the profiled tile costs: its choice is reported beside
    the measured-fastest kernel.
  * Section 5.5 / Table 3: granularities 2 x 1, 4 x 1, 8 x 1 and 32 x 1 at 95 % and 99 %, covered by the micro-tiles
    the kernels offer (32 x 1, 64 x 1, 128 x 1; the paper's CUDA-core tiles go down to 8 x 1).
  * Section 5.4 ("Sparsity detection"): the index build alone on 4096 x 4096 byte masks.

    python bench_micro.py [--reps 20] [--table]      (--table: a text table instead of JSON)
"""
import argparse
import json
import os
import sys
import time

import numpy as np
import torch

MTS = (128, 64, 32)


def _time(fn, reps):
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


def candidates(pit):
    """The (dense tile, PIT-axis) pairs of the GATHER_K family with the profiled cost of a step per covered
    micro-tile and its constant part (committed profile of this GPU type), and the dense kernel."""
    here = os.path.dirname(os.path.abspath(pit.__file__))
    prof = json.load(open(os.path.join(here, "tile_cost_mi355x.json")))["candidates"]
    names = {128: "gather_k", 64: "gather_k_64", 32: "gather_k_32"}
    c = [{"mt_rows": 1, "mt_cols": mt, "tile_cost": prof[names[mt]]["step_ns_per_tile"],
          "fixed_cost": prof[names[mt]]["step_fixed_ns"]} for mt in MTS]
    c.append({"mt_rows": 1, "mt_cols": 128, "tile_cost": prof["dense_k"]["step_ns_per_tile"],
              "fixed_cost": prof["dense_k"]["step_fixed_ns"], "dense": True})
    return c


def sweep_point(pit, At, B, n, reps, cands, t_dense_lib):
    """All kernels on one sparse operand At [K, M] (K-major); returns the record of the point."""
    C = torch.empty((n, n), dtype=torch.float32, device="cuda")
    rec = {"kernels": {}}
    for mt in MTS:
        ix = pit.PitIndex.empty(n // mt, (n // mt) * n)
        ws = torch.empty(pit.pit_build_index_workspace(n, n, 1, mt, 0), dtype=torch.uint8, device="cuda")

        def step():
            pit.pit_build_index(At, 1, mt, 0, out=ix, ws=ws)
            pit.pit_sread_gemm(pit.PIT_GEMM_GATHER_K, At, B, ix, mt, n, n, n, out=C)

        t = _time(step, reps)
        t_idx = _time(lambda: pit.pit_build_index(At, 1, mt, 0, out=ix, ws=ws), reps)
        cover = int(ix.seg_ptr[-1].item()) / float((n // mt) * n)
        rec["kernels"][f"gather_k_{mt}"] = {"cover": round(cover, 4), "step_us": round(t * 1e6, 1), "index_us": round(t_idx * 1e6, 1)}
    t = _time(lambda: pit.pit_sread_gemm(pit.PIT_GEMM_DENSE_K, At, B, None, 128, n, n, n, out=C), reps)
    rec["kernels"]["dense_k"] = {"cover": 1.0, "step_us": round(t * 1e6, 1), "index_us": 0.0}
    # Algorithm 1 on this point: CoverAlgo on the GPU, costs from the profile
    num = [[int(pit.pit_cover_count(At, 1, c["mt_cols"]).item()) for c in cands]]
    grid = [[n * (n // c["mt_cols"]) for c in cands]]
    chosen, _ = pit.pit_select_kernel(cands, num, grid)
    order = [f"gather_k_{mt}" for mt in MTS] + ["dense_k"]
    fastest = min(order, key=lambda k: rec["kernels"][k]["step_us"])
    rec["selected"] = order[chosen]
    rec["fastest"] = fastest
    rec["selected_over_fastest"] = round(rec["kernels"][order[chosen]]["step_us"] / rec["kernels"][fastest]["step_us"], 3)
    rec["speedup_vs_hipblaslt_selected"] = round(t_dense_lib * 1e6 / rec["kernels"][order[chosen]]["step_us"], 3)
    return rec


def probe():
    """Register-resident issue rate of the two MFMA shapes the kernels use (1 and 4 waves per SIMD), the rate at
    which a read-only kernel streams a mixture-of-experts matmul's weights, an empty kernel's launch, and three
    dependent launches back to back (the floor of a three-kernel step)."""
    import ctypes
    here = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_2301_10936_amd")
    lib = ctypes.CDLL(os.path.join(here, "libpit_probe.so"))
    lib.pit_probe_mfma.restype = ctypes.c_double
    lib.pit_probe_mfma.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
    lib.pit_probe_empty.argtypes = [ctypes.c_void_p]
    out = torch.zeros(4, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    res = {"compute_units": cus, "mfma": [], "launch": {}}
    for shape, name in ((0, "v_mfma_f32_16x16x32_bf16"), (1, "v_mfma_f32_32x32x16_bf16")):
        for waves_per_simd in (1, 4):
            blocks, iters = cus * waves_per_simd, 20000
            flops = [0.0]

            def run():
                flops[0] = lib.pit_probe_mfma(shape, blocks, iters, out.data_ptr(), st)

            t = _time(run, 5)
            per = t / (iters * 8.0) * 1e9
            res["mfma"].append({"instruction": name, "waves_per_simd": waves_per_simd, "TFLOP_per_s": round(flops[0] / t / 1e12, 1),
                                "ns_per_mfma_per_wave": round(per, 2)})
    # Streaming of the 302 MB of one MoE matmul's expert weights (read once per call; two such buffers alternate,
    # as the two matmuls of the call do, so nothing is left in the 256 MB Infinity Cache from the launch before):
    # contiguous ranges from a growing number of workgroups, and the 512-byte pieces of rows that a 256-column tile
    # of matmul 2 (3072 x 256 of an expert's 3072 x 768) and of matmul 1 (768 x 256 of 768 x 3072) reads
    lib.pit_probe_stream.restype = ctypes.c_double
    lib.pit_probe_stream.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_int, ctypes.c_long, ctypes.c_long,
                                     ctypes.c_int, ctypes.c_int, ctypes.c_long, ctypes.c_void_p, ctypes.c_void_p]
    half = 64 * 3072 * 768 * 2
    buf = torch.zeros(2 * half, dtype=torch.uint8, device="cuda")
    cases = []
    for wgs in (256, 512, 1024, 4096):
        per = (half // wgs) // 16384 * 16384
        cases.append((f"contiguous, {per >> 10} KB per workgroup", wgs, wgs, 0, per, per // 512, 512))
    cases.append(("matmul 2 tiles: 3072 pieces of 512 B at pitch 1536 B", 192, 3, 3072 * 1536, 512, 3072, 1536))
    cases.append(("matmul 1 tiles: 768 pieces of 512 B at pitch 6144 B", 768, 12, 768 * 6144, 512, 768, 6144))
    res["stream_302MB"] = []
    for name, wgs, per_group, gstride, wstride, rows, pitch in cases:
        flip, nbytes = [0], [0.0]

        def run():
            flip[0] ^= 1
            nbytes[0] = lib.pit_probe_stream(buf.data_ptr() + flip[0] * half, half, wgs, per_group, gstride, wstride, rows, 512, pitch,
                                             out.data_ptr(), st)

        t = _time(run, 20)
        if nbytes[0] <= 0:
            raise RuntimeError("pit_probe_stream rejected " + name)
        res["stream_302MB"].append({"pattern": name, "workgroups": wgs, "us": round(t * 1e6, 1), "TB_per_s": round(nbytes[0] / t / 1e12, 2)})
    res["launch"]["empty_kernel_us"] = round(_time(lambda: lib.pit_probe_empty(st), 200) * 1e6, 2)
    res["launch"]["three_dependent_empty_kernels_us"] = round(_time(lambda: [lib.pit_probe_empty(st) for _ in range(3)], 100) * 1e6, 2)
    print(json.dumps(res, indent=1))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--reps", type=int, default=20)
    ap.add_argument("--table", action="store_true")
    ap.add_argument("--probe", action="store_true", help="MFMA issue rates and launch floor instead of the sweeps")
    a = ap.parse_args()
    if not torch.cuda.is_available():
        print("bench_micro.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    if a.probe:
        probe()
        return
    from paper_2301_10936_amd import pit, workloads as wl
    n = 4096
    g = np.random.default_rng(0)

    def bf16(x):
        return torch.from_numpy(wl.to_bf16_bits(x).view(np.int16)).view(torch.bfloat16).cuda()

    B = bf16(g.standard_normal((n, n)).astype(np.float32))
    dense_A = bf16(g.standard_normal((n, n)).astype(np.float32))
    t_dense = _time(lambda: torch.matmul(dense_A, B), a.reps)
    cands = candidates(pit)
    out = {"shape": [n, n, n], "dense_hipblaslt_us": round(t_dense * 1e6, 1), "gemm": [], "table3": [], "index_build": []}

    # Section 5.3: A stored K-major (At[k][m]); zeros in blocks of gm tokens x gk channels, i.e. At blocks of gk x gm
    vals = g.standard_normal((n, n)).astype(np.float32)
    for gm, gk in ((32, 1), (64, 1), (128, 1), (32, 64)):
        for s in (0.0, 0.5, 0.9, 0.95, 0.99):
            keep = wl.iid_block_mask(n, n, gk, gm, s, seed=int(s * 100) + gm + gk)
            rec = sweep_point(pit, bf16(vals * keep), B, n, a.reps, cands, t_dense)
            out["gemm"].append({"granularity_tokens_x_channels": [gm, gk], "sparsity": s, **rec})
    # Table 3: fine granularities under the micro-tiles the kernels offer
    for gm in (2, 4, 8, 32):
        for s in (0.95, 0.99):
            keep = wl.iid_block_mask(n, n, 1, gm, s, seed=int(s * 100) + gm)
            rec = sweep_point(pit, bf16(vals * keep), B, n, a.reps, cands, t_dense)
            out["table3"].append({"granularity_tokens_x_channels": [gm, 1], "sparsity": s, **rec})

    # the headline step replayed from a HIP graph (every replay checked against the eager result)
    keep = wl.iid_block_mask(n, n, 1, 32, 0.9, seed=77)
    At = bf16(vals * keep)
    ix = pit.PitIndex.empty(n // 128, (n // 128) * n)
    ws = torch.empty(pit.pit_build_index_workspace(n, n, 1, 128, 0), dtype=torch.uint8, device="cuda")
    C = torch.empty((n, n), dtype=torch.float32, device="cuda")

    def step():
        pit.pit_build_index(At, 1, 128, 0, out=ix, ws=ws)
        pit.pit_sread_gemm(pit.PIT_GEMM_GATHER_K, At, B, ix, 128, n, n, n, out=C)

    t_eager = _time(step, a.reps)
    want = C.clone()
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
    out["graph_replay"] = {"point": "32x1 at 90 %, mt 128", "eager_us": round(t_eager * 1e6, 1),
                           "graph_us": round(_time(graph.replay, a.reps) * 1e6, 1), "graph_matches_eager": ok}

    # A row-major [m][k], zeros in blocks of 1 token x 64 channels: PIT-axis m inside k-slabs of 64
    # (GATHER_M, the slabs' partial products are added in strips of C held in LDS)
    out["gemm_row_major_1x64"] = []
    for s in (0.5, 0.9, 0.95, 0.99):
        keep = wl.iid_block_mask(n, n, 1, 64, s, seed=int(s * 100) + 7)
        A = bf16(vals * keep)
        ix = pit.PitIndex.empty(n // 64, (n // 64) * n)
        ws = torch.empty(pit.pit_build_index_workspace(n, n, 1, 64, 0), dtype=torch.uint8, device="cuda")

        def step_m():
            pit.pit_build_index(A, 1, 64, 0, out=ix, ws=ws)
            pit.pit_sread_gemm(pit.PIT_GEMM_GATHER_M, A, B, ix, 64, n, n, n, out=C)

        t = _time(step_m, a.reps)
        cover = int(ix.seg_ptr[-1].item()) / float((n // 64) * n)
        out["gemm_row_major_1x64"].append({"sparsity": s, "cover_1x64": round(cover, 4), "step_us": round(t * 1e6, 1),
                                           "speedup_vs_hipblaslt": round(t_dense / t, 3)})

    # Section 5.4: index build alone on byte masks, 99 % sparsity
    for gr in (1, 16, 32):
        m = torch.from_numpy(wl.iid_block_mask(n, n, gr, gr, 0.99, seed=gr)).cuda()
        ix = pit.PitIndex.empty(n // gr, (n // gr) * (n // gr))
        ws = torch.empty(pit.pit_build_index_workspace(n, n, gr, gr, 1), dtype=torch.uint8, device="cuda")
        t = _time(lambda: pit.pit_build_index(m, gr, gr, 1, out=ix, ws=ws), a.reps)
        out["index_build"].append({"mask": [n, n], "micro_tile": [gr, gr], "us": round(t * 1e6, 1),
                                   "GB_per_s": round(n * n / t / 1e9, 1)})
    if not a.table:
        print(json.dumps(out))
        return
    print(f"4096^3 bf16, sparse operand K-major; hipBLASLt dense GEMM {out['dense_hipblaslt_us']} us; step = index build + product")
    print("cover / step us per kernel; sel = Algorithm 1 with the profiled costs; best = measured fastest")
    hdr = f"{'granularity':>11} {'sparsity':>8} | " + " | ".join(f"{k:>16}" for k in ("gather_k 128", "gather_k 64", "gather_k 32")) + \
          f" | {'dense_k':>8} | {'sel':>12} {'best':>12} {'sel/best':>8} {'vs lib':>6}"
    for key, title in (("gemm", "Section 5.3 sweep"), ("table3", "Table 3 granularities")):
        print("\n" + title + "\n" + hdr)
        for r in out[key]:
            k = r["kernels"]
            gm, gk = r["granularity_tokens_x_channels"]
            cells = " | ".join(f"{k[f'gather_k_{mt}']['cover']:>6.3f} {k[f'gather_k_{mt}']['step_us']:>8.1f}" + " " for mt in MTS)
            print(f"{gm:>7}x{gk:<3} {r['sparsity']:>8} | {cells} | {k['dense_k']['step_us']:>8.1f} | {r['selected']:>12} {r['fastest']:>12} "
                  f"{r['selected_over_fastest']:>8} {r['speedup_vs_hipblaslt_selected']:>6}")
    print("\ngraph replay:", out["graph_replay"])
    print("row-major operand, zeros 1 x 64 (GATHER_M k-slabs):", out["gemm_row_major_1x64"])
    print("index build alone (Section 5.4), byte masks at 99 %:", out["index_build"])


if __name__ == "__main__":
    main()
