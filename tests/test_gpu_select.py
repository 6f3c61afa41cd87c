"""GPU parity: pit_cover_count (CoverAlgo of Algorithm 1) vs the oracle, and the selection made from
its counts vs the oracle's selection."""
import numpy as np
import pytest
import torch

from oracle import pit_oracle as orc
from paper_2301_10936_amd import workloads as wl
from tests.gpu_util import to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pit():
    from paper_2301_10936_amd import pit as p
    return p


@pytest.mark.parametrize("rows,cols,mt_rows,mt_cols", [
    (256, 512, 1, 32), (256, 512, 1, 64), (300, 192, 1, 8), (256, 256, 2, 1), (512, 128, 16, 1),
    (512, 128, 32, 1), (96, 160, 4, 4), (64, 64, 1, 1), (128, 2048, 1, 512), (37, 41, 1, 1)])
@pytest.mark.parametrize("kind", ["u8", "bf16"])
def test_cover_count_matches_oracle(pit, rows, cols, mt_rows, mt_cols, kind):
    g = np.random.default_rng(rows * 7 + cols + mt_rows + mt_cols)
    density = g.choice([0.001, 0.02, 0.2])
    keep = g.random((rows, cols)) < density
    if kind == "u8":
        src = keep.astype(np.uint8) * g.integers(1, 255, size=(rows, cols)).astype(np.uint8)
    else:
        src = wl.to_bf16_bits(np.where(keep, g.standard_normal((rows, cols)), 0.0).astype(np.float32))
    cnt = pit.pit_cover_count(to_dev(src), mt_rows, mt_cols)
    torch.cuda.synchronize()
    assert int(cnt.item()) == orc.cover_count(src, mt_rows, mt_cols)


def test_cover_count_special_values_and_degenerate_inputs(pit):
    src = np.zeros((64, 64), dtype=np.float32)
    assert int(pit.pit_cover_count(to_dev(src), 1, 32).item()) == 0
    src[3, 40] = -0.0
    assert int(pit.pit_cover_count(to_dev(src), 1, 32).item()) == 0          # -0 is zero
    src[3, 40] = np.nan
    src[9, 1] = np.inf
    src[10, 33] = 1e-45                                                       # subnormal
    assert int(pit.pit_cover_count(to_dev(src), 1, 32).item()) == orc.cover_count(src, 1, 32) == 3
    full = np.ones((64, 128), dtype=np.uint8)
    assert int(pit.pit_cover_count(to_dev(full), 2, 1).item()) == 32 * 128
    with pytest.raises(pit.PitError):
        pit.pit_cover_count(to_dev(full), 3, 1)                               # 64 % 3 != 0
    # a strided view: only the viewed columns count
    wide = torch.ones((64, 96), dtype=torch.uint8, device="cuda")
    wide[:, :64] = 0
    assert int(pit.pit_cover_count(wide[:, :64], 1, 16).item()) == 0
    assert int(pit.pit_cover_count(wide[:, 32:96], 1, 16).item()) == 64 * 2


def test_selection_from_gpu_counts_equals_oracle_selection(pit):
    """Table 3's setting at reduced size: iid sparsity at granularity g x 1; candidates are column
    micro-tiles of several heights plus the dense kernel; counts come from the GPU."""
    cands = [{"mt_rows": 8, "mt_cols": 1, "tile_cost": 8 * 1.00},
             {"mt_rows": 16, "mt_cols": 1, "tile_cost": 16 * 0.60},
             {"mt_rows": 32, "mt_cols": 1, "tile_cost": 32 * 0.40},
             {"mt_rows": 32, "mt_cols": 1, "tile_cost": 32 * 0.30, "dense": True}]
    picks = []
    for gran, s in [(2, 0.99), (2, 0.95), (8, 0.95), (32, 0.95), (32, 0.5), (2, 0.3)]:
        samples = [wl.iid_block_mask(1024, 1024, gran, 1, s, seed=100 + k) for k in range(2)]
        dev = [to_dev(D) for D in samples]
        counts = [[pit.pit_cover_count(d, c["mt_rows"], c["mt_cols"]) for c in cands] for d in dev]
        torch.cuda.synchronize()
        num = [[int(t.item()) for t in row] for row in counts]
        grid = [[(1024 // c["mt_rows"]) * 1024 for c in cands] for _ in samples]
        best, costs = pit.pit_select_kernel(cands, num, grid)
        want_best, want_costs = orc.select_kernel(samples, cands)
        assert num == [[orc.cover_count(D, c["mt_rows"], c["mt_cols"]) for c in cands] for D in samples]
        assert best == want_best and np.allclose(costs, want_costs, rtol=1e-12)
        picks.append(best)
    assert picks[0] != 3 and picks[-1] == 3      # very sparse: a sparse kernel; mostly dense data: the dense kernel


def test_cover_count_at_table3_size(pit):
    """4096 x 4096 mask, the size of the paper's micro-tile search: count vs the closed form s**(mt/g)."""
    D = wl.iid_block_mask(4096, 4096, 2, 1, 0.95, seed=3)
    d = to_dev(D)
    for mt in (2, 8, 16, 32):
        got = int(pit.pit_cover_count(d, mt, 1).item())
        assert got == orc.cover_count(D, mt, 1)
        ntiles = (4096 // mt) * 4096
        assert got == pytest.approx(ntiles * (1 - 0.95 ** (mt / 2)), rel=0.01)


# ------------------------------------------------------------------ the dense kernel and Algorithm 1 end to end
@pytest.mark.parametrize("mt", [128, 64, 32])
def test_dense_kernel_is_the_product_with_no_index(pit, mt):
    """PIT_GEMM_DENSE_K: identity addressing, every k multiplied; exact on integers, zeros in A or not."""
    for prob in (None, 0.3):
        w = wl.relu_ffn(M=384, K=333, N=256, seed=mt, integer=True, channel_live_prob=prob)
        Xt, W = to_dev(w.Xt), to_dev(w.W)
        C = torch.full((w.M, w.N), 5.0, device="cuda")
        pit.pit_sread_gemm(pit.PIT_GEMM_DENSE_K, Xt, W, None, mt, w.M, w.N, w.K, out=C)
        torch.cuda.synchronize()
        assert np.array_equal(C.cpu().numpy().astype(np.float64), orc.gemm_at(w.Xt, w.W))
    with pytest.raises(pit.PitError) as e:
        pit.pit_sread_gemm(pit.PIT_GEMM_DENSE_K, Xt, W, None, 48, w.M, w.N, w.K)
    assert e.value.code == pit.PIT_ESHAPE


def _gather_k_candidates(costs):
    """The (dense tile, PIT-axis) pairs the GATHER_K family offers on a K-major operand [K, M]: micro-tiles of
    128, 64 and 32 consecutive m of one k, and the dense kernel."""
    return [{"mt_rows": 1, "mt_cols": 128, "tile_cost": costs[0]}, {"mt_rows": 1, "mt_cols": 64, "tile_cost": costs[1]},
            {"mt_rows": 1, "mt_cols": 32, "tile_cost": costs[2]}, {"mt_rows": 1, "mt_cols": 128, "tile_cost": costs[3], "dense": True}]


@pytest.mark.parametrize("costs,want", [((1.0, 9.0, 9.0, 9.0), 0), ((9.0, 1.0, 9.0, 9.0), 1), ((9.0, 9.0, 1.0, 9.0), 2),
                                        ((9.0, 9.0, 9.0, 0.01), 3)])
def test_select_and_run_launches_the_winner(pit, costs, want):
    """Whatever Algorithm 1 selects, the product must be the oracle's; the selection itself must be the oracle's
    selection from the same samples, with CoverAlgo's counts taken on the GPU."""
    w = wl.relu_ffn(M=512, K=420, N=256, seed=17, integer=True, channel_live_prob=0.3, live_block=32)
    samples = [wl.relu_ffn(M=512, K=420, N=8, seed=18 + i, integer=True, channel_live_prob=0.3, live_block=32).Xt for i in range(2)]
    cands = _gather_k_candidates(costs)
    num = [[int(pit.pit_cover_count(to_dev(D), c["mt_rows"], c["mt_cols"]).item()) for c in cands] for D in samples]
    grid = [[D.shape[0] * (D.shape[1] // c["mt_cols"]) for c in cands] for D in samples]
    C = torch.full((w.M, w.N), -3.0, device="cuda")
    _, chosen = pit.pit_select_and_run_gemm(cands, num, grid, to_dev(w.Xt), to_dev(w.W), w.M, w.N, w.K, out=C)
    torch.cuda.synchronize()
    assert chosen == want == orc.select_kernel([orc.to_f64(D) for D in samples], cands)[0]
    assert np.array_equal(C.cpu().numpy().astype(np.float64), orc.gemm_at(w.Xt, w.W))


def test_select_and_run_with_the_profiled_costs(pit):
    """With the committed profile of this GPU type, on the product the profile was taken on (4096^3): iid ReLU
    zeros (98 % of the 32 x 1 micro-tiles live) fall back to the dense kernel and zeros correlated across tokens
    pick a sparse kernel (paper Section 3.2).  The product of whichever kernel ran is checked on sampled rows."""
    import json
    import os
    here = os.path.dirname(os.path.abspath(pit.__file__))
    prof = json.load(open(os.path.join(here, "tile_cost_mi355x.json")))["candidates"]
    names = ["gather_k", "gather_k_64", "gather_k_32", "dense_k"]
    cands = _gather_k_candidates([prof[k]["step_ns_per_tile"] for k in names])
    for c, k in zip(cands, names):
        c["fixed_cost"] = prof[k]["step_fixed_ns"]
    n = 4096
    picks = {}
    rows = np.random.default_rng(3).choice(n, 64, replace=False)
    for name, prob in (("iid", None), ("correlated", 0.1)):
        w = wl.relu_ffn(M=n, K=n, N=n, seed=1, channel_live_prob=prob)
        Xt = to_dev(w.Xt)
        num = [[int(pit.pit_cover_count(Xt, 1, c["mt_cols"]).item()) for c in cands]]
        grid = [[w.K * (w.M // c["mt_cols"]) for c in cands]]
        C, chosen = pit.pit_select_and_run_gemm(cands, num, grid, Xt, to_dev(w.W), w.M, w.N, w.K)
        torch.cuda.synchronize()
        picks[name] = chosen
        assert num[0][:3] == [orc.cover_count(w.Xt, 1, mt) for mt in (128, 64, 32)]
        ref = orc.gemm_at(np.ascontiguousarray(w.Xt[:, rows]), w.W)          # rows of C = columns of the K-major operand
        mx, fro = orc.rel_errors(C[to_dev(rows)].cpu().numpy(), ref)
        assert mx <= 2e-2 and fro <= 1e-3
    assert picks["iid"] == 3 and picks["correlated"] in (0, 1, 2)
