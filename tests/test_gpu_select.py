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
