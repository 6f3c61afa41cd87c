"""Pins for the oracle's kernel selection (Algorithm 1 of the paper): brute force on tiny inputs,
closed forms under iid block sparsity (the model behind Table 3), and the special cases."""
import itertools

import numpy as np
import pytest

from oracle import pit_oracle as orc
from paper_2301_10936_amd import workloads as wl


def _literal_selection(samples, candidates):
    """Algorithm 1 written with nested loops over tiles and elements, sharing nothing with the oracle."""
    best, best_cost = -1, float("inf")
    for ci, c in enumerate(candidates):
        r, q = c["mt_rows"], c["mt_cols"]
        cost = 0.0
        for D in samples:
            n = 0
            for i in range(0, D.shape[0], r):
                for j in range(0, D.shape[1], q):
                    hit = c.get("dense", False)
                    for a in range(r):
                        for b in range(q):
                            if float(D[i + a, j + b]) != 0.0:
                                hit = True
                    n += 1 if hit else 0
            cost += c.get("fixed_cost", 0.0) + n * c["tile_cost"]
        if cost < best_cost:
            best, best_cost = ci, cost
    return best


CANDS = [
    {"mt_rows": 1, "mt_cols": 2, "tile_cost": 1.0},
    {"mt_rows": 1, "mt_cols": 4, "tile_cost": 1.7},
    {"mt_rows": 2, "mt_cols": 1, "tile_cost": 1.1},
    {"mt_rows": 4, "mt_cols": 4, "tile_cost": 5.5},
    {"mt_rows": 4, "mt_cols": 4, "tile_cost": 4.0, "dense": True},
]


def test_brute_force_on_small_tensors():
    g = np.random.default_rng(5)
    for trial in range(60):
        density = g.choice([0.02, 0.1, 0.3, 0.6, 0.95])
        samples = [(g.random((8, 8)) < density).astype(np.float32) * g.standard_normal((8, 8)).astype(np.float32)
                   for _ in range(int(g.integers(1, 4)))]
        best, costs = orc.select_kernel(samples, CANDS)
        assert best == _literal_selection(samples, CANDS)
        assert costs[best] == min(costs) and len(costs) == len(CANDS)


def test_every_4x4_block_mask_of_an_8x8_tensor():
    for bits in itertools.product([0, 1], repeat=4):
        D = np.kron(np.array(bits, dtype=np.float32).reshape(2, 2), np.ones((4, 4), dtype=np.float32))
        best, costs = orc.select_kernel([D], CANDS)
        assert best == _literal_selection([D], CANDS)
        live = sum(bits)
        # block-structured data: the 4x4 micro-tile covers exactly the live blocks, the dense entry all four
        assert costs[3] == pytest.approx(live * 5.5) and costs[4] == pytest.approx(4 * 4.0)


def test_special_cases():
    z = np.zeros((8, 8), dtype=np.float32)
    best, costs = orc.select_kernel([z], CANDS)
    assert costs[:4] == [0.0, 0.0, 0.0, 0.0] and best == 0           # nothing to cover: first of the equals
    assert orc.select_kernel([], CANDS) == (0, [0.0] * 5)             # no samples: every cost is zero
    full = np.ones((8, 8), dtype=np.float32)
    best, costs = orc.select_kernel([full], CANDS)
    assert best == 4                                                  # dense data: the dense kernel is cheapest per element
    assert costs == pytest.approx([32 * 1.0, 16 * 1.7, 32 * 1.1, 4 * 5.5, 4 * 4.0])
    nz = np.zeros((8, 8), dtype=np.float32)
    nz[3, 5] = -0.0
    assert orc.select_kernel([nz], CANDS)[1][:4] == [0.0, 0.0, 0.0, 0.0]   # -0 is zero
    nz[3, 5] = np.nan
    assert orc.select_kernel([nz], CANDS)[1][:4] == pytest.approx([1.0, 1.7, 1.1, 5.5])   # NaN is not


@pytest.mark.parametrize("gran,sparsity", [(2, 0.95), (4, 0.95), (8, 0.99), (32, 0.95)])
def test_costs_follow_the_iid_cover_model(gran, sparsity):
    """Under iid block sparsity (granularity gran x 1, a block is zero with probability s) a micro-tile
    of mt x 1 is empty with probability s**(mt/gran) (the closed form behind Table 3), so the cost
    of a candidate is close to (#micro-tiles) * (1 - s**(mt/gran)) * tile_cost."""
    D = wl.iid_block_mask(1024, 512, gran, 1, sparsity, seed=gran)
    cands = [{"mt_rows": mt, "mt_cols": 1, "tile_cost": 1.0 + 0.05 * mt} for mt in (gran, 2 * gran, 4 * gran)
             if mt <= 64]
    _, costs = orc.select_kernel([D], cands)
    for c, cost in zip(cands, costs):
        ntiles = (1024 // c["mt_rows"]) * 512
        want = ntiles * (1.0 - sparsity ** (c["mt_rows"] / gran)) * c["tile_cost"]
        assert cost == pytest.approx(want, rel=0.08)


def test_selection_moves_to_dense_as_sparsity_drops():
    """With a per-element cost that favours big tiles, the choice goes small micro-tile -> big
    micro-tile -> dense as the data fills up (the fallback the paper describes), never back."""
    cands = [{"mt_rows": 2, "mt_cols": 1, "tile_cost": 2.0 * 1.00},
             {"mt_rows": 16, "mt_cols": 1, "tile_cost": 16.0 * 0.30},
             {"mt_rows": 16, "mt_cols": 1, "tile_cost": 16.0 * 0.25, "dense": True}]
    picks = []
    for s in (0.995, 0.98, 0.9, 0.7, 0.4, 0.1, 0.0):
        D = wl.iid_block_mask(512, 256, 2, 1, s, seed=11)
        picks.append(orc.select_kernel([D], cands)[0])
    assert picks[0] == 0 and picks[-1] == 2
    assert picks == sorted(picks)


def test_fixed_cost_is_added_once_per_sample():
    """The constant part of a run (the library's addition to the paper's proportional model): hand-computed costs
    on a tensor whose covers are known, and a case where the constant alone moves the choice."""
    D = np.zeros((8, 8), dtype=np.float32)
    D[0, 0] = D[5, 6] = 1.0                          # two non-zeros: 2 tiles of 1 x 2, 2 of 4 x 4, grid of 4 x 4 = 4
    cands = [{"mt_rows": 1, "mt_cols": 2, "tile_cost": 1.0, "fixed_cost": 10.0},
             {"mt_rows": 4, "mt_cols": 4, "tile_cost": 3.0, "fixed_cost": 2.5},
             {"mt_rows": 4, "mt_cols": 4, "tile_cost": 2.0, "dense": True}]
    best, costs = orc.select_kernel([D, D, D], cands)
    assert costs == [3 * (10.0 + 2 * 1.0), 3 * (2.5 + 2 * 3.0), 3 * (4 * 2.0)]
    assert best == 2 == _literal_selection([D, D, D], cands)
    cands[0]["fixed_cost"] = 0.0                     # the paper's formula: the fine micro-tile wins
    assert orc.select_kernel([D], cands)[0] == 0 == _literal_selection([D], cands)
    g = np.random.default_rng(11)
    for _ in range(30):
        samples = [(g.random((8, 8)) < 0.2).astype(np.float32) for _ in range(2)]
        cc = [dict(c, fixed_cost=float(g.choice([0.0, 1.0, 4.0]))) for c in CANDS]
        assert orc.select_kernel(samples, cc)[0] == _literal_selection(samples, cc)
