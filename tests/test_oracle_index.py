"""Pins for the oracle's index construction and CoverAlgo (no GPU)."""
import itertools
import os

import numpy as np
import pytest

from oracle import pit_oracle as orc
from paper_2301_10936_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def brute_index(src, mt_rows, mt_cols, pit_dim):
    """Literal nested loops over micro-tiles and their elements; written separately from the oracle."""
    rows, cols = len(src), len(src[0])
    gr, gc = rows // mt_rows, cols // mt_cols
    nseg = gc if pit_dim == 0 else gr
    npit = gr if pit_dim == 0 else gc
    seg_ptr, idx, bits = [0], [], []
    for s in range(nseg):
        for c in range(npit):
            tr, tc = (c, s) if pit_dim == 0 else (s, c)
            word = 0
            for r in range(mt_rows):
                for q in range(mt_cols):
                    v = src[tr * mt_rows + r][tc * mt_cols + q]
                    if v != 0:          # python: -0.0 != 0 is False, nan != 0 is True
                        word |= 1 << (r * mt_cols + q)
            if word:
                idx.append(c)
                bits.append(word)
        seg_ptr.append(len(idx))
    return seg_ptr, idx, bits


@pytest.mark.parametrize("mt_rows,mt_cols", [(1, 1), (1, 2), (2, 1), (2, 2)])
@pytest.mark.parametrize("pit_dim", [0, 1])
def test_exhaustive_masks_of_a_2x4_grid(mt_rows, mt_cols, pit_dim):
    """Every occupancy pattern of a 2 x 4 micro-tile grid, non-zero placed at a varying element."""
    rows, cols = 2 * mt_rows, 4 * mt_cols
    for pattern in range(256):
        src = np.zeros((rows, cols), dtype=np.float32)
        for t in range(8):
            if pattern >> t & 1:
                tr, tc = divmod(t, 4)
                e = (pattern + t) % (mt_rows * mt_cols)
                src[tr * mt_rows + e // mt_cols, tc * mt_cols + e % mt_cols] = 1.5
        sp, ix, bt = orc.build_index(src, mt_rows, mt_cols, pit_dim)
        bsp, bix, bbt = brute_index(src.tolist(), mt_rows, mt_cols, pit_dim)
        assert sp.tolist() == bsp and ix.tolist() == bix and bt.tolist() == bbt
        assert sp[-1] == bin(pattern).count("1")


def test_worked_example_by_hand():
    """A 4 x 8 tensor with 1 x 4 micro-tiles, answers written out by hand."""
    a = np.zeros((4, 8), dtype=np.float16)
    a[0, 1] = 1      # tile (0,0), element 1
    a[0, 3] = 2      # tile (0,0), element 3
    a[2, 4] = 3      # tile (2,1), element 0
    a[3, 0] = -1     # tile (3,0), element 0
    a[3, 7] = 5      # tile (3,1), element 3
    sp, ix, bt = orc.build_index(a, 1, 4, 0)       # PIT-axis = rows; segments = tile columns
    assert sp.tolist() == [0, 2, 4]
    assert ix.tolist() == [0, 3, 2, 3]
    assert bt.tolist() == [0b1010, 0b0001, 0b0001, 0b1000]
    sp, ix, bt = orc.build_index(a, 1, 4, 1)       # PIT-axis = columns; segments = rows
    assert sp.tolist() == [0, 1, 1, 2, 4]
    assert ix.tolist() == [0, 1, 0, 1]
    assert bt.tolist() == [0b1010, 0b0001, 0b0001, 0b1000]


def test_zero_test_special_values():
    a = np.zeros((1, 6), dtype=np.float32)
    a[0, 0] = -0.0
    a[0, 1] = np.nan
    a[0, 2] = np.inf
    a[0, 3] = 1e-45          # subnormal
    a[0, 4] = 0.0
    a[0, 5] = -1.0
    sp, ix, _ = orc.build_index(a, 1, 1, 1)
    assert ix.tolist() == [1, 2, 3, 5]
    # the same values as bf16 bit patterns: -0, nan, inf, smallest subnormal, +0, -1
    b = np.array([[0x8000, 0x7FC0, 0x7F80, 0x0001, 0x0000, 0xBF80]], dtype=np.uint16)
    sp, ix, _ = orc.build_index(b, 1, 1, 1)
    assert ix.tolist() == [1, 2, 3, 5]
    h = a.astype(np.float16)
    h[0, 3] = np.float16(6e-8)
    assert orc.build_index(h, 1, 1, 1)[1].tolist() == [1, 2, 3, 5]


@pytest.mark.parametrize("pit_dim", [0, 1])
def test_invariants_on_random_tensor(pit_dim):
    g = np.random.default_rng(5)
    src = (g.random((96, 160)) < 0.07) * g.standard_normal((96, 160))
    src = src.astype(np.float32)
    mt_rows, mt_cols = (1, 32) if pit_dim == 0 else (32, 1)
    sp, ix, bt = orc.build_index(src, mt_rows, mt_cols, pit_dim)
    nseg = len(sp) - 1
    assert sp[0] == 0 and np.all(np.diff(sp) >= 0)
    assert sp[-1] == orc.cover_count(src, mt_rows, mt_cols) == len(ix) == len(bt)
    covered = np.zeros_like(src, dtype=bool)
    for s in range(nseg):
        seg = ix[sp[s]:sp[s + 1]]
        assert np.all(np.diff(seg) > 0)                       # strictly ascending
        for j, c in enumerate(seg):
            tr, tc = (c, s) if pit_dim == 0 else (s, c)
            tile = src[tr * mt_rows:(tr + 1) * mt_rows, tc * mt_cols:(tc + 1) * mt_cols]
            assert np.any(tile != 0)                          # soundness
            assert bin(int(bt[sp[s] + j])).count("1") == np.count_nonzero(tile)
            covered[tr * mt_rows:(tr + 1) * mt_rows, tc * mt_cols:(tc + 1) * mt_cols] = True
    assert not np.any((src != 0) & ~covered)                  # completeness


def test_all_zero_and_all_full():
    z = np.zeros((8, 64), dtype=np.uint8)
    sp, ix, _ = orc.build_index(z, 1, 32, 0)
    assert sp.tolist() == [0, 0, 0] and ix.size == 0
    f = np.ones((8, 64), dtype=np.uint8)
    sp, ix, bt = orc.build_index(f, 1, 32, 0)
    assert sp.tolist() == [0, 8, 16] and ix.tolist() == list(range(8)) * 2
    assert np.all(bt == 0xFFFFFFFF)


def test_route_index_is_stable_counting_sort():
    g = np.random.default_rng(11)
    eid = g.integers(0, 7, size=200).astype(np.int32)
    sp, ix = orc.route_index(eid, 7)
    assert sorted(ix.tolist()) == list(range(200))                       # a permutation of the tokens
    assert np.array_equal(np.diff(sp), np.bincount(eid, minlength=7))
    assert np.array_equal(ix, np.argsort(eid, kind="stable"))            # library routine, special case
    # same thing through the generic builder on the one-hot routing matrix
    onehot = np.zeros((200, 7), dtype=np.uint8)
    onehot[np.arange(200), eid] = 1
    sp2, ix2, _ = orc.build_index(onehot, 1, 1, 0)
    assert np.array_equal(sp, sp2) and np.array_equal(ix, ix2)


def _table3_rows():
    rows = []
    with open(os.path.join(GOLDEN, "table3_cover.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                rows.append([float(x) for x in line.split()])
    return rows


@pytest.mark.parametrize("row", _table3_rows())
def test_cover_ratio_matches_table3(row):
    """CoverAlgo on a seeded iid pattern reproduces the printed 'sparsity after cover' (Table 3).

    The printed figures are single samples on a 4096 x 4096 tensor; the closed form is
    s**(g_mt/g).  Both the closed form and the paper's sample must be within 0.15 points.
    """
    g_r, g_c, s_pct, mt_r, mt_c, printed = row
    g_r, g_c, mt_r, mt_c = int(g_r), int(g_c), int(mt_r), int(mt_c)
    mask = wl.iid_block_mask(4096, 4096, g_r, g_c, s_pct / 100.0, seed=int(1000 * s_pct + g_r))
    got = 100.0 * orc.sparsity_after_cover(mask, mt_r, mt_c)
    closed = 100.0 * (s_pct / 100.0) ** ((mt_r * mt_c) / (g_r * g_c))
    assert abs(got - closed) < 0.15
    assert abs(got - printed) < 0.15
    # the index builder must list exactly CoverAlgo's count, whichever axis is the PIT-axis
    if mt_r == 32:
        sp, ix, _ = orc.build_index(mask, mt_r, mt_c, 1)
        assert sp[-1] == orc.cover_count(mask, mt_r, mt_c)


def test_relu_microtile_density_closed_form():
    """ReLU(N(-1.2,1)) zeros are iid with P(zero)=Phi(1.2); a 32-token micro-tile is non-empty
    with probability 1 - Phi(1.2)**32 = 0.980."""
    from math import erf, sqrt
    w = wl.relu_ffn(M=1024, K=2048, N=8, seed=3)
    pz = 0.5 * (1 + erf(1.2 / sqrt(2)))
    assert abs(np.mean(orc.is_nonzero(w.Xt) == 0) - pz) < 2e-3
    dens = orc.cover_count(w.Xt, 1, 32) / (2048 * 1024 / 32)
    assert abs(dens - (1 - pz ** 32)) < 3e-3
