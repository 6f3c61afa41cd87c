"""Pins for the oracle's GEMM definitions (no GPU)."""
import itertools

import numpy as np
import pytest

from oracle import pit_oracle as orc
from paper_2301_10936_amd import workloads as wl


def brute_matmul(A, B):
    """C[i][j] = sum_k A[i][k]*B[k][j] with Python floats (fp64), separate from the oracle."""
    M, K, N = len(A), len(B), len(B[0])
    return [[sum(A[i][k] * B[k][j] for k in range(K)) for j in range(N)] for i in range(M)]


def test_bruteforce_8x8_all_4x4_tile_masks():
    g = np.random.default_rng(0)
    A0 = g.integers(-4, 5, (8, 8)).astype(np.float16)
    B = g.integers(-4, 5, (8, 8)).astype(np.float16)
    for pattern in range(16):
        keep = np.array([[pattern >> (2 * r + c) & 1 for c in range(2)] for r in range(2)])
        A = (A0 * np.kron(keep, np.ones((4, 4)))).astype(np.float16)
        C = orc.gemm(A, B)
        assert C.tolist() == brute_matmul(A.astype(float).tolist(), B.astype(float).tolist())
        for pit_dim in (0, 1):
            sp, ix, _ = orc.build_index(A, 4, 4, pit_dim)
            assert np.array_equal(orc.gemm_over_index(A, B, sp, ix, 4, 4, pit_dim), C)


def test_bruteforce_8x8_all_row_masks():
    g = np.random.default_rng(1)
    A0 = g.standard_normal((8, 8)).astype(np.float16)
    B = g.standard_normal((8, 8)).astype(np.float16)
    for pattern in range(256):
        mask = np.array([pattern >> r & 1 for r in range(8)], dtype=np.uint8)
        C = orc.gemm_rows_masked(A0, mask, B)
        Az = (A0.astype(float) * mask[:, None]).tolist()
        ref = np.array(brute_matmul(Az, B.astype(float).tolist()))
        assert np.allclose(C, ref, rtol=0, atol=1e-13)
        assert np.all(C[mask == 0] == 0.0)


def test_bf16_operands_decode_exactly():
    bits = np.array([[0x3F80, 0xC000], [0x3E00, 0x0000]], dtype=np.uint16)   # [[1,-2],[0.125,0]]
    B = np.array([[3.0, 1.0], [0.5, -1.0]], dtype=np.float32)
    assert orc.gemm(bits, B).tolist() == [[2.0, 3.0], [0.375, 0.125]]
    assert orc.gemm_at(bits, B).tolist() == [[3.0 + 0.0625, 1.0 - 0.125], [-6.0, -2.0]]


def test_closed_forms():
    g = np.random.default_rng(2)
    B = g.standard_normal((16, 5)).astype(np.float32)
    assert np.array_equal(orc.gemm(np.eye(16, dtype=np.float16), B), B.astype(np.float64))
    ones = np.ones((3, 16), dtype=np.float16)
    assert np.allclose(orc.gemm(ones, B), np.tile(B.astype(np.float64).sum(0), (3, 1)), atol=1e-12)
    # a transposed operand would break this non-square, non-symmetric case
    A = np.arange(6, dtype=np.float32).reshape(2, 3)
    Bm = np.arange(12, dtype=np.float32).reshape(3, 4)
    assert orc.gemm(A, Bm).tolist() == [[20, 23, 26, 29], [56, 68, 80, 92]]
    assert orc.gemm_at(np.ascontiguousarray(A.T), Bm).tolist() == [[20, 23, 26, 29], [56, 68, 80, 92]]


@pytest.mark.parametrize("seed", [0, 1])
def test_sparse_loop_equals_dense_with_zeros(seed):
    w = wl.microtile_gemm(M=96, K=128, N=40, mt_k=32, p_keep=0.2, seed=seed)
    dense = orc.gemm(w.A, w.B)
    sp, ix, _ = orc.build_index(w.A, 1, 32, 0)
    sparse = orc.gemm_over_index(w.A, w.B, sp, ix, 1, 32, 0)
    assert np.abs(sparse - dense).max() <= 1e-12 * np.abs(dense).max()
    # on integers both are exact, so identical
    wi = wl.microtile_gemm(M=96, K=128, N=40, mt_k=32, p_keep=0.2, seed=seed, integer=True)
    sp, ix, _ = orc.build_index(wi.A, 1, 32, 0)
    assert np.array_equal(orc.gemm_over_index(wi.A, wi.B, sp, ix, 1, 32, 0), orc.gemm(wi.A, wi.B))
    # dropping one listed micro-tile must change the answer (the check can fail)
    if len(ix) > 1:
        sp2 = sp.copy()
        sp2[1:] -= 1
        bad = orc.gemm_over_index(wi.A, wi.B, sp2, ix[1:], 1, 32, 0)
        assert not np.array_equal(bad, orc.gemm(wi.A, wi.B))


def test_permutation_round_trips_are_bit_identical():
    """Rows of A (with rows of C) and the k-axis of A and B jointly are PIT-axes (Table 1):
    permuting and un-permuting leaves C unchanged; exact on small integers."""
    w = wl.microtile_gemm(M=64, K=96, N=48, mt_k=32, p_keep=0.3, seed=7, integer=True)
    C = orc.gemm(w.A, w.B)
    g = np.random.default_rng(3)
    pm = g.permutation(64)
    Cp = orc.gemm(w.A[pm], w.B)
    back = np.empty_like(Cp)
    back[pm] = Cp
    assert np.array_equal(back, C)
    pk = g.permutation(96)
    assert np.array_equal(orc.gemm(w.A[:, pk], w.B[pk]), C)
    # a permutation applied to only one operand is NOT legal and must be caught
    assert not np.array_equal(orc.gemm(w.A[:, pk], w.B), C)


def test_kmajor_and_rowmajor_agree():
    w = wl.relu_ffn(M=64, K=96, N=32, seed=4)
    X = np.ascontiguousarray(w.Xt.T)
    assert np.array_equal(orc.gemm_at(w.Xt, w.W), orc.gemm(X, w.W))


def test_padded_rows_are_zero_and_ignored():
    w = wl.padded_linear(batch=3, max_len=16, hidden=32, out=8, min_len=2, seed=5)
    Y = orc.gemm_rows_masked(w.X, w.row_mask, w.W)
    assert np.all(Y[w.row_mask == 0] == 0)
    X2 = w.X.copy()
    X2[w.row_mask == 0] = 0x7FC0          # NaN in the padding must not leak
    assert np.array_equal(orc.gemm_rows_masked(X2, w.row_mask, w.W)[w.row_mask == 1], Y[w.row_mask == 1])
    for b in range(3):                     # valid rows are left-aligned inside each sequence
        m = w.row_mask[b * 16:(b + 1) * 16]
        assert m[:w.lengths[b]].all() and not m[w.lengths[b]:].any()


def test_rel_errors_measure():
    ref = np.array([1.0, -2.0, 0.0, 4.0])
    got = ref + np.array([0.0, 0.02, 0.01, 0.0])
    mx, fro = orc.rel_errors(got, ref)
    rms = np.sqrt(np.mean(ref ** 2))
    assert np.isclose(mx, max(0.02 / max(2.0, rms), 0.01 / rms))
    assert np.isclose(fro, np.sqrt(0.02 ** 2 + 0.01 ** 2) / np.sqrt(21.0))
