"""GPU parity: the sparsity on the *other* operand and in the backward pass, served by the same entry points.

The method only asks which axis of the product carries the permutation (Table 1, Figure "matmul example"):
* block-pruned weights W[K][N] (Section 5.2, sparse training) are the K-major sparse operand of C^T = W^T . X^T
  when the activations are kept channel-major, i.e. GATHER_K with the operand roles swapped;
* weights pruned in 32 x 1 blocks along k are the row-major sparse operand W^T[N][K] of the k-slab mode;
* padding-free training (Section 5.1): dgrad is the forward call with W^T, wgrad sums over the valid tokens
  only -- tokens are the reduction axis, so the token rows are the k-list of GATHER_K.
"""
import numpy as np
import pytest
import torch

from oracle import pit_oracle as orc
from paper_2301_10936_amd import workloads as wl
from tests.gpu_util import assert_close, assert_index_equal, dev, to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pit():
    from paper_2301_10936_amd import pit as p
    return p


def _block_pruned(g, K, N, bk, bn, sparsity, integer=True):
    keep = np.repeat(np.repeat(g.random((K // bk, N // bn)) >= sparsity, bk, axis=0), bn, axis=1)
    vals = g.integers(-3, 4, size=(K, N)) if integer else g.standard_normal((K, N)) * 0.05
    vals = np.where(vals == 0, 1, vals) if integer else vals           # kept blocks hold no zeros of their own
    return (vals * keep).astype(np.float32)


@pytest.mark.parametrize("K,N,M,sparsity", [(256, 256, 128, 0.5), (512, 384, 256, 0.9), (192, 128, 384, 0.0), (320, 256, 128, 1.0)])
def test_weights_pruned_in_32x64_blocks(pit, K, N, M, sparsity):
    """C^T[N][M] = W^T . X^T with W zero in blocks of 32 k x 64 n; the index lists, for every block of
    128 output features, the k-rows of W that are not all zero."""
    g = np.random.default_rng(K + N + M)
    W = wl.to_bf16_bits(_block_pruned(g, K, N, 32, 64, sparsity))
    Xt = wl.to_bf16_bits(g.integers(-3, 4, size=(K, M)).astype(np.float32))
    tW, tX = to_dev(W), to_dev(Xt)
    ix = pit.pit_build_index(tW, 1, 128, 0)
    Ct = pit.pit_sread_gemm(pit.PIT_GEMM_GATHER_K, tW, tX, ix, 128, N, M, K)
    torch.cuda.synchronize()
    want_ix = orc.build_index(W, 1, 128, 0)
    assert_index_equal(ix, want_ix)
    if 0.0 < sparsity < 1.0:
        assert 0 < int(want_ix[0][-1]) < K * (N // 128)                # the pruning is visible at 1 x 128
    assert np.array_equal(Ct.cpu().numpy().astype(np.float64), orc.gemm_at(W, Xt))


@pytest.mark.parametrize("K,N,M,sparsity", [(256, 200, 128, 0.8), (128, 130, 256, 0.95), (96, 64, 128, 0.0)])
def test_weights_pruned_in_32x1_blocks(pit, K, N, M, sparsity):
    """W zero in runs of 32 k per output feature: W^T[N][K] is the row-major sparse operand of the k-slab
    mode (a slab lists the output features with a live run), C^T[N][M] is accumulated slab by slab."""
    g = np.random.default_rng(K * 3 + N)
    Wt = wl.to_bf16_bits(_block_pruned(g, K, N, 32, 1, sparsity).T.copy())     # [N][K]
    Xt = wl.to_bf16_bits(g.integers(-3, 4, size=(K, M)).astype(np.float32))
    tW, tX = to_dev(Wt), to_dev(Xt)
    ix = pit.pit_build_index(tW, 1, 32, 0)
    Ct = torch.full((N, M), 5.0, device=dev())
    pit.pit_sread_gemm(pit.PIT_GEMM_GATHER_M, tW, tX, ix, 32, N, M, K, out=Ct)
    torch.cuda.synchronize()
    assert_index_equal(ix, orc.build_index(Wt, 1, 32, 0))
    assert np.array_equal(Ct.cpu().numpy().astype(np.float64), orc.gemm(Wt, Xt))


@pytest.mark.parametrize("batch,max_len,hidden,out", [(3, 64, 128, 128), (4, 150, 256, 384)])
def test_padding_free_backward(pit, batch, max_len, hidden, out):
    """dX = dY . W^T on the valid rows (the forward call with W^T) and dW = X^T . dY summed over the
    valid tokens only: X[T][hidden] is K-major for that product, and the k-list of every 128-wide block
    of hidden units is the list of tokens whose rows are not zero."""
    w = wl.padded_linear(batch=batch, max_len=max_len, hidden=hidden, out=out, min_len=1, seed=batch + out, integer=True)
    g = np.random.default_rng(out)
    T = batch * max_len
    X = w.X.copy()
    X[w.row_mask == 0] = 0                                             # padding rows are zero rows
    valid = np.flatnonzero(w.row_mask)
    Xf = orc.to_f64(X)
    X[valid[Xf[valid].any(axis=1) == 0], 0] = wl.to_bf16_bits(np.ones(1, np.float32))[0]   # no valid row is all zero
    dY = g.integers(-3, 4, size=(T, out)).astype(np.float32) * w.row_mask[:, None]
    dYb = wl.to_bf16_bits(dY)
    Wt = wl.to_bf16_bits(orc.to_f64(w.W).T.astype(np.float32).copy())  # [out][hidden]

    # dgrad: rows from the mask
    tdY, tWt, tmask = to_dev(dYb), to_dev(Wt), to_dev(w.row_mask.reshape(-1, 1))
    ixm = pit.pit_build_index(tmask, 1, 1, 0)
    dX = torch.full((T, hidden), 9.0, device=dev())
    pit.pit_sread_gemm(pit.PIT_GEMM_GATHER_M, tdY, tWt, ixm, out, T, hidden, out, out=dX)
    # wgrad: tokens are the reduction axis
    tX = to_dev(X)
    ixk = pit.pit_build_index(tX, 1, 128, 0)
    dW = pit.pit_sread_gemm(pit.PIT_GEMM_GATHER_K, tX, tdY, ixk, 128, hidden, out, T)
    torch.cuda.synchronize()

    assert np.array_equal(dX.cpu().numpy().astype(np.float64), orc.gemm_rows_masked(dYb, w.row_mask, Wt))
    sp, idx, _ = ixk.to_host()
    for s in range(hidden // 128):                                     # every block lists exactly the valid tokens
        lst = idx[sp[s]:sp[s + 1]]
        assert set(lst.tolist()) <= set(valid.tolist())
    assert_index_equal(ixk, orc.build_index(X, 1, 128, 0))
    assert np.array_equal(dW.cpu().numpy().astype(np.float64), orc.gemm_at(X, dYb))


def test_weights_pruned_float_values(pit):
    g = np.random.default_rng(21)
    K, N, M = 1024, 512, 256
    W = wl.to_bf16_bits(_block_pruned(g, K, N, 32, 64, 0.9, integer=False))
    Xt = wl.to_bf16_bits(g.standard_normal((K, M)).astype(np.float32))
    tW, tX = to_dev(W), to_dev(Xt)
    ix = pit.pit_build_index(tW, 1, 128, 0)
    Ct = pit.pit_sread_gemm(pit.PIT_GEMM_GATHER_K, tW, tX, ix, 128, N, M, K)
    torch.cuda.synchronize()
    assert_close(Ct, orc.gemm_at(W, Xt), "block-pruned weights")
