"""Pins for the oracle's producer of activation sparsity (oracle.relu, oracle.relu_channel_major).  CPU only."""
import numpy as np

from oracle import pit_oracle as orc
from paper_2301_10936_amd import workloads as wl


def test_relu_literal_loop_and_library_maximum():
    g = np.random.default_rng(0)
    H = g.standard_normal((9, 7)).astype(np.float32)
    H[2, 3] = 0.0
    R = orc.relu(H)
    for i in range(9):
        for j in range(7):
            assert R[i, j] == (H[i, j] if H[i, j] > 0 else 0.0)
    assert np.array_equal(R, np.maximum(H, 0))                 # finite values: the library routine
    h16 = H.astype(np.float16)
    assert np.array_equal(orc.relu(h16), np.maximum(h16, 0)) and orc.relu(h16).dtype == np.float16


def test_relu_special_values_bit_for_bit():
    # bf16 bit patterns: input -> expected output
    table = [
        (0x0000, 0x0000), (0x8000, 0x0000),      # both zeros give +0
        (0x3F80, 0x3F80), (0xBF80, 0x0000),      # +1, -1
        (0x7F80, 0x7F80), (0xFF80, 0x0000),      # +Inf stays, -Inf is clamped
        (0x7FC0, 0x7FC0), (0xFFC0, 0xFFC0),      # NaN of either sign is passed through unchanged
        (0x0001, 0x0001), (0x8001, 0x0000),      # subnormals
        (0x7F7F, 0x7F7F), (0xFF7F, 0x0000),      # largest finite magnitudes
    ]
    src = np.array([[a for a, _ in table]], dtype=np.uint16)
    want = np.array([[b for _, b in table]], dtype=np.uint16)
    got = orc.relu(src)
    assert got.dtype == np.uint16 and np.array_equal(got, want)
    f = np.array([[-0.0, np.nan, -np.inf, np.inf, -1e-45]], dtype=np.float32)
    r = orc.relu(f)
    assert not np.signbit(r[0, 0]) and np.isnan(r[0, 1]) and r[0, 2] == 0 and not np.signbit(r[0, 2])
    assert r[0, 3] == np.inf and r[0, 4] == 0 and not np.signbit(r[0, 4])


def test_channel_major_output_and_index_by_brute_force():
    g = np.random.default_rng(1)
    T, K, mt = 12, 10, 4
    Hf = g.standard_normal((T, K)).astype(np.float32) - 1.0       # mostly negative: a sparse activation
    Hf[:, 3] = -1.0                                               # a channel that is dead everywhere
    Hf[4:8, 5] = -2.0                                             # and one dead in a single token block
    Hf[5, 5] = np.nan                                             # ... except for a NaN, which stays visible
    H = wl.to_bf16_bits(Hf)
    Xt, sp, idx = orc.relu_channel_major(H, mt)
    assert Xt.shape == (K, T) and Xt.dtype == np.uint16
    vals = orc.bf16_bits_to_f64(H)
    for k in range(K):
        for t in range(T):
            x = vals[t, k]
            want = x if (x > 0 or np.isnan(x)) else 0.0
            got = orc.bf16_bits_to_f64(Xt[k:k + 1, t:t + 1])[0, 0]
            assert (np.isnan(want) and np.isnan(got)) or want == got
    lists = []
    for s in range(T // mt):
        live = []
        for k in range(K):
            blk = vals[s * mt:(s + 1) * mt, k]
            if any((x > 0) or np.isnan(x) for x in blk):
                live.append(k)
        lists.append(live)
    assert sp.tolist() == np.cumsum([0] + [len(l) for l in lists]).tolist()
    assert idx.tolist() == [k for l in lists for k in l]
    assert 3 not in idx.tolist() and 5 in lists[1]


def test_product_through_the_fused_producer_equals_the_plain_product():
    g = np.random.default_rng(2)
    T, K, N = 16, 24, 5
    H = wl.to_bf16_bits(g.integers(-3, 3, size=(T, K)).astype(np.float32))
    W = wl.to_bf16_bits(g.integers(-2, 3, size=(K, N)).astype(np.float32))
    Xt, sp, idx = orc.relu_channel_major(H, 8)
    want = np.maximum(orc.to_f64(H), 0) @ orc.to_f64(W)
    assert np.array_equal(orc.gemm_at(Xt, W), want)
    # the listed micro-tiles alone carry the product (storage order of Xt: rows = channels)
    assert np.array_equal(orc.gemm_over_index(np.ascontiguousarray(Xt.T), W, *_as_row_index(sp, idx, T, K, 8)), want)


def _as_row_index(sp, idx, T, K, mt):
    """The index of Xt (segments = token blocks, coordinates = channels) read as an index of X = Xt^T
    with micro-tiles of mt tokens x 1 channel and the column (channel) as PIT coordinate."""
    return sp, idx, mt, 1, 1
