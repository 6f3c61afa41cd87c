"""GPU parity: online sparsity detection (pit_build_index, pit_build_route_index) vs the oracle, bit for bit."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import pit_oracle as orc
from paper_2301_10936_amd import workloads as wl
from tests.gpu_util import assert_index_equal, dev, to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pit():
    from paper_2301_10936_amd import pit as p
    return p


def _check(pit, src_np, mt_rows, mt_cols, pit_dim, want_bits=False, src_t=None):
    t = to_dev(src_np) if src_t is None else src_t
    ix = pit.pit_build_index(t, mt_rows, mt_cols, pit_dim, want_bits=want_bits)
    torch.cuda.synchronize()
    assert_index_equal(ix, orc.build_index(src_np, mt_rows, mt_cols, pit_dim))
    return ix


def test_c1_fp16_1x32_full_size(pit):
    w = wl.microtile_gemm()
    ix = _check(pit, w.A, 1, 32, 0)
    assert int(ix.seg_ptr[-1]) == int(w.keep.sum())


@pytest.mark.parametrize("mt", [32, 128])
def test_c2_relu_bf16_full_size(pit, mt):
    w = wl.relu_ffn()
    _check(pit, w.Xt, 1, mt, 0)


def test_c2_correlated_zeros(pit):
    w = wl.relu_ffn(M=1024, K=2048, N=8, channel_live_prob=0.25, seed=5)
    _check(pit, w.Xt, 1, 128, 0)
    _check(pit, w.Xt, 1, 32, 0, want_bits=True)   # bits force the generic pass


def test_c4_row_mask_full_size(pit):
    w = wl.padded_linear(hidden=8, out=8)
    m = w.row_mask.reshape(-1, 1)
    ix = _check(pit, m, 1, 1, 0)
    assert int(ix.seg_ptr[-1]) == int(w.lengths.sum())


@pytest.mark.parametrize("rows", [1, 15, 16, 17, 1000, 1024, 16384, 40000, 65536, 65537, 100000])
@pytest.mark.parametrize("density", [0.0, 0.5, 1.0])
def test_row_mask_of_any_length(pit, rows, density):
    """A byte mask over rows (one column): up to 65536 rows one launch builds the whole index, longer
    masks take the two passes; contiguous and strided masks, any non-zero byte counts."""
    g = np.random.default_rng(rows + int(density * 10))
    mask = (g.random(rows) < density).astype(np.uint8) * g.integers(1, 256, size=rows).astype(np.uint8)
    want = orc.build_index(mask.reshape(-1, 1), 1, 1, 0)
    assert_index_equal(pit.pit_build_index(to_dev(mask.reshape(-1, 1)), 1, 1, 0), want)
    wide = torch.zeros((rows, 3), dtype=torch.uint8, device=dev())
    wide[:, 1] = to_dev(mask)
    assert_index_equal(pit.pit_build_index(wide[:, 1:2], 1, 1, 0), want)      # stride 3 between rows
    if rows > 1:
        off = to_dev(np.concatenate([np.zeros(1, np.uint8), mask]))[1:].reshape(-1, 1)   # not 16-byte aligned
        assert_index_equal(pit.pit_build_index(off, 1, 1, 0), want)


def test_c5_attention_mask_full_size_with_bits(pit):
    w = wl.sparse_attn(H=1, D=8)
    _check(pit, w.mask, 32, 1, 1, want_bits=True)
    _check(pit, w.mask, 32, 1, 1, want_bits=False)


@pytest.mark.parametrize("shape,mt,pit_dim,dtype", [
    ((96, 160), (1, 32), 0, np.float16),      # ragged: 96 rows (1.5 words), 320-byte rows
    ((200, 96), (1, 8), 0, np.float16),       # 16-byte micro-tiles
    ((130, 1024), (1, 512), 0, np.float16),   # 1 KiB micro-tiles
    ((77, 64), (1, 64), 0, np.float32),       # fp32 256-byte micro-tiles
    ((64, 48), (2, 2), 0, np.float32),        # generic
    ((64, 48), (2, 2), 1, np.float32),
    ((48, 80), (16, 16), 1, np.float16),
    ((33, 7), (1, 1), 0, np.float32),
    ((33, 7), (1, 1), 1, np.float32),
    ((96, 208), (32, 1), 1, np.uint8),        # column fast path, ragged chunk
    ((80, 2064), (16, 1), 1, np.uint8),       # > 2 chunks, mt_rows 16
    ((120, 64), (40, 1), 1, np.uint8),        # mt_rows > 32: flags only
    ((64, 100), (32, 1), 1, np.uint8),        # cols % 16 != 0 -> generic
    ((4, 8), (4, 8), 0, np.float16),          # a single micro-tile
])
def test_shapes_and_paths(pit, shape, mt, pit_dim, dtype):
    g = np.random.default_rng(hash((shape, mt, pit_dim)) % 2**32)
    src = ((g.random(shape) < 0.06) * (1 + g.random(shape))).astype(dtype)
    want_bits = mt[0] * mt[1] <= 32
    _check(pit, src, mt[0], mt[1], pit_dim, want_bits=want_bits)
    _check(pit, src, mt[0], mt[1], pit_dim, want_bits=False)


def _tile_cases():
    out = []
    for dtype, es in ((np.uint8, 1), (np.float16, 2), (np.float32, 4)):
        for mt_bytes in (1, 2, 4, 8, 16, 32, 64, 256, 1024):
            if mt_bytes < es:
                continue
            mt_cols = mt_bytes // es
            for mt_rows in (1, 2, 3, 16, 24, 64, 80):
                # rows: several 64-row blocks with a ragged tail; row bytes: two strips and a ragged third
                rows = mt_rows * max(1, 200 // mt_rows)
                row_bytes = max(mt_bytes, 16) * max(1, 2064 // max(mt_bytes, 16))
                if mt_bytes == 1024:
                    row_bytes = 3072
                out.append((rows, row_bytes // es, mt_rows, mt_cols, dtype))
    return out


@pytest.mark.parametrize("rows,cols,mt_rows,mt_cols,dtype", _tile_cases())
def test_vector_path_for_any_micro_tile(pit, rows, cols, mt_rows, mt_cols, dtype):
    """Power-of-two micro-tile widths from one byte to 1 KiB, heights that divide, straddle and exceed the
    64-row block of a workgroup, both PIT dimensions."""
    g = np.random.default_rng(rows * 7919 + cols * 31 + mt_rows)
    src = ((g.random((rows, cols)) < 0.02) * (1 + g.random((rows, cols)))).astype(dtype)
    if dtype != np.uint8:
        src[g.random((rows, cols)) < 0.01] = -0.0       # negative zero is zero
    _check(pit, src, mt_rows, mt_cols, 0)
    _check(pit, src, mt_rows, mt_cols, 1)


def test_vector_path_dense_and_strided(pit):
    g = np.random.default_rng(11)
    full = (1 + g.random((192, 1088))).astype(np.float16)
    for mt in ((1, 1), (2, 4), (32, 8), (48, 64)):
        _check(pit, full, mt[0], mt[1], 0)
        _check(pit, full, mt[0], mt[1], 1)
    big = np.zeros((130, 4096), dtype=np.uint8)
    sub = big[:, 1024:3104]                    # ld = 4096, 2080 columns, 16-byte aligned start
    sub[g.integers(0, 130, 300), g.integers(0, 2080, 300)] = 7
    t = to_dev(big)[:, 1024:3104]
    for mt in ((1, 1), (2, 2), (10, 16), (26, 32), (130, 4)):
        _check(pit, np.ascontiguousarray(sub), mt[0], mt[1], 0, src_t=t)
        _check(pit, np.ascontiguousarray(sub), mt[0], mt[1], 1, src_t=t)


@pytest.mark.parametrize("seed", range(48))
def test_random_shapes_either_path(pit, seed):
    """Seeded random shapes, micro-tiles, element sizes and densities: whichever bitmap and emit kernels the
    library picks, the index must equal the oracle's."""
    g = np.random.default_rng(9000 + seed)
    dtype = [np.uint8, np.float16, np.float32][seed % 3]
    mt_rows = int(g.choice([1, 1, 2, 3, 4, 5, 7, 8, 16, 17, 32, 33, 64, 65, 100]))
    mt_cols = int(g.choice([1, 1, 2, 4, 8, 16, 32, 64, 128, 3, 5, 24]))
    rows = mt_rows * int(g.integers(1, 10 if mt_rows > 8 else 300))
    cols = mt_cols * int(g.integers(1, 12 if mt_cols > 8 else 700))
    density = float(g.choice([0.0, 0.003, 0.05, 0.5, 1.0]))
    src = ((g.random((rows, cols)) < density) * (1 + g.random((rows, cols)))).astype(dtype)
    for pit_dim in (0, 1):
        _check(pit, src, mt_rows, mt_cols, pit_dim)


def test_strided_view_and_special_values(pit):
    g = np.random.default_rng(3)
    big = np.zeros((64, 256), dtype=np.float16)
    sub = big[:, 64:192]                      # ld = 256, cols = 128
    sub[g.integers(0, 64, 40), g.integers(0, 128, 40)] = 1
    sub[5, 0] = -0.0
    sub[6, 32] = np.nan
    sub[7, 64] = np.inf
    sub[8, 96] = np.float16(6e-8)             # subnormal
    t = to_dev(big)[:, 64:192]
    _check(pit, np.ascontiguousarray(sub), 1, 32, 0, src_t=t)
    _check(pit, np.ascontiguousarray(sub), 1, 32, 1, want_bits=True, src_t=t)
    b = np.array([[0x8000, 0x7FC0, 0x7F80, 0x0001, 0x0000, 0xBF80, 0, 0]] * 3, dtype=np.uint16)
    _check(pit, b, 1, 1, 1, want_bits=True)
    _check(pit, b, 1, 8, 0)


def test_all_zero_all_full_and_empty(pit):
    z = np.zeros((128, 128), dtype=np.float16)
    ix = _check(pit, z, 1, 32, 0)
    assert int(ix.seg_ptr[-1]) == 0
    f = np.ones((128, 128), dtype=np.float16)
    _check(pit, f, 1, 32, 0)
    _check(pit, f.astype(np.uint8), 32, 1, 1, want_bits=True)
    e = torch.empty((0, 64), dtype=torch.float16, device=dev())
    ix = pit.pit_build_index(e, 1, 32, 0)
    torch.cuda.synchronize()
    assert ix.seg_ptr.cpu().tolist() == [0, 0, 0]


def test_many_segments_path(pit):
    """1x1 granularity on 4096 x 4096 (Section 5.4's shape): 4096 segments, separate count pass."""
    m = wl.iid_block_mask(4096, 4096, 1, 1, 0.95, seed=1)
    _check(pit, m, 1, 1, 0)
    _check(pit, m, 1, 1, 1)
    m32 = wl.iid_block_mask(4096, 4096, 32, 32, 0.9, seed=2)
    _check(pit, m32, 32, 32, 1)
    _check(pit, m32, 32, 32, 0)
    _check(pit, m32, 16, 16, 0)
    h = (wl.iid_block_mask(4096, 4096, 32, 64, 0.9, seed=3) * 1.5).astype(np.float16)
    _check(pit, h, 32, 64, 0)
    _check(pit, h, 32, 64, 1)
    _check(pit, h, 1, 1, 1)


def test_repeatable(pit):
    w = wl.relu_ffn(M=512, K=1024, N=8, seed=9)
    t = to_dev(w.Xt)
    a = pit.pit_build_index(t, 1, 32, 0)
    b = pit.pit_build_index(t, 1, 32, 0)
    torch.cuda.synchronize()
    assert torch.equal(a.seg_ptr, b.seg_ptr)
    n = int(a.seg_ptr[-1])
    assert torch.equal(a.idx[:n], b.idx[:n])


# up to 8192 tokens and 64 experts the index is built by one workgroup in one launch; beyond, by the bitmap
# pass and the ordered emit: (8192, 64) and (200, 64) are the largest and a small case of the first path,
# (8200, 64), (9000, 16) and (300, 130) take the second
@pytest.mark.parametrize("T,E", [(4096, 64), (1000, 7), (63, 1), (300, 130), (1, 3), (8192, 64), (200, 64), (8200, 64), (9000, 16)])
def test_route_index(pit, T, E):
    w = wl.moe_ffn(T=T, d_model=8, d_ff=8, E=E, seed=T + E)
    eid = to_dev(w.expert_id)
    status = torch.full((1,), -7, dtype=torch.int32, device=dev())
    ix = pit.pit_build_route_index(eid, E, status=status)
    torch.cuda.synchronize()
    sp, idx, _ = ix.to_host()
    rsp, ridx = orc.route_index(w.expert_id, E)
    assert np.array_equal(sp, rsp) and np.array_equal(idx, ridx)
    assert int(status[0]) == 0


def test_route_index_invalid_ids_and_empty(pit):
    eid_np = np.array([0, 5, -1, 2, 2, 9, 1], dtype=np.int32)     # E = 3: 5, -1, 9 are invalid
    status = torch.zeros(1, dtype=torch.int32, device=dev())
    ix = pit.pit_build_route_index(to_dev(eid_np), 3, status=status)
    torch.cuda.synchronize()
    sp, idx, _ = ix.to_host()
    assert sp.tolist() == [0, 1, 2, 4] and idx.tolist() == [0, 6, 3, 4] and int(status[0]) == 3
    ix = pit.pit_build_route_index(torch.empty(0, dtype=torch.int32, device=dev()), 4, status=status)
    torch.cuda.synchronize()
    assert ix.seg_ptr.cpu().tolist() == [0] * 5 and int(status[0]) == 0


@pytest.mark.parametrize("T,E", [(5000, 20), (9000, 20)])
def test_route_index_invalid_ids_on_both_paths(pit, T, E):
    rng = np.random.default_rng(T)
    eid_np = rng.integers(0, E, size=T).astype(np.int32)
    badpos = rng.choice(T, size=37, replace=False)
    eid_np[badpos] = rng.choice(np.array([-1, -5, E, E + 44, 64, 1 << 20], dtype=np.int32), size=37)
    status = torch.zeros(1, dtype=torch.int32, device=dev())
    ix = pit.pit_build_route_index(to_dev(eid_np), E, status=status)
    torch.cuda.synchronize()
    sp, idx, _ = ix.to_host()
    rsp, ridx = orc.route_index(eid_np, E)
    assert np.array_equal(sp, rsp) and np.array_equal(idx, ridx)
    assert int(status[0]) == 37


def test_error_returns(pit):
    lib, CIndex = pit.raw()
    t = torch.zeros((64, 64), dtype=torch.float16, device=dev())
    ws = torch.empty(1 << 16, dtype=torch.uint8, device=dev())
    ix = pit.PitIndex.empty(2, 64 * 2)
    def call(rows=64, cols=64, mt_r=1, mt_c=32, pd=0, dt=pit.PIT_F16, idx=ix, src=t.data_ptr(), wsb=ws.numel(), ld=64):
        ci = idx.c()
        return lib.pit_build_index(src, dt, rows, cols, ld, mt_r, mt_c, pd, ctypes.byref(ci), ws.data_ptr(), wsb, None)
    assert call() == pit.PIT_OK
    assert call(mt_c=24) == pit.PIT_ESHAPE
    assert call(pd=2) == pit.PIT_EINVAL
    assert call(dt=9) == pit.PIT_EINVAL
    assert call(src=None) == pit.PIT_EINVAL
    assert call(wsb=8) == pit.PIT_ECAPACITY
    assert call(idx=pit.PitIndex.empty(3, 128)) == pit.PIT_ECAPACITY       # wrong nseg
    assert call(idx=pit.PitIndex.empty(2, 100)) == pit.PIT_ECAPACITY       # cap below worst case
    assert call(ld=32) == pit.PIT_EINVAL
    with_bits = pit.PitIndex.empty(1, 64, want_bits=True)
    assert call(mt_c=64, idx=with_bits) == pit.PIT_EINVAL                  # bits need <= 32 elements
    torch.cuda.synchronize()


def test_check_index_counts_violations(pit):
    """pit_check_index: zero on what the library builds, and every planted fault of a hand-made index counted."""
    w = wl.relu_ffn(M=256, K=300, N=8, seed=2, channel_live_prob=0.3)
    ix = pit.pit_build_index(to_dev(w.Xt), 1, 128, 0)
    assert int(pit.pit_check_index(ix, 300).item()) == 0
    assert int(pit.pit_check_index(ix, 10).item()) > 0                      # the same lists against a shorter axis
    sp = torch.tensor([0, 3, 3, 6], dtype=torch.int32, device="cuda")
    idx = torch.tensor([1, 5, 9, 0, 2, 4, 0, 0], dtype=torch.int32, device="cuda")
    good = pit.PitIndex(sp, idx, None, 3, 8)
    assert int(pit.pit_check_index(good, 10).item()) == 0
    idx2 = idx.clone(); idx2[2] = 10                                        # out of range (last of its segment)
    assert int(pit.pit_check_index(pit.PitIndex(sp, idx2, None, 3, 8), 10).item()) == 1
    idx3 = idx.clone(); idx3[4] = 0                                         # not above its predecessor (0 after 0)
    assert int(pit.pit_check_index(pit.PitIndex(sp, idx3, None, 3, 8), 10).item()) == 1
    idx4 = idx.clone(); idx4[0] = -1; idx4[5] = 2                           # negative; equal to its predecessor
    assert int(pit.pit_check_index(pit.PitIndex(sp, idx4, None, 3, 8), 10).item()) == 2
    sp2 = torch.tensor([0, 4, 3, 6], dtype=torch.int32, device="cuda")      # segment 1 ends before it starts
    assert int(pit.pit_check_index(pit.PitIndex(sp2, idx, None, 3, 8), 10).item()) >= 1
    sp3 = torch.tensor([0, 3, 3, 9], dtype=torch.int32, device="cuda")      # beyond the capacity
    assert int(pit.pit_check_index(pit.PitIndex(sp3, idx, None, 3, 8), 10).item()) == 1
    torch.cuda.synchronize()
