"""GPU parity: pit_sparse_attn vs the fp64 masked-softmax oracle."""
import numpy as np
import pytest
import torch

from oracle import pit_oracle as orc
from paper_2301_10936_amd import workloads as wl
from tests.gpu_util import assert_close, bf16_bits, dev, to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pit():
    from paper_2301_10936_amd import pit as p
    return p


def _run(pit, w, mask=None, o_dtype=torch.float32, sentinel=None):
    mask = w.mask if mask is None else mask
    out = None
    if sentinel is not None:
        out = torch.full(w.Q.shape, sentinel, dtype=o_dtype, device=dev())
    O = pit.pit_sparse_attn(to_dev(w.Q), to_dev(w.K), to_dev(w.V), to_dev(mask), w.scale, out=out, o_dtype=o_dtype)
    torch.cuda.synchronize()
    return O


@pytest.mark.parametrize("H,S,window,density", [(1, 32, 8, 0.2), (2, 64, 16, 0.1), (3, 160, 32, 0.3), (2, 512, 64, 0.05), (1, 1024, 256, 0.05)])
def test_against_oracle(pit, H, S, window, density):
    w = wl.sparse_attn(H=H, S=S, window=window, density=density, seed=S + H)
    O = _run(pit, w, sentinel=9.0)
    assert_close(O, orc.sparse_attn(w.Q, w.K, w.V, w.mask, w.scale), "sparse_attn")


def test_full_mask_is_dense_attention(pit):
    w = wl.sparse_attn(H=2, S=256, seed=3)
    full = np.ones((256, 256), dtype=np.uint8)
    O = _run(pit, w, mask=full)
    assert_close(O, orc.sparse_attn(w.Q, w.K, w.V, full, w.scale), "full mask")


def test_element_mask_inside_kept_microtiles(pit):
    """A key column kept for a single query of a block must not leak to the block's other 31 queries."""
    w = wl.sparse_attn(H=1, S=128, window=2, density=0.0, seed=4)
    m = w.mask.copy()
    m[5, 100] = 1
    m[40, 3] = 1
    m[70, :] = 0            # a query with no key at all
    O = _run(pit, w, mask=m, sentinel=4.0)
    ref = orc.sparse_attn(w.Q, w.K, w.V, m, w.scale)
    assert_close(O, ref, "element mask")
    assert torch.count_nonzero(O[0, 70]) == 0


def test_single_key_per_query_copies_value_rows(pit):
    w = wl.sparse_attn(H=2, S=96, seed=5)
    m = np.zeros((96, 96), dtype=np.uint8)
    tgt = (np.arange(96) * 7) % 96
    m[np.arange(96), tgt] = 1
    O = _run(pit, w, mask=m).cpu().numpy()
    V = orc.to_f64(w.V)
    assert np.array_equal(O, V[:, tgt])     # P = 1 exactly and bf16 V enters the product unchanged


def test_all_masked_gives_zeros(pit):
    w = wl.sparse_attn(H=1, S=64, seed=6)
    O = _run(pit, w, mask=np.zeros((64, 64), dtype=np.uint8), sentinel=2.0)
    assert torch.count_nonzero(O) == 0


def test_fp16_inputs_and_rounded_outputs(pit):
    w = wl.sparse_attn(H=2, S=256, window=32, density=0.1, seed=7)
    Q, K, V = (orc.bf16_bits_to_f64(x).astype(np.float16) for x in (w.Q, w.K, w.V))
    ref = orc.sparse_attn(Q, K, V, w.mask, w.scale)
    O = pit.pit_sparse_attn(to_dev(Q), to_dev(K), to_dev(V), to_dev(w.mask), w.scale)
    Oh = pit.pit_sparse_attn(to_dev(Q), to_dev(K), to_dev(V), to_dev(w.mask), w.scale, o_dtype=torch.float16)
    torch.cuda.synchronize()
    assert_close(O, ref, "fp16 attn")
    mx, fro = orc.rel_errors(Oh.float().cpu().numpy(), ref)
    assert fro < 1e-3 and mx < 2e-2
    wb = wl.sparse_attn(H=1, S=128, window=32, density=0.1, seed=8)
    Ob = _run(pit, wb, o_dtype=torch.bfloat16)
    mx, fro = orc.rel_errors(orc.bf16_bits_to_f64(bf16_bits(Ob)), orc.sparse_attn(wb.Q, wb.K, wb.V, wb.mask, wb.scale))
    assert fro < 3e-3   # bf16 storage costs ~1.7e-3 by itself


def test_c5_full_size(pit):
    w = wl.sparse_attn()
    O = _run(pit, w, sentinel=9.0)
    assert_close(O, orc.sparse_attn(w.Q, w.K, w.V, w.mask, w.scale), "C5 full size")


def test_attn_error_returns(pit):
    w = wl.sparse_attn(H=1, S=64, D=32, seed=1)
    with pytest.raises(pit.PitError) as e:
        _run(pit, w)
    assert e.value.code == pit.PIT_ESHAPE
    assert pit.pit_sparse_attn_workspace(1, 40, 64) == 0


def test_values_far_outside_the_fp16_range(pit):
    """bf16 V rows of magnitude 1e5 (beyond fp16's largest finite value) and 1e-9 (below its smallest
    subnormal) must come through: V enters the second product as bf16, not through a narrower type."""
    w = wl.sparse_attn(H=3, S=256, window=32, density=0.1, seed=21)
    V = orc.bf16_bits_to_f64(w.V)
    V[0] *= 1e5
    V[1] *= 1e-9
    V[2, ::2] *= 1e5          # both magnitudes among the keys of one query
    V[2, 1::2] *= 1e-9
    w.V = wl.to_bf16_bits(V.astype(np.float32))
    O = _run(pit, w, sentinel=3.0)
    assert bool(torch.isfinite(O).all())
    ref = orc.sparse_attn(w.Q, w.K, w.V, w.mask, w.scale)
    assert float(np.abs(ref[0]).max()) > 65504.0 and 0.0 < float(np.abs(ref[1]).max()) < 2.0 ** -24
    for h in range(3):
        assert_close(O[h], ref[h], f"head {h}")
    # a query that sees only tiny values: single-key mask over the 1e-9 rows of head 2 copies them exactly
    m = np.zeros((256, 256), dtype=np.uint8)
    m[np.arange(256), 1] = 1
    O1 = _run(pit, w, mask=m).cpu().numpy()
    Vq = orc.to_f64(w.V)
    assert np.array_equal(O1[2], np.broadcast_to(Vq[2, 1], (256, 64))) and np.all(O1[2, 0] != 0)


def test_key_lists_longer_than_one_pass_of_the_index_kernel(pit):
    # S = 4256: the one-launch index of the mask walks the keys in passes of 4096, so the lists of a
    # query block continue in a second pass whose last threads lie beyond the row
    w = wl.sparse_attn(H=1, S=4256, window=64, density=0.02, seed=31)
    O = _run(pit, w, sentinel=9.0)
    assert_close(O, orc.sparse_attn(w.Q, w.K, w.V, w.mask, w.scale), "sparse_attn S=4256")


def test_mask_at_an_odd_address_takes_the_general_index_build(pit):
    # a mask whose rows cannot be read 16 bytes at a time goes through pit_build_index instead of the
    # one-launch index; both must give the same attention
    w = wl.sparse_attn(H=2, S=160, window=32, density=0.2, seed=32)
    S = 160
    buf = torch.zeros(S * S + 16, dtype=torch.uint8, device=dev())
    odd = buf[3:3 + S * S].view(S, S)
    odd.copy_(to_dev(w.mask))
    assert odd.data_ptr() % 16 != 0
    Q, K, V = to_dev(w.Q), to_dev(w.K), to_dev(w.V)
    O_odd = pit.pit_sparse_attn(Q, K, V, odd, w.scale)
    O_al = pit.pit_sparse_attn(Q, K, V, to_dev(w.mask), w.scale)
    torch.cuda.synchronize()
    assert_close(O_odd, orc.sparse_attn(w.Q, w.K, w.V, w.mask, w.scale), "sparse_attn, mask at an odd address")
    assert torch.equal(O_odd, O_al)
