"""pit_build_index_static (the entry point for callers that cannot allocate) against pit_build_index:
bit-identical indices through the C ABI, two calls in a row, the second on a smaller input."""
import numpy as np
import pytest
import torch

from paper_2301_10936_amd import pit, workloads as wl
from tests.gpu_util import to_dev

pytestmark = pytest.mark.gpu


def _both(src, mt_rows, mt_cols, pit_dim, want_bits=False):
    rows, cols = src.shape
    gr, gc = rows // mt_rows, cols // mt_cols
    ref = pit.pit_build_index(src, mt_rows, mt_cols, pit_dim, want_bits=want_bits)
    out = pit.PitIndex.empty(gc if pit_dim == 0 else gr, gr * gc, want_bits, src.device)
    out.idx.fill_(-7)
    pit.pit_build_index_static(src, mt_rows, mt_cols, pit_dim, out)
    torch.cuda.synchronize()
    a, b = ref.to_host(), out.to_host()
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    if want_bits:
        assert np.array_equal(a[2], b[2])
    return int(a[0][-1])


def test_static_workspace_matches_caller_workspace_two_calls_second_smaller():
    big = to_dev(wl.relu_ffn(M=1024, K=2048, N=8, seed=5, channel_live_prob=0.4).Xt)      # [2048 ch, 1024 tok]
    small = to_dev(wl.relu_ffn(M=256, K=384, N=8, seed=6, channel_live_prob=0.2).Xt)      # [384 ch, 256 tok]
    n_big = _both(big, 1, 128, 0)
    n_small = _both(small, 1, 128, 0)
    assert n_big > n_small > 0
    # again the large one (the array now holds the small call's words), then other kernel paths of the build
    assert _both(big, 1, 128, 0) == n_big
    mask = to_dev(wl.sparse_attn(H=1, S=512, D=8, seed=3).mask)
    _both(mask, 32, 1, 1, want_bits=True)
    _both(mask[:256, :256].contiguous(), 32, 1, 1, want_bits=True)
    blocks = to_dev(wl.iid_block_mask(512, 1024, 8, 1, 0.9, seed=2))
    _both(blocks, 32, 1, 0)            # shared bitmap units: the build clears the words itself
    _both(blocks[:128, :64].contiguous(), 32, 1, 0)
    rowmask = to_dev(wl.padded_linear(batch=4, max_len=64, hidden=8, out=8, seed=1).row_mask.reshape(-1, 1))
    _both(rowmask, 1, 1, 0)


def test_static_workspace_rejects_what_does_not_fit():
    lib, CIndex = pit.raw()
    cap = pit.pit_build_index_static_capacity()
    assert cap == 1 << 20
    assert pit.pit_build_index_workspace(4096, 4096, 1, 1, 0) > cap
    mask = torch.ones((4096, 4096), dtype=torch.uint8, device="cuda")
    out = pit.PitIndex.empty(4096, 4096 * 4096, False, mask.device)
    out.seg_ptr.fill_(-3)
    with pytest.raises(pit.PitError) as e:
        pit.pit_build_index_static(mask, 1, 1, 0, out)
    assert e.value.code == pit.PIT_ECAPACITY
    torch.cuda.synchronize()
    assert int(out.seg_ptr[0].item()) == -3          # nothing was enqueued
    # argument errors as in pit_build_index
    with pytest.raises(pit.PitError) as e:
        pit.pit_build_index_static(mask[:100, :96], 1, 64, 0, out)
    assert e.value.code in (pit.PIT_ESHAPE, pit.PIT_EINVAL)
