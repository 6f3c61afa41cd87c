"""GPU parity: pit_relu_channel_major_index (ReLU + layout change + detection in one pass) vs the oracle, bit for bit."""
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


def _pre_activation(g, tokens, channels, dead=0.3, shift=1.2):
    """N(-shift, 1) values; a share of the channels is dead (negative) in whole 128-token blocks."""
    H = g.standard_normal((tokens, channels)).astype(np.float32) - np.float32(shift)
    blocks = tokens // 128
    kill = g.random((blocks, channels)) < dead
    H = np.where(np.repeat(kill, 128, axis=0), -np.abs(H) - 0.5, H)
    return H.astype(np.float32)


def _check(pit, H_np, H_t=None):
    H_t = to_dev(H_np) if H_t is None else H_t
    Xt, ix = pit.pit_relu_channel_major_index(H_t)
    torch.cuda.synchronize()
    want_xt, sp, idx = orc.relu_channel_major(H_np, 128)
    got = Xt.view(torch.int16).cpu().numpy().view(np.uint16)
    assert np.array_equal(got, want_xt.view(np.uint16))
    assert_index_equal(ix, (sp, idx, None))
    return Xt, ix


@pytest.mark.parametrize("tokens,channels", [(128, 128), (256, 8), (384, 200), (128, 1000), (640, 328), (2048, 8192)])
def test_bf16_shapes(pit, tokens, channels):
    g = np.random.default_rng(tokens + channels)
    _check(pit, wl.to_bf16_bits(_pre_activation(g, tokens, channels)))


def test_fp16_and_special_values(pit):
    g = np.random.default_rng(5)
    H = _pre_activation(g, 256, 72).astype(np.float16)
    H[0, 0] = -0.0
    H[1, 1] = np.nan
    H[2, 2] = -np.inf
    H[3, 3] = np.inf
    H[4, 4] = np.float16(-6e-8)
    H[5, 5] = np.float16(6e-8)
    H[128:, 7] = -1.0
    H[130, 7] = np.nan                      # a NaN keeps an otherwise dead channel listed
    _check(pit, H)
    b = wl.to_bf16_bits(_pre_activation(g, 128, 16))
    b[0, :12] = [0x0000, 0x8000, 0x3F80, 0xBF80, 0x7F80, 0xFF80, 0x7FC0, 0xFFC0, 0x0001, 0x8001, 0x7F7F, 0xFF7F]
    _check(pit, b)


def test_strided_views_all_dead_and_all_live(pit):
    g = np.random.default_rng(6)
    big = wl.to_bf16_bits(_pre_activation(g, 256, 512))
    sub = np.ascontiguousarray(big[:, 128:328])                   # ld = 512, 200 channels, 16-byte aligned start
    t = to_dev(big)[:, 128:328]
    out_big = torch.full((200, 384), -1, dtype=torch.int16, device=dev()).view(torch.bfloat16)
    out_view = out_big[:, :256]
    ix = pit.PitIndex.empty(2, 2 * 200)
    pit.pit_relu_channel_major_index(t, out_xt=out_view, out=ix)
    torch.cuda.synchronize()
    want_xt, sp, idx = orc.relu_channel_major(sub, 128)
    assert np.array_equal(out_view.contiguous().view(torch.int16).cpu().numpy().view(np.uint16), want_xt)
    assert torch.all(out_big[:, 256:].view(torch.int16) == -1)     # nothing written beyond the token columns
    assert_index_equal(ix, (sp, idx, None))
    dead = wl.to_bf16_bits(-np.abs(_pre_activation(g, 256, 64)) - 1)
    _, ixd = _check(pit, dead)
    assert int(ixd.seg_ptr[-1]) == 0
    live = wl.to_bf16_bits(np.abs(_pre_activation(g, 256, 64)) + 1)
    _, ixl = _check(pit, live)
    assert int(ixl.seg_ptr[-1]) == 2 * 64


def test_feeds_the_gather_k_product(pit):
    """The fused producer followed by the GATHER_K product equals ReLU(H) . W of the oracle."""
    g = np.random.default_rng(7)
    tokens, channels, N = 256, 320, 128
    H = wl.to_bf16_bits(g.integers(-4, 3, size=(tokens, channels)).astype(np.float32))
    W = wl.to_bf16_bits(g.integers(-3, 4, size=(channels, N)).astype(np.float32))
    Xt, ix = pit.pit_relu_channel_major_index(to_dev(H))
    C = pit.pit_sread_gemm(pit.PIT_GEMM_GATHER_K, Xt, to_dev(W), ix, 128, tokens, N, channels)
    torch.cuda.synchronize()
    assert np.array_equal(C.cpu().numpy().astype(np.float64), np.maximum(orc.to_f64(H), 0) @ orc.to_f64(W))


def test_without_an_index_the_layout_change_is_the_same(pit):
    """index=False (out == NULL at the C ABI): the same Xt, bit for bit, and nothing else is written."""
    g = np.random.default_rng(77)
    H_np = wl.to_bf16_bits(_pre_activation(g, 384, 200))
    Xt, none = pit.pit_relu_channel_major_index(to_dev(H_np), index=False)
    torch.cuda.synchronize()
    assert none is None
    want_xt, _, _ = orc.relu_channel_major(H_np, 128)
    assert np.array_equal(Xt.view(torch.int16).cpu().numpy().view(np.uint16), want_xt.view(np.uint16))


def test_empty_and_error_returns(pit):
    lib, _ = pit.raw()
    e = torch.empty((0, 64), dtype=torch.bfloat16, device=dev())
    Xt, ix = pit.pit_relu_channel_major_index(e)
    torch.cuda.synchronize()
    assert ix.seg_ptr.cpu().tolist() == [0]
    H = torch.zeros((128, 64), dtype=torch.bfloat16, device=dev())
    Xo = torch.zeros((64, 128), dtype=torch.bfloat16, device=dev())
    ws = torch.empty(1 << 16, dtype=torch.uint8, device=dev())
    ix = pit.PitIndex.empty(1, 64)
    def call(tokens=128, channels=64, dt=pit.PIT_BF16, ldh=64, ldxt=128, idx=ix, src=H.data_ptr(), wsb=ws.numel()):
        ci = idx.c()
        return lib.pit_relu_channel_major_index(src, ldh, tokens, channels, dt, Xo.data_ptr(), ldxt, ctypes.byref(ci),
                                                ws.data_ptr(), wsb, None)
    assert call() == pit.PIT_OK
    assert call(tokens=100) == pit.PIT_ESHAPE
    assert call(channels=60) == pit.PIT_ESHAPE
    assert call(dt=pit.PIT_F32) == pit.PIT_EINVAL
    assert call(ldh=32) == pit.PIT_EINVAL
    assert call(ldxt=64) == pit.PIT_EINVAL
    assert call(src=None) == pit.PIT_EINVAL
    assert call(wsb=8) == pit.PIT_ECAPACITY
    assert call(idx=pit.PitIndex.empty(2, 128)) == pit.PIT_ECAPACITY
    assert call(idx=pit.PitIndex.empty(1, 10)) == pit.PIT_ECAPACITY
    assert call(idx=pit.PitIndex.empty(1, 64, want_bits=True)) == pit.PIT_EINVAL
    torch.cuda.synchronize()
