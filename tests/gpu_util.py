"""Helpers for the GPU parity tests: move seeded numpy inputs to the device and back."""
import numpy as np
import torch

MAX_REL_TOL = 2e-2     # max |got-ref| / max(|ref|, rms(ref))
FRO_TOL = 1e-3         # ||got-ref||_F / ||ref||_F


def dev():
    return torch.device("cuda:0")


def to_dev(a: np.ndarray) -> torch.Tensor:
    """uint16 arrays are bf16 bit patterns; everything else maps to the same torch dtype."""
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16).copy()).view(torch.bfloat16).to(dev())
    return torch.from_numpy(np.ascontiguousarray(a)).to(dev())


def bf16_bits(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().view(torch.int16).numpy().view(np.uint16)


def assert_index_equal(ix, ref):
    sp, idx, bits = ix.to_host()
    rsp, ridx, rbits = ref
    assert np.array_equal(sp, rsp), "seg_ptr differs"
    assert np.array_equal(idx, ridx), "idx differs"
    if ix.bits is not None:
        assert np.array_equal(bits, rbits), "bits differ"


def assert_close(got: torch.Tensor, ref: np.ndarray, what=""):
    from oracle import pit_oracle as orc
    g = got.detach().float().cpu().numpy() if got.dtype != torch.float32 else got.detach().cpu().numpy()
    mx, fro = orc.rel_errors(g, ref)
    assert mx <= MAX_REL_TOL and fro <= FRO_TOL, f"{what}: max_rel={mx:.3e} fro={fro:.3e}"
    return mx, fro
