"""The erf approximation of the GELU epilogue (paper_2301_10936_amd/csrc/pit_gemm_dev.hpp, gelu_erf_fast), evaluated
here in numpy float32 with the constants of the kernel, against scipy's erf: the bound the kernel's comment states."""
import numpy as np
from scipy.special import erf

C = np.array([1.6278890371, 0.9185093641, 0.1486656219, -0.02959003858, 0.00294415676], dtype=np.float32)


def gelu_kernel_formula(x):
    x = x.astype(np.float32)
    z = np.abs(x) * np.float32(0.70710678118654752)
    with np.errstate(over="ignore", invalid="ignore"):
        acc = np.full_like(z, C[4])
        for k in (3, 2, 1, 0):
            acc = acc * z + C[k]
        q = acc * z
        p = np.exp2(-q.astype(np.float64))
    p[p < 2.0 ** -126] = 0.0                    # the hardware exp2 flushes denormal results to zero
    e = np.float32(1) - p.astype(np.float32)
    return e, np.float32(0.5) * x * (np.float32(1) + np.copysign(e, x))


def test_erf_error_bound_and_tails():
    x = np.linspace(-40.0, 40.0, 2000001)
    e, g = gelu_kernel_formula(x)
    exact_erf = erf(np.abs(x) / np.sqrt(2.0))
    assert np.abs(e - exact_erf).max() <= 7e-7
    exact = 0.5 * x * (1.0 + erf(x / np.sqrt(2.0)))
    assert np.abs(g - exact).max() <= 3e-6
    # far tails: exactly x for large positive, exactly (minus) zero for large negative arguments
    _, t = gelu_kernel_formula(np.array([1e3, 1e6, -9.0, -50.0, -1e4, -1e30]))
    assert t[0] == np.float32(1e3) and t[1] == np.float32(1e6) and np.all(t[2:] == 0.0)
    _, n = gelu_kernel_formula(np.array([np.nan]))
    assert np.isnan(n[0])
