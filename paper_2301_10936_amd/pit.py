"""Thin ctypes binding of the C-ABI library declared in include/pit.h.

Argument marshalling only: every step of the hot path (index build, SRead gather, MFMA tiles,
SWrite scatter) runs inside libpit_hip.so.  PyTorch supplies device memory and the current stream.
Importing this module raises if the library has not been built -- there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpit_hip.so")
if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2301_10936_amd.build`")
_lib = ctypes.CDLL(LIB_PATH)

PIT_OK, PIT_EINVAL, PIT_ESHAPE, PIT_ECAPACITY, PIT_EHIP = 0, -1, -2, -3, -4
PIT_U8, PIT_F16, PIT_BF16, PIT_F32 = 0, 1, 2, 3
PIT_GEMM_GATHER_M, PIT_GEMM_GATHER_K, PIT_GEMM_DENSE_K = 0, 1, 2
_STATUS = {0: "PIT_OK", -1: "PIT_EINVAL", -2: "PIT_ESHAPE", -3: "PIT_ECAPACITY", -4: "PIT_EHIP"}

EXPORTS = ["pit_last_hip_error", "pit_version", "pit_build_index_workspace", "pit_build_index",
           "pit_build_index_static_capacity", "pit_build_index_static", "pit_check_index",
           "pit_build_route_index_workspace", "pit_build_route_index",
           "pit_relu_channel_major_index_workspace", "pit_relu_channel_major_index",
           "pit_cover_count_workspace", "pit_cover_count", "pit_select_kernel", "pit_sread_gemm",
           "pit_select_and_run_gemm_workspace", "pit_select_and_run_gemm",
           "pit_moe_workspace", "pit_moe_dispatch_gemm", "pit_sparse_attn_workspace", "pit_sparse_attn"]


class _CIndex(ctypes.Structure):
    _fields_ = [("seg_ptr", ctypes.c_void_p), ("idx", ctypes.c_void_p), ("bits", ctypes.c_void_p),
                ("nseg", ctypes.c_int32), ("cap", ctypes.c_int32)]


c_int, c_i64, c_vp, c_sz, c_f = ctypes.c_int, ctypes.c_int64, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_float
_P = ctypes.POINTER(_CIndex)
_lib.pit_last_hip_error.restype = c_int
_lib.pit_version.restype = c_int
_lib.pit_build_index_workspace.restype = c_sz
_lib.pit_build_index_workspace.argtypes = [c_int] * 6
_lib.pit_build_index.restype = c_int
_lib.pit_build_index.argtypes = [c_vp, c_int, c_int, c_int, c_i64, c_int, c_int, c_int, _P, c_vp, c_sz, c_vp]
_lib.pit_build_index_static_capacity.restype = c_sz
_lib.pit_build_index_static_capacity.argtypes = []
_lib.pit_build_index_static.restype = c_int
_lib.pit_build_index_static.argtypes = [c_vp, c_int, c_int, c_int, c_i64, c_int, c_int, c_int, _P, c_vp]
_lib.pit_check_index.restype = c_int
_lib.pit_check_index.argtypes = [_P, c_int, c_vp, c_vp]
_lib.pit_build_route_index_workspace.restype = c_sz
_lib.pit_build_route_index_workspace.argtypes = [c_int, c_int]
_lib.pit_build_route_index.restype = c_int
_lib.pit_build_route_index.argtypes = [c_vp, c_int, c_int, _P, c_vp, c_vp, c_sz, c_vp]
_lib.pit_relu_channel_major_index_workspace.restype = c_sz
_lib.pit_relu_channel_major_index_workspace.argtypes = [c_int, c_int]
_lib.pit_relu_channel_major_index.restype = c_int
_lib.pit_relu_channel_major_index.argtypes = [c_vp, c_i64, c_int, c_int, c_int, c_vp, c_i64, _P, c_vp, c_sz, c_vp]


class _CCandidate(ctypes.Structure):
    _fields_ = [("mt_rows", ctypes.c_int32), ("mt_cols", ctypes.c_int32), ("dense", ctypes.c_int32),
                ("tile_cost", ctypes.c_double), ("fixed_cost", ctypes.c_double)]


_lib.pit_cover_count_workspace.restype = c_sz
_lib.pit_cover_count_workspace.argtypes = [c_int] * 4
_lib.pit_cover_count.restype = c_int
_lib.pit_cover_count.argtypes = [c_vp, c_int, c_int, c_int, c_i64, c_int, c_int, c_vp, c_vp, c_sz, c_vp]
_lib.pit_select_kernel.restype = c_int
_lib.pit_select_kernel.argtypes = [ctypes.POINTER(_CCandidate), c_int, ctypes.POINTER(c_i64), ctypes.POINTER(c_i64),
                                   c_int, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(c_int)]
_lib.pit_sread_gemm.restype = c_int
_lib.pit_sread_gemm.argtypes = [c_int, c_vp, c_i64, c_vp, c_i64, c_vp, c_i64, c_int, c_int, c_int, c_int, c_int,
                                _P, c_int, c_int, c_vp]
_lib.pit_select_and_run_gemm_workspace.restype = c_sz
_lib.pit_select_and_run_gemm_workspace.argtypes = [c_int, c_int]
_lib.pit_select_and_run_gemm.restype = c_int
_lib.pit_select_and_run_gemm.argtypes = [ctypes.POINTER(_CCandidate), c_int, ctypes.POINTER(c_i64), ctypes.POINTER(c_i64), c_int,
                                         c_vp, c_i64, c_vp, c_i64, c_vp, c_i64, c_int, c_int, c_int, c_int, c_int,
                                         c_vp, c_sz, ctypes.POINTER(c_int), c_vp]
_lib.pit_moe_workspace.restype = c_sz
_lib.pit_moe_workspace.argtypes = [c_int] * 4
_lib.pit_moe_dispatch_gemm.restype = c_int
_lib.pit_moe_dispatch_gemm.argtypes = [c_vp, c_vp, c_vp, c_vp, c_vp, c_vp, c_int, c_int, c_int, c_int, c_int, c_int,
                                       c_int, c_vp, c_vp, c_sz, c_vp]
_lib.pit_sparse_attn_workspace.restype = c_sz
_lib.pit_sparse_attn_workspace.argtypes = [c_int] * 3
_lib.pit_sparse_attn.restype = c_int
_lib.pit_sparse_attn.argtypes = [c_vp, c_vp, c_vp, c_vp, c_vp, c_int, c_int, c_int, c_int, c_f, c_int,
                                 c_vp, c_sz, c_vp]


class PitError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        extra = f" (hip error {_lib.pit_last_hip_error()})" if code == PIT_EHIP else ""
        super().__init__(f"{where}: {_STATUS.get(code, code)}{extra}")


def _check(code: int, where: str) -> None:
    if code != PIT_OK:
        raise PitError(code, where)


def _dt(t: torch.Tensor) -> int:
    return {torch.uint8: PIT_U8, torch.bool: PIT_U8, torch.float16: PIT_F16, torch.bfloat16: PIT_BF16,
            torch.float32: PIT_F32}[t.dtype]


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t) -> int | None:
    return None if t is None else t.data_ptr()


@dataclass
class PitIndex:
    """Device-resident sparse index: seg_ptr int32[nseg+1], idx int32[cap], bits uint32-as-int32[cap] or None."""
    seg_ptr: torch.Tensor
    idx: torch.Tensor
    bits: torch.Tensor | None
    nseg: int
    cap: int

    def c(self) -> _CIndex:
        return _CIndex(self.seg_ptr.data_ptr(), self.idx.data_ptr(), _ptr(self.bits), self.nseg, self.cap)

    @staticmethod
    def empty(nseg: int, cap: int, want_bits: bool = False, device="cuda") -> "PitIndex":
        return PitIndex(torch.empty(nseg + 1, dtype=torch.int32, device=device),
                        torch.empty(max(cap, 1), dtype=torch.int32, device=device),
                        torch.empty(max(cap, 1), dtype=torch.int32, device=device) if want_bits else None,
                        nseg, cap)

    def to_host(self):
        """(seg_ptr, idx[:nnz], bits[:nnz] or None) as numpy arrays -- synchronises; for tests."""
        sp = self.seg_ptr.cpu().numpy()
        n = int(sp[-1])
        ix = self.idx[:n].cpu().numpy()
        bt = None if self.bits is None else self.bits[:n].cpu().numpy().view("uint32")
        return sp, ix, bt


def pit_build_index_workspace(rows, cols, mt_rows, mt_cols, pit_dim, want_bits=False) -> int:
    return _lib.pit_build_index_workspace(rows, cols, mt_rows, mt_cols, pit_dim, int(want_bits))


def pit_build_index(src: torch.Tensor, mt_rows: int, mt_cols: int, pit_dim: int, want_bits: bool = False,
                    out: PitIndex | None = None, ws: torch.Tensor | None = None) -> PitIndex:
    """Online sparsity detection on a 2-D tensor (last dim contiguous).  See include/pit.h."""
    assert src.dim() == 2 and src.stride(1) == 1
    rows, cols = src.shape
    if out is None:
        if rows % mt_rows or cols % mt_cols:
            raise PitError(PIT_ESHAPE, "pit_build_index")
        gr, gc = rows // mt_rows, cols // mt_cols
        out = PitIndex.empty(gc if pit_dim == 0 else gr, gr * gc, want_bits, src.device)
    if ws is None:
        ws = torch.empty(max(pit_build_index_workspace(rows, cols, mt_rows, mt_cols, pit_dim, want_bits), 8),
                         dtype=torch.uint8, device=src.device)
    ci = out.c()
    _check(_lib.pit_build_index(src.data_ptr(), _dt(src), rows, cols, src.stride(0) if rows > 1 else max(cols, src.stride(0)),
                                mt_rows, mt_cols, pit_dim, ctypes.byref(ci), ws.data_ptr(), ws.numel(), _stream()),
           "pit_build_index")
    return out


def pit_build_index_static_capacity() -> int:
    return _lib.pit_build_index_static_capacity()


def pit_build_index_static(src: torch.Tensor, mt_rows: int, mt_cols: int, pit_dim: int, out: PitIndex) -> PitIndex:
    """pit_build_index with the workspace inside the library (no allocation anywhere on the way: `out` is
    the caller's).  See include/pit.h."""
    assert src.dim() == 2 and src.stride(1) == 1
    rows, cols = src.shape
    ci = out.c()
    _check(_lib.pit_build_index_static(src.data_ptr(), _dt(src), rows, cols, src.stride(0) if rows > 1 else max(cols, src.stride(0)),
                                       mt_rows, mt_cols, pit_dim, ctypes.byref(ci), _stream()), "pit_build_index_static")
    return out


def pit_check_index(ix: PitIndex, npit: int, out: torch.Tensor | None = None) -> torch.Tensor:
    """Number of violations in an index (device int32[1]): see include/pit.h."""
    if out is None:
        out = torch.empty(1, dtype=torch.int32, device=ix.seg_ptr.device)
    ci = ix.c()
    _check(_lib.pit_check_index(ctypes.byref(ci), npit, out.data_ptr(), _stream()), "pit_check_index")
    return out


def pit_build_route_index_workspace(T, E) -> int:
    return _lib.pit_build_route_index_workspace(T, E)


def pit_build_route_index(expert_id: torch.Tensor, E: int, out: PitIndex | None = None,
                          status: torch.Tensor | None = None, ws: torch.Tensor | None = None) -> PitIndex:
    assert expert_id.dtype == torch.int32 and expert_id.is_contiguous()
    T = expert_id.numel()
    if out is None:
        out = PitIndex.empty(E, T, False, expert_id.device)
    if ws is None:
        ws = torch.empty(max(pit_build_route_index_workspace(T, E), 8), dtype=torch.uint8, device=expert_id.device)
    ci = out.c()
    _check(_lib.pit_build_route_index(expert_id.data_ptr(), T, E, ctypes.byref(ci), _ptr(status), ws.data_ptr(),
                                      ws.numel(), _stream()), "pit_build_route_index")
    return out


def pit_relu_channel_major_index_workspace(tokens, channels) -> int:
    return _lib.pit_relu_channel_major_index_workspace(tokens, channels)


def pit_relu_channel_major_index(H: torch.Tensor, out_xt: torch.Tensor | None = None, out: PitIndex | None = None,
                                 ws: torch.Tensor | None = None, index: bool = True):
    """Xt = ReLU(H)^T ([channels, tokens]) and its index at 1 x 128 micro-tiles in one pass over H
    ([tokens, channels], last dim contiguous).  Returns (Xt, index); with index=False no index is
    written and (Xt, None) is returned.  See include/pit.h."""
    assert H.dim() == 2 and H.stride(1) == 1
    tokens, channels = H.shape
    if out_xt is None:
        out_xt = torch.empty((channels, tokens), dtype=H.dtype, device=H.device)
    if not index:
        out = None
    elif out is None:
        if tokens % 128:
            raise PitError(PIT_ESHAPE, "pit_relu_channel_major_index")
        out = PitIndex.empty(tokens // 128, (tokens // 128) * channels, False, H.device)
    if ws is None:
        ws = torch.empty(max(pit_relu_channel_major_index_workspace(tokens, channels), 8), dtype=torch.uint8,
                         device=H.device)
    ci = out.c() if out is not None else None
    _check(_lib.pit_relu_channel_major_index(H.data_ptr(), H.stride(0) if tokens > 1 else max(channels, H.stride(0)),
                                             tokens, channels, _dt(H), out_xt.data_ptr(),
                                             out_xt.stride(0) if channels > 1 else max(tokens, out_xt.stride(0)),
                                             ctypes.byref(ci) if ci is not None else None, ws.data_ptr(), ws.numel(), _stream()),
           "pit_relu_channel_major_index")
    return out_xt, out


def pit_cover_count_workspace(rows, cols, mt_rows, mt_cols) -> int:
    return _lib.pit_cover_count_workspace(rows, cols, mt_rows, mt_cols)


def pit_cover_count(src: torch.Tensor, mt_rows: int, mt_cols: int, out: torch.Tensor | None = None,
                    ws: torch.Tensor | None = None) -> torch.Tensor:
    """CoverAlgo of Algorithm 1 on a 2-D tensor; returns a device int32[1].  See include/pit.h."""
    assert src.dim() == 2 and src.stride(1) == 1
    rows, cols = src.shape
    if out is None:
        out = torch.empty(1, dtype=torch.int32, device=src.device)
    if ws is None:
        ws = torch.empty(max(pit_cover_count_workspace(rows, cols, mt_rows, mt_cols), 8), dtype=torch.uint8,
                         device=src.device)
    _check(_lib.pit_cover_count(src.data_ptr(), _dt(src), rows, cols, src.stride(0) if rows > 1 else max(cols, src.stride(0)),
                                mt_rows, mt_cols, out.data_ptr(), ws.data_ptr(), ws.numel(), _stream()),
           "pit_cover_count")
    return out


def pit_select_kernel(candidates, num_tiles, grid_tiles):
    """Algorithm 1 on the host.  candidates: sequence of dicts (mt_rows, mt_cols, tile_cost, optional dense,
    optional fixed_cost); num_tiles / grid_tiles: [nsamples][ncand] integers.  Returns (best index, list of costs)."""
    cands, flat_n, flat_g, ncand, nsamples = _candidates(candidates, num_tiles, grid_tiles)
    costs = (ctypes.c_double * max(ncand, 1))()
    best = c_int(-1)
    _check(_lib.pit_select_kernel(cands, ncand, flat_n, flat_g, nsamples, costs, ctypes.byref(best)), "pit_select_kernel")
    return best.value, [costs[j] for j in range(ncand)]


def _check_operands(A: torch.Tensor, B: torch.Tensor, where: str) -> None:
    if A.dtype != B.dtype or A.dim() != 2 or B.dim() != 2 or (A.numel() and A.stride(1) != 1) or (B.numel() and B.stride(1) != 1):
        raise PitError(PIT_EINVAL, where + " (operands must be 2-D, of one 16-bit type, last dimension contiguous)")


def pit_sread_gemm(mode: int, A: torch.Tensor, B: torch.Tensor, ix: PitIndex | None, mt: int, M: int, N: int, K: int,
                   out: torch.Tensor | None = None, c_dtype=torch.float32, zero_uncovered: bool = True) -> torch.Tensor:
    """C = A.B over the listed micro-tiles.  GATHER_M: A is [M,K]; GATHER_K and DENSE_K (ix = None): A is At [K,M].
    B is [K,N]."""
    _check_operands(A, B, "pit_sread_gemm")
    if out is None:
        out = torch.empty((M, N), dtype=c_dtype, device=B.device)
    ci = ix.c() if ix is not None else None
    _check(_lib.pit_sread_gemm(mode, A.data_ptr(), A.stride(0), B.data_ptr(), B.stride(0), out.data_ptr(), out.stride(0),
                               M, N, K, _dt(B), _dt(out), ctypes.byref(ci) if ci is not None else None, mt,
                               int(zero_uncovered), _stream()),
           "pit_sread_gemm")
    return out


def _candidates(candidates, num_tiles, grid_tiles):
    ncand, nsamples = len(candidates), len(num_tiles)
    cands = (_CCandidate * max(ncand, 1))()
    for j, c in enumerate(candidates):
        cands[j] = _CCandidate(int(c["mt_rows"]), int(c["mt_cols"]), int(bool(c.get("dense", False))), float(c["tile_cost"]),
                               float(c.get("fixed_cost", 0.0)))
    flat_n = (c_i64 * max(ncand * nsamples, 1))(*[int(v) for row in num_tiles for v in row])
    flat_g = (c_i64 * max(ncand * nsamples, 1))(*[int(v) for row in grid_tiles for v in row])
    return cands, flat_n, flat_g, ncand, nsamples


def pit_select_and_run_gemm_workspace(M, K) -> int:
    return _lib.pit_select_and_run_gemm_workspace(M, K)


def pit_select_and_run_gemm(candidates, num_tiles, grid_tiles, At: torch.Tensor, B: torch.Tensor, M: int, N: int, K: int,
                            out: torch.Tensor | None = None, c_dtype=torch.float32, ws: torch.Tensor | None = None):
    """Algorithm 1 over `candidates` (as for pit_select_kernel) and the winner's kernel on At [K,M], B [K,N].
    Returns (C, index of the chosen candidate).  See include/pit.h."""
    _check_operands(At, B, "pit_select_and_run_gemm")
    if out is None:
        out = torch.empty((M, N), dtype=c_dtype, device=B.device)
    if ws is None:
        ws = torch.empty(max(pit_select_and_run_gemm_workspace(M, K), 256), dtype=torch.uint8, device=B.device)
    cands, flat_n, flat_g, ncand, nsamples = _candidates(candidates, num_tiles, grid_tiles)
    chosen = c_int(-1)
    _check(_lib.pit_select_and_run_gemm(cands, ncand, flat_n, flat_g, nsamples, At.data_ptr(), At.stride(0), B.data_ptr(),
                                        B.stride(0), out.data_ptr(), out.stride(0), M, N, K, _dt(B), _dt(out),
                                        ws.data_ptr(), ws.numel(), ctypes.byref(chosen), _stream()),
           "pit_select_and_run_gemm")
    return out, chosen.value


def pit_moe_workspace(T, d_model, d_ff, E) -> int:
    return _lib.pit_moe_workspace(T, d_model, d_ff, E)


def pit_moe_dispatch_gemm(X, expert_id, gate, W1, W2, out=None, y_dtype=torch.float32, act: int = 0,
                          status=None, ws=None) -> torch.Tensor:
    T, d_model = X.shape
    E, _, d_ff = W1.shape
    if not (X.dtype == W1.dtype == W2.dtype and X.is_contiguous() and W1.is_contiguous() and W2.is_contiguous()
            and expert_id.dtype == torch.int32 and expert_id.is_contiguous() and tuple(W2.shape) == (E, d_ff, d_model)
            and (gate is None or (gate.dtype == torch.float32 and gate.is_contiguous()))):
        raise PitError(PIT_EINVAL, "pit_moe_dispatch_gemm (contiguous X, W1, W2 of one 16-bit type, int32 expert ids, fp32 gate)")
    if out is None:
        out = torch.empty((T, d_model), dtype=y_dtype, device=X.device)
    if ws is None:
        ws = torch.empty(max(pit_moe_workspace(T, d_model, d_ff, E), 256), dtype=torch.uint8, device=X.device)
    _check(_lib.pit_moe_dispatch_gemm(X.data_ptr(), expert_id.data_ptr(), _ptr(gate), W1.data_ptr(), W2.data_ptr(),
                                      out.data_ptr(), _dt(out), T, d_model, d_ff, E, _dt(X), act, _ptr(status),
                                      ws.data_ptr(), ws.numel(), _stream()), "pit_moe_dispatch_gemm")
    return out


def pit_sparse_attn_workspace(H, S, D) -> int:
    return _lib.pit_sparse_attn_workspace(H, S, D)


def pit_sparse_attn(Q, K, V, mask, scale: float, out=None, o_dtype=torch.float32, ws=None) -> torch.Tensor:
    H, S, D = Q.shape
    if not (Q.dtype == K.dtype == V.dtype and Q.is_contiguous() and K.is_contiguous() and V.is_contiguous()
            and K.shape == Q.shape and V.shape == Q.shape and mask.dtype in (torch.uint8, torch.bool)
            and mask.is_contiguous() and tuple(mask.shape) == (S, S)):
        raise PitError(PIT_EINVAL, "pit_sparse_attn (contiguous Q, K, V of one 16-bit type and shape, byte mask [S, S])")
    if out is None:
        out = torch.empty((H, S, D), dtype=o_dtype, device=Q.device)
    if ws is None:
        ws = torch.empty(max(pit_sparse_attn_workspace(H, S, D), 256), dtype=torch.uint8, device=Q.device)
    _check(_lib.pit_sparse_attn(Q.data_ptr(), K.data_ptr(), V.data_ptr(), mask.data_ptr(), out.data_ptr(), _dt(out),
                                H, S, D, float(scale), _dt(Q), ws.data_ptr(), ws.numel(), _stream()), "pit_sparse_attn")
    return out


def raw():
    """The ctypes handle, for tests that exercise error returns with hand-made arguments."""
    return _lib, _CIndex
