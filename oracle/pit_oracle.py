"""CPU oracle for the PIT dynamic-sparse GEMM hot path.  TEST INFRASTRUCTURE ONLY.

This file is the slow, plain definition of what the hot path computes.  It is imported only by
``tests/``, by ``__graft_entry__.smoke()`` and by the ``cpu_baseline`` leg of ``bench.py``.  The HIP
library never calls into it and shares no code, tables or helpers with it.

What is defined here and where the paper fixes it
-------------------------------------------------
* ``build_index``      -- online sparsity detection (Section 3.3): the coordinates, along the
  PIT-axis, of the micro-tiles that contain a non-zero value.  The paper leaves the order of the
  list free (any order is legal on a PIT-axis, Theorem 1); this oracle fixes the canonical order
  "ascending inside each segment" so that results are comparable bit for bit.
* ``gemm`` / ``gemm_rows_masked`` -- C = A.B (Table 1, MatMul).  The method gathers micro-tiles
  along m or k, runs dense tiles and scatters back; by the permutation-invariance argument
  (Section 2.3, Figure "Examples of sparse matrix multiplication") the result is exactly the dense
  product with the skipped entries being zeros.  So the oracle *is* the dense product, in fp64.
* ``gemm_over_index`` -- the same product written as a loop over the listed micro-tiles only; it
  exists to check the oracle against itself (sparse loop == dense-with-zeros).
* ``moe_ffn``          -- top-1 mixture-of-experts FFN (Section 2.1 "Mixture-of-Experts",
  Section 5.1 "Switch Transformer"): every token goes through its own expert's two matmuls;
  results land at the token's original position.  Written as a per-token loop, no grouping.
* ``sparse_attn``      -- attention restricted to a run-time mask (Section 5.1 "Longformer"):
  softmax over the allowed keys only.
* ``relu_channel_major`` -- the activation that produces C2-like sparsity, handed over in the layout
  Section 3.2 asks for when k is the PIT-axis (not contiguous along k), together with the index
  Section 3.3's detection gives on that tensor.  It is the plain composition ReLU -> transpose ->
  ``build_index``; the HIP side fuses the three.
* ``cover_count`` / ``sparsity_after_cover`` -- CoverAlgo of Algorithm 1: how many micro-tiles of
  a given shape are needed to cover all non-zeros (Table 3, column "Sparsity Ratio After Cover").

Readings taken where the paper is silent are listed next to each function.

Pins (tests/test_oracle_*.py, none of which use the GPU): brute force with pure-Python loops on
8x8 problems under exhaustive masks; bit-identical permutation round trips on small-integer data;
sparse-loop == dense-with-zeros; the cover ratios Table 3 prints (tests/golden/table3_cover.txt);
closed forms for GELU, softmax special cases and bf16 rounding.  No function here is
"parity unpinned".
"""
from __future__ import annotations

import math
import numpy as np
from scipy.special import erf as _erf


# ------------------------------------------------------------------------------------------------
# number formats
# ------------------------------------------------------------------------------------------------
def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact value of bf16 bit patterns (uint16): bf16 is the top half of an IEEE fp32."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def to_f64(x: np.ndarray) -> np.ndarray:
    """uint16 arrays are bf16 bit patterns; float16/float32/float64 arrays convert exactly."""
    if x.dtype == np.uint16:
        return bf16_bits_to_f64(x)
    return np.asarray(x).astype(np.float64)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round fp64 values to the nearest bf16 value (8-bit significand, ties to even), returned as fp64.

    Done on the fp64 value directly (one rounding): x = m * 2**e with 0.5 <= |m| < 1, the bf16
    spacing at x is 2**(e-8), floored at the subnormal spacing 2**-133.  Magnitudes beyond the
    bf16 range are not expected in this path and are left to overflow to inf like fp32 would.
    """
    x = np.asarray(x, dtype=np.float64)
    _, e = np.frexp(x)
    q = np.maximum(e - 8, -133)
    r = np.ldexp(np.rint(np.ldexp(x, -q)), q)
    r = np.where(np.abs(r) >= 2.0 ** 128, np.copysign(np.inf, x), r)
    return np.where(np.isfinite(x), r, x)


def is_nonzero(src: np.ndarray) -> np.ndarray:
    """The zero test of sparsity detection: numeric ``x != 0``.

    Reading (the paper gives no threshold): -0.0 counts as zero; NaN, Inf and subnormals count as
    non-zero.  For a mask tensor (uint8) any non-zero byte counts.
    """
    if src.dtype == np.uint16:                       # bf16 bit patterns
        return (src & np.uint16(0x7FFF)) != 0
    if src.dtype.kind == "f":
        return ~(src == 0)                           # NaN != 0 -> True
    return src != 0


# ------------------------------------------------------------------------------------------------
# index construction (Section 3.3)
# ------------------------------------------------------------------------------------------------
def build_index(src: np.ndarray, mt_rows: int, mt_cols: int, pit_dim: int):
    """Canonical micro-tile index of a 2-D tensor held in its ordinary dense storage.

    The tensor is cut into a grid of ``mt_rows x mt_cols`` micro-tiles (both must divide the
    shape).  ``pit_dim`` names the storage dimension that is the PIT-axis: 0 = rows, 1 = columns.
    A *segment* is one line of the micro-tile grid running along the PIT-axis: with pit_dim = 0
    there is one segment per micro-tile column, with pit_dim = 1 one per micro-tile row.

    Returns
      seg_ptr : int32 [nseg + 1]   exclusive prefix sums of the per-segment counts
      idx     : int32 [nnz]        for segment s, idx[seg_ptr[s]:seg_ptr[s+1]] are the micro-tile
                                   coordinates along the PIT-axis, ascending, of the micro-tiles
                                   that contain at least one non-zero
      bits    : uint32 [nnz] or None   when a micro-tile has <= 32 elements: bit (r*mt_cols + c) is
                                   set iff element (r, c) of that micro-tile is non-zero
    """
    rows, cols = src.shape
    if rows % mt_rows or cols % mt_cols:
        raise ValueError("shape must be a multiple of the micro-tile")
    gr, gc = rows // mt_rows, cols // mt_cols
    nz = is_nonzero(src).reshape(gr, mt_rows, gc, mt_cols)
    grid = nz.any(axis=(1, 3))                                       # [gr, gc]
    want_bits = mt_rows * mt_cols <= 32
    if want_bits:
        # element (r, c) of a micro-tile -> bit r*mt_cols + c
        weight = (np.uint64(1) << np.arange(mt_rows * mt_cols, dtype=np.uint64))
        flat = nz.transpose(0, 2, 1, 3).reshape(gr, gc, mt_rows * mt_cols)
        bits_grid = (flat.astype(np.uint64) * weight).sum(axis=2).astype(np.uint32)
    seg_ptr = [0]
    idx: list[np.ndarray] = []
    bits: list[np.ndarray] = []
    nseg = gc if pit_dim == 0 else gr
    for s in range(nseg):
        line = grid[:, s] if pit_dim == 0 else grid[s, :]
        coords = np.flatnonzero(line)                                # ascending
        idx.append(coords)
        if want_bits:
            bits.append(bits_grid[coords, s] if pit_dim == 0 else bits_grid[s, coords])
        seg_ptr.append(seg_ptr[-1] + len(coords))
    cat = lambda parts, dt: (np.concatenate(parts).astype(dt) if parts else np.zeros(0, dt))
    return (np.asarray(seg_ptr, dtype=np.int32), cat(idx, np.int32),
            cat(bits, np.uint32) if want_bits else None)


def route_index(expert_id: np.ndarray, E: int):
    """Index of a top-1 routing decision: segment e lists, ascending, the tokens sent to expert e.

    This is ``build_index`` applied to the [T x E] one-hot routing matrix with 1x1 micro-tiles and
    the token axis as PIT-axis; it is written out directly because the one-hot matrix is never
    materialised by the method either (Section 5.1, "Switch Transformer").
    """
    seg_ptr = [0]
    idx: list[int] = []
    for e in range(E):
        for t in range(len(expert_id)):
            if int(expert_id[t]) == e:
                idx.append(t)
        seg_ptr.append(len(idx))
    return np.asarray(seg_ptr, dtype=np.int32), np.asarray(idx, dtype=np.int32)


def cover_count(src: np.ndarray, mt_rows: int, mt_cols: int) -> int:
    """CoverAlgo (Algorithm 1): number of micro-tiles of this shape needed to cover all non-zeros."""
    rows, cols = src.shape
    nz = is_nonzero(src).reshape(rows // mt_rows, mt_rows, cols // mt_cols, mt_cols)
    return int(nz.any(axis=(1, 3)).sum())


def sparsity_after_cover(src: np.ndarray, mt_rows: int, mt_cols: int) -> float:
    """Fraction of the tensor NOT touched once every non-zero is covered (Table 3, 4th column)."""
    rows, cols = src.shape
    return 1.0 - cover_count(src, mt_rows, mt_cols) * mt_rows * mt_cols / float(rows * cols)


def select_kernel(samples, candidates):
    """Kernel selection (Algorithm 1, Section 3.2 "Micro-tile and Kernel Selection").

    ``candidates`` is the algorithm's double loop over dense computation tiles T and PIT-axes A
    written out: each entry is a dict with the micro-tile shape that (T, A) induces on the sparse
    operand (``mt_rows``, ``mt_cols``) and ``tile_cost``, the profiled running time of the sparse
    kernel per covered micro-tile.  An entry with ``dense=True`` stands for the dense kernel: it
    processes every micro-tile of the grid whatever the data, which is how low sparsity falls back
    to dense computation.  For every candidate the cost is the sum over the sparsity samples of
    CoverAlgo(sample, micro-tile) * tile_cost; the result is (index of the cheapest candidate, the
    first one among equals; list of all costs).  An optional ``fixed_cost`` per candidate (default 0,
    which is the paper's formula) is added once per sample: a reading that goes beyond the paper, for
    hardware where a run has a constant part next to the part proportional to the tiles.
    parity pinned in tests/test_oracle_select.py."""
    best, best_cost, costs = -1, math.inf, []
    for i, c in enumerate(candidates):
        cost = 0.0
        for D in samples:
            rows, cols = D.shape
            if c.get("dense", False):
                num_tiles = (rows // c["mt_rows"]) * (cols // c["mt_cols"])
            else:
                num_tiles = cover_count(D, c["mt_rows"], c["mt_cols"])
            cost += c.get("fixed_cost", 0.0) + num_tiles * c["tile_cost"]
        costs.append(cost)
        if cost < best_cost:
            best, best_cost = i, cost
    return best, costs


# ------------------------------------------------------------------------------------------------
# the producer of activation sparsity (Sections 2.1 "ReLU", 3.2 layout, 3.3 detection)
# ------------------------------------------------------------------------------------------------
def relu(H: np.ndarray) -> np.ndarray:
    """ReLU(x) = max(x, 0), element by element, in the storage type of H (uint16 = bf16 bits).

    Reading (the paper does not discuss special values): both zeros and every negative value,
    -Inf included, give +0; NaN is passed through unchanged (max with one NaN operand is not
    ordered, and a NaN must stay visible); +Inf stays +Inf.
    """
    x = to_f64(H)
    clamp = x <= 0                                   # False for NaN
    zero = np.zeros((), dtype=H.dtype)
    return np.where(clamp, zero, H)


def relu_channel_major(H: np.ndarray, mt_tokens: int = 128):
    """H is [tokens, channels].  Returns (Xt, seg_ptr, idx): Xt = ReLU(H) transposed to
    [channels, tokens] and the index of Xt over micro-tiles of 1 channel x ``mt_tokens`` tokens with the
    channel as PIT coordinate (one segment per block of ``mt_tokens`` tokens, listing its live channels)."""
    Xt = np.ascontiguousarray(relu(H).T)
    seg_ptr, idx, _ = build_index(Xt, 1, mt_tokens, 0)
    return Xt, seg_ptr, idx


# ------------------------------------------------------------------------------------------------
# GEMM (Table 1 "MatMul": C[m,n] += A[m,k] * B[k,n])
# ------------------------------------------------------------------------------------------------
def gemm(A: np.ndarray, B: np.ndarray) -> np.ndarray:
    """C = A.B in fp64.  A is [M, K], B is [K, N]; zeros of the sparse operand are literal zeros."""
    return np.matmul(to_f64(A), to_f64(B))


def gemm_at(At: np.ndarray, B: np.ndarray) -> np.ndarray:
    """C = At^T . B for an operand stored K-major ([K, M], the layout Section 3.2 asks for when
    k is the PIT-axis: non-contiguous along the PIT-axis)."""
    return np.matmul(to_f64(At).T, to_f64(B))


def gemm_rows_masked(A: np.ndarray, row_mask: np.ndarray, B: np.ndarray) -> np.ndarray:
    """C = diag(row_mask != 0) . A . B : rows outside the mask are zero rows whatever A holds there
    (padding tokens, Section 2.1 "Dynamic Sequence Length"); their outputs are exactly zero."""
    Af = np.where((np.asarray(row_mask) != 0)[:, None], to_f64(A), 0.0)   # padding may hold NaN/Inf
    return np.matmul(Af, to_f64(B))


def gemm_over_index(A: np.ndarray, B: np.ndarray, seg_ptr, idx, mt_rows: int, mt_cols: int,
                    pit_dim: int) -> np.ndarray:
    """The product as a loop over the *listed* micro-tiles of A only (A is [M, K] in storage order).

    Every listed micro-tile A[r0:r1, k0:k1] adds A[r0:r1, k0:k1] . B[k0:k1, :] to C[r0:r1, :].
    Used to check the oracle against itself: it must agree with ``gemm`` when the index covers
    all non-zeros of A.
    """
    Af, Bf = to_f64(A), to_f64(B)
    C = np.zeros((Af.shape[0], Bf.shape[1]), dtype=np.float64)
    nseg = len(seg_ptr) - 1
    for s in range(nseg):
        for j in range(int(seg_ptr[s]), int(seg_ptr[s + 1])):
            c = int(idx[j])
            tr, tc = (c, s) if pit_dim == 0 else (s, c)
            r0, k0 = tr * mt_rows, tc * mt_cols
            C[r0:r0 + mt_rows, :] += Af[r0:r0 + mt_rows, k0:k0 + mt_cols] @ Bf[k0:k0 + mt_cols, :]
    return C


# ------------------------------------------------------------------------------------------------
# mixture of experts (Sections 2.1 and 5.1)
# ------------------------------------------------------------------------------------------------
def gelu(x: np.ndarray) -> np.ndarray:
    """Exact GELU: x * Phi(x) = 0.5 x (1 + erf(x / sqrt 2)).  (Reading: the paper names no form.)"""
    return 0.5 * x * (1.0 + _erf(x / math.sqrt(2.0)))


def moe_ffn(X, expert_id, gate, W1, W2, activation: str = "gelu", round_hidden: bool = True) -> np.ndarray:
    """Y[t] = gate[t] * ( act( X[t] . W1[e] ) . W2[e] ),  e = expert_id[t];  top-1, no capacity limit.

    Readings: no bias; exact-erf GELU; the hidden vector is rounded to bf16 before the second
    matmul because the method stores it as a bf16 matmul operand (``round_hidden=False`` gives
    the unrounded value for error reporting); ``gate=None`` means 1.
    ``activation='identity'`` is used by exact-integer tests.
    """
    Xf = to_f64(X)
    T = Xf.shape[0]
    E = W1.shape[0]
    cache: dict[int, tuple[np.ndarray, np.ndarray]] = {}
    Y = np.zeros((T, W2.shape[2]), dtype=np.float64)
    for t in range(T):
        e = int(expert_id[t])
        if not 0 <= e < E:
            raise ValueError("expert id out of range")
        if e not in cache:
            cache[e] = (to_f64(W1[e]), to_f64(W2[e]))
        w1, w2 = cache[e]
        h = Xf[t] @ w1
        if activation == "gelu":
            h = gelu(h)
        elif activation != "identity":
            raise ValueError(activation)
        if round_hidden:
            h = round_to_bf16(h)
        y = h @ w2
        Y[t] = y * (1.0 if gate is None else float(gate[t]))
    return Y


# ------------------------------------------------------------------------------------------------
# dynamic sparse attention (Section 5.1 "Longformer")
# ------------------------------------------------------------------------------------------------
def sparse_attn(Q, K, V, mask, scale: float) -> np.ndarray:
    """O[h] = softmax_over_allowed_keys( scale * Q[h] K[h]^T ) V[h];  mask [S, S] shared by heads.

    Readings: mask[i, j] != 0 lets query i see key j; not causal; a query with no allowed key
    gives a zero row.
    """
    Qf, Kf, Vf = to_f64(Q), to_f64(K), to_f64(V)
    allow = np.asarray(mask) != 0
    H = Qf.shape[0]
    O = np.zeros_like(Vf)
    for h in range(H):
        S_ = (Qf[h] @ Kf[h].T) * scale
        S_ = np.where(allow, S_, -np.inf)
        mx = S_.max(axis=1, keepdims=True)
        mx = np.where(np.isfinite(mx), mx, 0.0)
        P = np.exp(S_ - mx)                      # exp(-inf) = 0 for masked entries
        den = P.sum(axis=1, keepdims=True)
        P = np.divide(P, den, out=np.zeros_like(P), where=den > 0)
        O[h] = P @ Vf[h]
    return O


# ------------------------------------------------------------------------------------------------
# error measures used by the parity tests
# ------------------------------------------------------------------------------------------------
def rel_errors(got: np.ndarray, ref: np.ndarray):
    """(max relative error, Frobenius relative error).

    max relative error = max |got - ref| / max(|ref|, rms(ref)): errors on elements much smaller
    than the typical magnitude are measured against the typical magnitude.
    """
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    diff = np.abs(got - ref)
    rms = math.sqrt(float(np.mean(ref * ref))) if ref.size else 0.0
    if rms == 0.0:
        return (float(diff.max()) if diff.size else 0.0), float(np.linalg.norm(diff))
    max_rel = float((diff / np.maximum(np.abs(ref), rms)).max())
    fro = float(np.linalg.norm(diff) / np.linalg.norm(ref))
    return max_rel, fro
