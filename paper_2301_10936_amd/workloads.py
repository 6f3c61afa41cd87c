"""Seeded synthetic inputs for the dynamic-sparse GEMM hot path.

This module only *draws inputs* (random tensors, masks, routing decisions, lengths).  It holds
none of the method's arithmetic: no index construction, no GEMM, no softmax.  Both the CPU
oracle's tests and the HIP path's tests/bench read their inputs from here, so both sides see
identical bytes.

Conventions
-----------
* bf16 tensors are carried as ``numpy.uint16`` bit patterns (numpy has no bf16 type); fp16 tensors
  as ``numpy.float16``.  ``to_bf16_bits`` is the only numeric helper here: it quantises the
  *inputs* (round-to-nearest-even of an fp32 draw), which is input preparation, not part of the
  method.
* Every generator takes an explicit ``seed`` and uses ``numpy.random.Generator(PCG64(seed))``.
* Shapes default to the full workload sizes; tests pass smaller ones.

The five workloads mirror the situations the paper evaluates (Section 2.1 "Dynamic Sparsity" and
Section 5): fine-grained micro-tile sparsity in a matmul operand, ReLU activation sparsity in an
FFN, top-1 mixture-of-experts routing, padded variable-length batches, and dynamic sparse
attention (local window plus input-dependent global columns).
"""
from __future__ import annotations

import dataclasses
import numpy as np

BASE_SEED = 20230110


def rng_for(config: int, call: int = 0, seed: int | None = None) -> np.random.Generator:
    s = (BASE_SEED + 1000 * config + call) if seed is None else seed
    return np.random.Generator(np.random.PCG64(s))


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit pattern (uint16), round-to-nearest-even.  Input quantisation only."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    rounding = ((u >> 16) & 1) + np.uint32(0x7FFF)
    out = ((u + rounding) >> 16).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        out[nan] = 0x7FC0
    return out


# --------------------------------------------------------------------------------------------
# C1: micro-tile sparsity along K in a row-major operand
# --------------------------------------------------------------------------------------------
@dataclasses.dataclass
class MicroTileGemm:
    A: np.ndarray      # [M, K] float16, zero outside kept 1 x mt_k micro-tiles
    B: np.ndarray      # [K, N] float16
    keep: np.ndarray   # [M, K // mt_k] bool, the Bernoulli draw (for bookkeeping only)
    mt_k: int


def microtile_gemm(M=1024, K=1024, N=1024, mt_k=32, p_keep=0.1, seed=None, call=0,
                   integer=False) -> MicroTileGemm:
    """fp16 A with independent Bernoulli(p_keep) 1 x mt_k micro-tiles kept, fp16 B, N(0,1) values.

    ``integer=True`` draws small integers in [-4, 4] instead, so every partial sum is exactly
    representable in fp32 and the product has one right answer regardless of summation order.
    """
    g = rng_for(1, call, seed)
    if integer:
        A = g.integers(-4, 5, size=(M, K)).astype(np.float16)
        B = g.integers(-4, 5, size=(K, N)).astype(np.float16)
    else:
        A = g.standard_normal((M, K), dtype=np.float32).astype(np.float16)
        B = g.standard_normal((K, N), dtype=np.float32).astype(np.float16)
    keep = g.random((M, K // mt_k)) < p_keep
    A = (A.reshape(M, K // mt_k, mt_k) * keep[:, :, None]).reshape(M, K).astype(np.float16)
    return MicroTileGemm(A=A, B=B, keep=keep, mt_k=mt_k)


# --------------------------------------------------------------------------------------------
# C2: ReLU activation sparsity feeding an FFN down-projection
# --------------------------------------------------------------------------------------------
@dataclasses.dataclass
class ReluFfn:
    Xt: np.ndarray     # [K channels, M tokens] bf16 bits, channel-major (tokens contiguous)
    W: np.ndarray      # [K, N] bf16 bits
    M: int
    K: int
    N: int


def relu_ffn(M=2048, K=8192, N=2048, mean=-1.2, w_std=0.02, seed=None, call=0, integer=False,
             channel_live_prob: float | None = None, live_block: int = 128, live_offset: int = 0) -> ReluFfn:
    """X = ReLU(N(mean, 1)) stored channel-major, W ~ N(0, w_std).

    ``channel_live_prob`` (optional) adds zeros that are correlated across tokens: a channel is
    silenced for a whole run of ``live_block`` consecutive tokens with probability
    1 - channel_live_prob, which is the regime where whole micro-tiles vanish.  The runs start at
    tokens ``live_offset + i * live_block`` (the tokens before ``live_offset`` form a shorter first
    run), so with ``live_offset`` = 64 a run of 128 straddles two aligned blocks of 128 tokens.
    The default (None) is the independent-zeros recipe.
    """
    g = rng_for(2, call, seed)
    if integer:
        X = g.integers(-6, 3, size=(K, M)).astype(np.float32)
        W = g.integers(-4, 5, size=(K, N)).astype(np.float32)
    else:
        X = g.standard_normal((K, M), dtype=np.float32) + np.float32(mean)
        W = g.standard_normal((K, N), dtype=np.float32) * np.float32(w_std)
    X = np.maximum(X, np.float32(0.0))
    if channel_live_prob is not None:
        blk = int(live_block)
        lead = (blk - int(live_offset) % blk) % blk          # tokens dropped from the front of the first run
        nb = (M + lead + blk - 1) // blk
        live = g.random((K, nb)) < channel_live_prob
        live = np.repeat(live, blk, axis=1)[:, lead:lead + M]
        X = X * live
    return ReluFfn(Xt=to_bf16_bits(X), W=to_bf16_bits(W), M=M, K=K, N=N)


def relu_ffn_preactivation(M=2048, K=8192, mean=-1.2, seed=None, call=0, channel_live_prob: float | None = None) -> np.ndarray:
    """The tensor one step before ``relu_ffn``'s X: H[M tokens, K channels] ~ N(mean, 1) as bf16 bits, token-major
    (what an up-projection writes).  With ``channel_live_prob`` a channel is pushed below zero for a whole block of
    128 tokens with probability 1 - channel_live_prob, so that ReLU(H) has the correlated zeros of ``relu_ffn``."""
    g = rng_for(12, call, seed)
    H = g.standard_normal((M, K), dtype=np.float32) + np.float32(mean)
    if channel_live_prob is not None:
        blk = 128
        nb = (M + blk - 1) // blk
        dead = g.random((nb, K)) >= channel_live_prob
        dead = np.repeat(dead, blk, axis=0)[:M]
        H = np.where(dead, -np.abs(H) - np.float32(0.5), H)
    return to_bf16_bits(H)


# --------------------------------------------------------------------------------------------
# C3: top-1 mixture-of-experts FFN with skewed expert popularity
# --------------------------------------------------------------------------------------------
@dataclasses.dataclass
class MoeFfn:
    X: np.ndarray          # [T, d_model] bf16 bits
    expert_id: np.ndarray  # [T] int32
    gate: np.ndarray       # [T] float32
    W1: np.ndarray         # [E, d_model, d_ff] bf16 bits
    W2: np.ndarray         # [E, d_ff, d_model] bf16 bits


def moe_ffn(T=4096, d_model=768, d_ff=3072, E=64, zipf_s=1.1, w_std=0.02, seed=None, call=0,
            integer=False, unit_gate=False) -> MoeFfn:
    """Tokens iid over experts with popularity p_r ~ r^-zipf_s; rank->expert by a seeded permutation."""
    g = rng_for(3, call, seed)
    ranks = np.arange(1, E + 1, dtype=np.float64)
    p = ranks ** (-zipf_s)
    p /= p.sum()
    perm = g.permutation(E)
    expert_id = perm[g.choice(E, size=T, p=p)].astype(np.int32)
    if integer:
        X = g.integers(-2, 3, size=(T, d_model)).astype(np.float32)
        W1 = g.integers(-1, 2, size=(E, d_model, d_ff)).astype(np.float32)
        W2 = g.integers(-1, 2, size=(E, d_ff, d_model)).astype(np.float32)
    else:
        X = g.standard_normal((T, d_model), dtype=np.float32)
        W1 = g.standard_normal((E, d_model, d_ff), dtype=np.float32) * np.float32(w_std)
        W2 = g.standard_normal((E, d_ff, d_model), dtype=np.float32) * np.float32(w_std)
    gate = np.ones(T, dtype=np.float32) if unit_gate else (0.5 + 0.5 * g.random(T)).astype(np.float32)
    return MoeFfn(X=to_bf16_bits(X), expert_id=expert_id, gate=gate,
                  W1=to_bf16_bits(W1), W2=to_bf16_bits(W2))


# --------------------------------------------------------------------------------------------
# C4: padded batch of variable-length sequences through a linear layer
# --------------------------------------------------------------------------------------------
@dataclasses.dataclass
class PaddedLinear:
    X: np.ndarray        # [batch * max_len, hidden] bf16 bits; rows past a sequence's length hold junk
    W: np.ndarray        # [hidden, out] bf16 bits
    lengths: np.ndarray  # [batch] int32
    row_mask: np.ndarray # [batch * max_len] uint8, 1 for valid token rows (left-aligned)
    max_len: int


def padded_linear(batch=32, max_len=512, hidden=1024, out=4096, min_len=16, w_std=0.02, seed=None,
                  call=0, integer=False) -> PaddedLinear:
    g = rng_for(4, call, seed)
    lengths = g.integers(min_len, max_len + 1, size=batch).astype(np.int32)
    if integer:
        X = g.integers(-4, 5, size=(batch * max_len, hidden)).astype(np.float32)
        W = g.integers(-4, 5, size=(hidden, out)).astype(np.float32)
    else:
        X = g.standard_normal((batch * max_len, hidden), dtype=np.float32)
        W = g.standard_normal((hidden, out), dtype=np.float32) * np.float32(w_std)
    pos = np.arange(max_len)[None, :]
    row_mask = (pos < lengths[:, None]).astype(np.uint8).reshape(-1)
    return PaddedLinear(X=to_bf16_bits(X), W=to_bf16_bits(W), lengths=lengths, row_mask=row_mask,
                        max_len=max_len)


# --------------------------------------------------------------------------------------------
# C5: dynamic sparse attention mask (local window + per-query-block random key columns)
# --------------------------------------------------------------------------------------------
@dataclasses.dataclass
class SparseAttn:
    Q: np.ndarray     # [H, S, D] bf16 bits
    K: np.ndarray     # [H, S, D] bf16 bits
    V: np.ndarray     # [H, S, D] bf16 bits
    mask: np.ndarray  # [S, S] uint8, shared by heads; 1 = attend
    scale: float


def sparse_attn(H=12, S=4096, D=64, window=256, qblock=32, density=0.05, seed=None, call=0,
                integer=False) -> SparseAttn:
    """mask[i, j] = |i - j| <= window/2  OR  (key column j drawn for i's query block w.p. density)."""
    g = rng_for(5, call, seed)
    if integer:
        Q = g.integers(-1, 2, size=(H, S, D)).astype(np.float32)
        K = g.integers(-1, 2, size=(H, S, D)).astype(np.float32)
        V = g.integers(-4, 5, size=(H, S, D)).astype(np.float32)
    else:
        Q = g.standard_normal((H, S, D), dtype=np.float32)
        K = g.standard_normal((H, S, D), dtype=np.float32)
        V = g.standard_normal((H, S, D), dtype=np.float32)
    i = np.arange(S)[:, None]
    j = np.arange(S)[None, :]
    band = np.abs(i - j) <= window // 2
    nqb = (S + qblock - 1) // qblock
    cols = g.random((nqb, S)) < density
    glob = np.repeat(cols, qblock, axis=0)[:S]
    mask = (band | glob).astype(np.uint8)
    return SparseAttn(Q=to_bf16_bits(Q), K=to_bf16_bits(K), V=to_bf16_bits(V), mask=mask,
                      scale=1.0 / float(np.sqrt(D)))


# --------------------------------------------------------------------------------------------
# iid block patterns for the cover-density closed form (Table 3 of the paper)
# --------------------------------------------------------------------------------------------
def iid_block_mask(rows=4096, cols=4096, g_rows=2, g_cols=1, sparsity=0.95, seed=None, call=0) -> np.ndarray:
    """uint8 [rows, cols] mask whose g_rows x g_cols blocks are zero independently w.p. ``sparsity``."""
    g = rng_for(9, call, seed)
    keep = g.random((rows // g_rows, cols // g_cols)) >= sparsity
    return np.repeat(np.repeat(keep, g_rows, axis=0), g_cols, axis=1).astype(np.uint8)
