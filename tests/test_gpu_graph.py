"""GPU: the four calls of the hot path recorded into HIP graphs.

Every entry point is stream-ordered and allocates nothing, so a caller may capture it.  Each test records one
step into a graph with all buffers supplied, then replays the graph several times with new input contents
copied into the recorded buffers and with unrelated eager work and synchronisations between the replays, and
demands the bits of the eager call on the same inputs from every replay (a node that only works on the first
replay, e.g. a fill recorded as a memset, fails on the later ones)."""
import numpy as np
import pytest
import torch

from paper_2301_10936_amd import workloads as wl
from tests.gpu_util import dev, to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pit():
    from paper_2301_10936_amd import pit as p
    return p


def _capture(step):
    """Warm the step up on a side stream (first-call set-up must not be recorded), then record it."""
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        step()
    torch.cuda.current_stream().wait_stream(s)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    return g


def _replays(g, load, outs, eager, n=3):
    """load(i) fills the recorded input buffers with case i; eager(i) returns the outputs of a plain call on case i."""
    noise = torch.randn(1 << 20, device=dev())
    for i in list(range(n)) + [0]:
        load(i)
        for o in outs:
            o.fill_(float("nan")) if o.is_floating_point() else o.fill_(-7)
        g.replay()
        torch.cuda.synchronize()
        got = [o.clone() for o in outs]
        noise.mul_(1.0001).add_(1.0)              # unrelated eager work between the replays
        want = eager(i)
        torch.cuda.synchronize()
        for a, b in zip(got, want):
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), f"replay of case {i} differs from the eager call"


def test_index_and_gather_k_product(pit):
    M, K, N, MT = 512, 1024, 256, 128
    ws_ = [wl.relu_ffn(M=M, K=K, N=N, seed=s, channel_live_prob=0.3) for s in range(3)]
    W = to_dev(ws_[0].W)
    Xt = torch.empty((K, M), dtype=torch.bfloat16, device=dev())
    ix = pit.PitIndex.empty(M // MT, (M // MT) * K)
    wsb = torch.empty(pit.pit_build_index_workspace(K, M, 1, MT, 0), dtype=torch.uint8, device=dev())
    C = torch.empty((M, N), dtype=torch.float32, device=dev())

    def step():
        pit.pit_build_index(Xt, 1, MT, 0, out=ix, ws=wsb)
        pit.pit_sread_gemm(pit.PIT_GEMM_GATHER_K, Xt, W, ix, MT, M, N, K, out=C)

    Xt.copy_(to_dev(ws_[0].Xt))
    g = _capture(step)

    def eager(i):
        x = to_dev(ws_[i].Xt)
        jx = pit.pit_build_index(x, 1, MT, 0)
        return [pit.pit_sread_gemm(pit.PIT_GEMM_GATHER_K, x, W, jx, MT, M, N, K), jx.seg_ptr]

    _replays(g, lambda i: Xt.copy_(to_dev(ws_[i].Xt)), [C, ix.seg_ptr], eager)


def test_row_mask_index_and_gather_m_product_with_clearing(pit):
    cases = [wl.padded_linear(batch=8, max_len=128, hidden=128, out=256, min_len=1, seed=s) for s in range(3)]
    M, K = cases[0].X.shape
    N = cases[0].W.shape[1]
    X, W = to_dev(cases[0].X), to_dev(cases[0].W)
    mask = torch.empty((M, 1), dtype=torch.uint8, device=dev())
    ix = pit.PitIndex.empty(1, M)
    wsb = torch.empty(pit.pit_build_index_workspace(M, 1, 1, 1, 0), dtype=torch.uint8, device=dev())
    Y = torch.empty((M, N), dtype=torch.bfloat16, device=dev())

    def step():
        pit.pit_build_index(mask, 1, 1, 0, out=ix, ws=wsb)
        pit.pit_sread_gemm(pit.PIT_GEMM_GATHER_M, X, W, ix, K, M, N, K, out=Y, zero_uncovered=True)

    mask.copy_(to_dev(cases[0].row_mask.reshape(-1, 1)))
    g = _capture(step)

    def eager(i):
        m = to_dev(cases[i].row_mask.reshape(-1, 1))
        jx = pit.pit_build_index(m, 1, 1, 0)
        out = torch.full((M, N), 5.0, dtype=torch.bfloat16, device=dev())
        pit.pit_sread_gemm(pit.PIT_GEMM_GATHER_M, X, W, jx, K, M, N, K, out=out, zero_uncovered=True)
        return [out]

    _replays(g, lambda i: mask.copy_(to_dev(cases[i].row_mask.reshape(-1, 1))), [Y], eager)


def test_moe_call(pit):
    T, d_model, d_ff, E = 600, 128, 256, 8
    cases = [wl.moe_ffn(T=T, d_model=d_model, d_ff=d_ff, E=E, seed=s) for s in range(3)]
    W1, W2 = to_dev(cases[0].W1), to_dev(cases[0].W2)
    X = torch.empty((T, d_model), dtype=torch.bfloat16, device=dev())
    eid = torch.empty((T,), dtype=torch.int32, device=dev())
    gate = torch.empty((T,), dtype=torch.float32, device=dev())
    Y = torch.empty((T, d_model), dtype=torch.float32, device=dev())
    status = torch.zeros((1,), dtype=torch.int32, device=dev())
    wsb = torch.empty(pit.pit_moe_workspace(T, d_model, d_ff, E), dtype=torch.uint8, device=dev())

    def load(i):
        ids = cases[i].expert_id.copy()
        ids[i::97] = -1                           # some tokens without an expert: their rows of Y must come out zero
        X.copy_(to_dev(cases[i].X)); eid.copy_(to_dev(ids)); gate.copy_(to_dev(cases[i].gate))

    def step():
        pit.pit_moe_dispatch_gemm(X, eid, gate, W1, W2, out=Y, status=status, ws=wsb)

    load(0)
    g = _capture(step)

    def eager(i):
        ids = cases[i].expert_id.copy()
        ids[i::97] = -1
        st = torch.zeros((1,), dtype=torch.int32, device=dev())
        out = torch.full((T, d_model), 3.0, dtype=torch.float32, device=dev())
        pit.pit_moe_dispatch_gemm(to_dev(cases[i].X), to_dev(ids), to_dev(cases[i].gate), W1, W2, out=out, status=st)
        return [out, st]

    _replays(g, load, [Y, status], eager)


def test_sparse_attention_call(pit):
    H, S, D = 2, 512, 64
    cases = [wl.sparse_attn(H=H, S=S, D=D, window=64, density=0.1, seed=s) for s in range(3)]
    Q, K, V = (torch.empty((H, S, D), dtype=torch.bfloat16, device=dev()) for _ in range(3))
    mask = torch.empty((S, S), dtype=torch.uint8, device=dev())
    O = torch.empty((H, S, D), dtype=torch.float32, device=dev())
    wsb = torch.empty(pit.pit_sparse_attn_workspace(H, S, D), dtype=torch.uint8, device=dev())
    scale = float(cases[0].scale)

    def load(i):
        Q.copy_(to_dev(cases[i].Q)); K.copy_(to_dev(cases[i].K)); V.copy_(to_dev(cases[i].V)); mask.copy_(to_dev(cases[i].mask))

    def step():
        pit.pit_sparse_attn(Q, K, V, mask, scale, out=O, ws=wsb)

    load(0)
    g = _capture(step)

    def eager(i):
        return [pit.pit_sparse_attn(to_dev(cases[i].Q), to_dev(cases[i].K), to_dev(cases[i].V), to_dev(cases[i].mask), scale)]

    _replays(g, load, [O], eager)
