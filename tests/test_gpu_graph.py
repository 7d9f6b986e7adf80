"""The library's launches captured in a HIP graph and replayed.

Nothing in the entry points allocates, synchronises or clears memory, so a caller may capture them
(after one eager call: the first launch of a kernel on a device sets its LDS limit).  Every replay is
checked against an eager call on the same inputs, bit for bit, with new inputs and unrelated eager
work between the replays.  The tail split is the case with state across launches: its hand-over
flags carry a per-launch value that a replay repeats, so the collecting work-group takes them down
again after use."""
import numpy as np
import pytest
import torch

import paper_2604_26666_amd as fact
import workloads as wl
from oracle import check, ref

pytestmark = pytest.mark.gpu


def _bits(t):
    torch.cuda.synchronize()
    return wl.bits(t.cpu().contiguous())


def _replays(capture_fn, eager_fn, inputs, refresh, out, n=6):
    """capture_fn() issues the launches on the current stream; refresh(i) puts input set i into the
    static buffers; eager_fn() -> bits of an eager run on the buffers' current contents.
    The eager results come first: between two replays no other launch of the library runs, so a
    replay that relied on state left by the one before it (with the other inputs) would show."""
    want = []
    for i in range(inputs):
        refresh(i)
        want.append(eager_fn().copy())           # also the first launches, outside the capture
    assert not np.array_equal(want[0], want[1])
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        with torch.cuda.graph(g, stream=s):
            capture_fn()
    torch.cuda.current_stream().wait_stream(s)
    torch.cuda.synchronize()
    junk = torch.randn(512, 512, device="cuda")
    for i in range(n):
        refresh(i % inputs)
        out.fill_(0)
        (junk @ junk).sum().item()               # the program's own eager work and a synchronisation in between
        g.replay()
        got = _bits(out)
        assert np.array_equal(got, want[i % inputs]), f"replay {i} differs from the eager result"


@pytest.mark.parametrize("cfg,split", [(0, -2), (3, -2), (3, 4), (0, 1)])
def test_gemm_graph_replay(cfg, split):
    M, N, K = 512, 512, 2048                     # 4 (16) tiles: every tile is a tail tile shared by two work-groups
    sets = [(wl.normal((M, K), 1.0, f"gr.A{i}"), wl.normal((N, K), 0.05, f"gr.W{i}"), wl.normal((N,), 1.0, f"gr.b{i}")) for i in range(2)]
    A, W, b = (torch.empty_like(x).cuda() for x in sets[0])
    C = torch.zeros(M, N, dtype=torch.bfloat16, device="cuda")
    need = fact.fact_gemm_splitk_workspace_bytes(M, N, K, split)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
    ep = fact.Epilogue(bias=b, act=fact.ACT_GELU_TANH)

    def launch():
        fact.binding.check(fact.fact_gemm_ex(1, M, N, K, A, K, 0, W, K, 0, 1, C, N, 0, ep, cfg, split, 0, ws, need))

    def refresh(i):
        for dst, src in zip((A, W, b), sets[i]):
            dst.copy_(src)

    def eager():
        launch()
        return _bits(C)

    _replays(launch, eager, len(sets), refresh, C)
    refresh(1)
    launch()
    check.assert_close(_bits(C), ref.gemm_epilogue(sets[1][0], sets[1][1], True, bias=sets[1][2], act=fact.ACT_GELU_TANH), what="after the replays")


def test_persistent_gemm_graph_replay():
    # A persistent launch reads its parameters from the kernel-argument segment once per tile; a graph keeps
    # its own copy of that segment.  600 tiles of 128 x 128 on 512 resident work-groups: two rounds, the second ragged.
    cfg, M, N, K = 3, 24 * 128, 25 * 128, 264
    before = fact.fact_tune_persistent(1)
    try:
        assert fact.fact_persistent_grid(1, M, N, K, 1, fact.ACT_NONE, cfg) > 0
        sets = [(wl.normal((M, K), 1.0, f"gp.A{i}"), wl.normal((N, K), 0.05, f"gp.W{i}"), wl.normal((N,), 1.0, f"gp.b{i}")) for i in range(2)]
        A, W, b = (torch.empty_like(x).cuda() for x in sets[0])
        C = torch.zeros(M, N, dtype=torch.bfloat16, device="cuda")
        ep = fact.Epilogue(bias=b)

        def launch():
            fact.binding.check(fact.fact_gemm_ex(1, M, N, K, A, K, 0, W, K, 0, 1, C, N, 0, ep, cfg, 1, 0, None, 0))

        def refresh(i):
            for dst, src in zip((A, W, b), sets[i]):
                dst.copy_(src)

        def eager():
            launch()
            return _bits(C)

        _replays(launch, eager, len(sets), refresh, C)
        rows = np.arange(0, M, 131)
        check.assert_close(_bits(C)[rows], ref.gemm_epilogue(sets[1][0], sets[1][1], True, bias=sets[1][2], rows=rows), what="after the replays")
    finally:
        fact.fact_tune_persistent(before)


def test_attention_and_block_graph_replay():
    from test_gpu_block import make_block
    p, t, X0 = make_block("llama", 2, 200, 256, 4, 2, 64, 512)
    X1 = wl.normal(tuple(X0.shape), 1.0, "gr.X1")
    B, T, d = 2, 200, 256
    blk = fact.Block(B, T, d, 4, 2, 64, 512, 1, fact.ACT_SILU_GATE, 1, 1e-5, 500000.0, **{k: v.cuda() for k, v in t.items()})
    need = fact.fact_block_scratch_bytes(blk)
    scratch = torch.empty(need, dtype=torch.uint8, device="cuda")
    X = torch.empty_like(X0).cuda()
    Y = torch.zeros(B * T, d, dtype=torch.bfloat16, device="cuda")

    def launch():
        fact.binding.check(fact.fact_block_forward(blk, X, Y, scratch, need))

    def refresh(i):
        X.copy_((X0, X1)[i])

    def eager():
        launch()
        return _bits(Y)

    _replays(launch, eager, 2, refresh, Y)
