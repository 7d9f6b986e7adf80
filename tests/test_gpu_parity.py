"""GPU parity: the HIP path through the C ABI against the CPU oracle, element by element.

Exact tests (identity, permutations, small integers, rounding ties) demand equal bits;
tolerance tests demand |got - z| <= 1e-2 * bound + 1e-3 per element and a relative
Frobenius error <= 5e-3 (the workload definition's criteria, written out in oracle/check.py).
"""
import numpy as np
import pytest
import torch

import paper_2604_26666_amd as fact
import workloads as wl
from oracle import check, ref

pytestmark = pytest.mark.gpu

@pytest.fixture(scope="module", autouse=True)
def _gpu():
    if not torch.cuda.is_available():
        pytest.fail("these tests need the GPU; none is visible")
    import os
    assert os.path.exists(fact.lib_path()), "libfact_gemm.so is not built"
    fact.lib()


def G():
    import gpu_util
    return gpu_util


def ncfg():
    return fact.fact_num_configs()


def cfgs(trans_b):
    """Tile configurations that serve this layout of B: [K][N] operands are staged in whole K-rows of
    the tile, which takes a power-of-two number of 16-byte chunks per row (not the 192-wide tiles)."""
    return [c for c in range(ncfg()) if trans_b or 64 % (fact.fact_config_info(c)[1] // 8) == 0]


def gate_capable(cfg):
    return True          # every compiled configuration pairs gate and up tiles inside a wave


# ---- exact: layouts, tile mapping, every configuration -------------------------------------

@pytest.mark.parametrize("trans_b", [0, 1])
def test_permutation_matrices_every_config(trans_b):
    n = 512
    X = wl.uniform((n, 384), "gp.X")                  # C = P X must reproduce rows of X bit for bit
    p = wl.permutation(n, "gp.perm")
    P = torch.eye(n, dtype=torch.bfloat16)[p].contiguous()
    Bmat = X if not trans_b else X.t().contiguous()
    want = wl.bits(X[p].contiguous())
    for cfg in cfgs(trans_b):
        got = G().gemm(P, Bmat, trans_b, cfg=cfg)
        assert np.array_equal(got, want), f"cfg {cfg}"
    # B = I: C = A
    A = wl.uniform((300, n), "gp.A")
    eye = torch.eye(n, dtype=torch.bfloat16)
    for cfg in cfgs(trans_b):
        assert np.array_equal(G().gemm(A, eye, trans_b, cfg=cfg), wl.bits(A)), f"cfg {cfg}"


@pytest.mark.parametrize("trans_b", [0, 1])
@pytest.mark.parametrize("shape", [(300, 264, 200), (520, 776, 1096), (64, 64, 64), (1, 8, 8), (257, 520, 72)])
def test_small_integers_bit_exact_every_config(shape, trans_b):
    M, N, K = shape
    A = wl.small_int((M, K), -2, 2, f"gi.A{shape}")
    B = wl.small_int((K, N), -2, 2, f"gi.B{shape}")
    Bs = B if not trans_b else B.t().contiguous()
    r = ref.gemm_epilogue(A, Bs, bool(trans_b))
    assert np.abs(r.z).max() <= 256 * 64       # exactly representable sums; bf16 rounding is the oracle's
    for cfg in cfgs(trans_b):
        got = G().gemm(A, Bs, trans_b, cfg=cfg, pad=8 if cfg % 2 else 0)
        check.assert_bits_equal(got, r, what=f"cfg {cfg} {shape} tb {trans_b}")


def test_rounding_ties_through_the_mfma_path_and_the_fallback():
    a = torch.tensor([1.0078125, 1.0234375, 1.0078125, -1.0078125] * 16, dtype=torch.float32)
    b = torch.tensor([1.5, 1.25] * 32, dtype=torch.float32)
    for K, entry in ((1, "fallback"), (64, "mfma")):
        A = torch.zeros(64, K)
        A[:, 0] = a
        B = torch.zeros(K, 64)
        B[0, :] = b
        A, B = A.to(torch.bfloat16), B.to(torch.bfloat16)
        r = ref.gemm_epilogue(A, B)
        rc, cfg, _ = fact.fact_select_config(1, 64, 64, K, 0, 0)
        assert (cfg < 0) == (entry == "fallback")
        got = G().gemm(A, B, 0)
        check.assert_bits_equal(got, r, what=entry)
        w = ref.widen(got)
        assert w[0, 0] == 1.515625 and w[1, 0] == 1.53125 and w[0, 1] == 1.2578125 and w[3, 0] == -1.515625


@pytest.mark.parametrize("trans_b", [0, 1])
def test_tiny_and_unaligned_shapes_use_the_guarded_kernel(trans_b):
    for (M, N, K) in [(1, 1, 1), (2, 3, 5), (5, 7, 3), (17, 33, 9), (33, 20, 100)]:
        A = wl.small_int((M, K), -3, 3, f"gt.A{M}{N}{K}")
        B = wl.small_int((K, N), -3, 3, f"gt.B{M}{N}{K}")
        Bs = B if not trans_b else B.t().contiguous()
        bias = wl.small_int((N,), -3, 3, "gt.bias")
        res = wl.small_int((M, N), -3, 3, "gt.res")
        r = ref.gemm_epilogue(A, Bs, bool(trans_b), bias=bias, residual=res)
        got = G().gemm(A, Bs, trans_b, bias=bias, residual=res, pad=3)
        check.assert_bits_equal(got, r, what=f"{(M, N, K)}")


def test_guarded_kernel_gated_epilogue_and_batches():
    # K = 9 is served by the guarded kernel only.  Small integers keep the gate and up sums exact, so
    # the only inexact step is SiLU in fp32: the output is held to the usual tolerance and to a much
    # tighter one that an up-weight matrix taken from another batch entry cannot meet.
    M, K, I = 13, 9, 11
    rc, cfg, _ = fact.fact_select_config(1, M, 2 * I, K, 1, fact.ACT_SILU_GATE)
    assert cfg < 0, "this shape is meant for the guarded kernel"
    for batch in (1, 3):
        X = wl.small_int((batch, M, K), -2, 2, f"gg.X{batch}")
        W = wl.small_int((batch, 2 * I, K), -2, 2, f"gg.W{batch}")        # distinct gate and up rows in every batch entry
        C = G().poisoned(batch * M, I).view(batch, M, I)
        ep = fact.Epilogue(act=fact.ACT_SILU_GATE)
        fact.binding.check(fact.fact_gemm_batched(batch, M, 2 * I, K, X.cuda(), K, M * K, W.cuda(), K, 2 * I * K, 1,
                                                  C, I, M * I, ep))
        out = G().bits_of(C)
        for b in range(batch):
            r = ref.gemm_epilogue(X[b], W[b], True, act=ref.ACT_SILU_GATE)
            check.assert_close(out[b], r, what=f"gated fallback batch {b} of {batch}")
            # tight: the only inexact step is SiLU in fp32 (relative 1e-6) before one bf16 rounding
            got = ref.widen(out[b])
            assert np.abs(got - r.z).max() <= 2.0 ** -8 * np.abs(r.z).max() + 1e-6, f"batch {b}: up weights of another batch entry?"
            assert len({out[b].tobytes() for b in range(batch)}) == batch


def test_all_ones_closed_form():
    for K in (64, 256, 1024, 4096):
        A = torch.ones(256, K, dtype=torch.bfloat16)
        B = torch.ones(K, 256, dtype=torch.bfloat16)
        got = ref.widen(G().gemm(A, B, 0))
        assert (got == K).all()


# ---- epilogues --------------------------------------------------------------------------------

@pytest.mark.parametrize("trans_b", [0, 1])
def test_epilogue_wiring_exact(trans_b):
    # integer bias / residual keep every value exact: bits must match
    M, N, K = 200, 328, 136
    A = wl.small_int((M, K), -2, 2, "ge.A")
    B = wl.small_int((K, N), -2, 2, "ge.B")
    Bs = B if not trans_b else B.t().contiguous()
    bias = wl.small_int((N,), -5, 5, "ge.bias")
    res = wl.small_int((M, N), -5, 5, "ge.res")
    for kw in (dict(bias=bias), dict(residual=res), dict(bias=bias, residual=res),
               dict(bias=bias, residual=res, in_place=True)):
        oracle_kw = {k: v for k, v in kw.items() if k != "in_place"}
        r = ref.gemm_epilogue(A, Bs, bool(trans_b), **oracle_kw)
        for cfg in (0, 3, cfgs(trans_b)[-1]):
            got = G().gemm(A, Bs, trans_b, cfg=cfg, pad=8, **kw)
            check.assert_bits_equal(got, r, what=f"{list(kw)} cfg {cfg}")


@pytest.mark.parametrize("act", [fact.ACT_GELU_TANH, fact.ACT_SILU_GATE])
def test_activation_epilogues_within_tolerance(act):
    M, K, Nout = 264, 192, 328
    X = wl.normal((M, K), 1.0, "ga.X")
    res = wl.normal((M, Nout), 1.0, "ga.R")
    if act == fact.ACT_SILU_GATE:
        W = wl.normal((2 * Nout, K), 0.1, "ga.W2")
        bias = None
    else:
        W = wl.normal((Nout, K), 0.1, "ga.W")
        bias = wl.normal((Nout,), 0.5, "ga.b")
    r = ref.gemm_epilogue(X, W, True, bias=bias, residual=res, act=act)
    for cfg in range(ncfg()):
        if act == fact.ACT_SILU_GATE and not gate_capable(cfg):
            continue
        got = G().gemm(X, W, 1, bias=bias, residual=res, act=act, cfg=cfg)
        s = check.assert_close(got, r, what=f"act {act} cfg {cfg}")
        # far tighter than the tolerance: fp32 accumulation flips a bf16 rounding only near ties
        assert s["bits_equal_frac"] >= 0.99, s
    # the table's own choice, and the split-K path with the same epilogue
    check.assert_close(G().gemm(X, W, 1, bias=bias, residual=res, act=act), r)
    check.assert_close(G().gemm(X, W, 1, bias=bias, residual=res, act=act, cfg=3, split=3), r)


def test_gate_wiring_exact():
    # gate = an integer input feature, up = 1 exactly -> out = RNE(SiLU(g)): tells the gate
    # half from the up half (swapped, the result would be SiLU(1) * g)
    M, K, I = 128, 64, 128
    X = wl.small_int((M, K), -3, 3, "gg.X")
    X[:, 0] = 1.0
    Wg = torch.zeros(I, K)
    Wu = torch.zeros(I, K)
    for j in range(I):
        Wg[j, j % K] = 1.0                        # g_j = x_{j mod K}
    Wu[:, 0] = 1.0                                # u_j = x_0 = 1
    W = torch.cat([Wg, Wu]).to(torch.bfloat16)
    r = ref.gemm_epilogue(X, W, True, act=fact.ACT_SILU_GATE)
    got = G().gemm(X, W, 1, act=fact.ACT_SILU_GATE)
    s = check.compare(got, r)
    assert s["ok"] and s["bits_equal_frac"] >= 0.99, s
    xs = X.to(torch.float64).numpy()
    want = ref.silu(xs[:, np.arange(I) % K])
    assert np.allclose(ref.widen(got), want, rtol=2 ** -7, atol=1e-6)


def test_gated_epilogue_keeps_the_sign_of_zero_in_every_config():
    # g = 0 exactly and u = -1: SiLU(0) * (-1) = -0, and without a bias nothing may turn it
    # into +0 (two such elements turn up in the 32768 x 14336 Llama gate/up output); with
    # u = +1 the result is +0.  Every tile configuration must give the oracle's bits.
    M, K, I = 512, 64, 384
    X = torch.zeros(M, K)
    X[:, 0] = 1.0
    Wg = torch.zeros(I, K)                          # g_j = 0
    Wu = torch.zeros(I, K)
    Wu[:, 0] = torch.where(torch.arange(I) % 2 == 0, -1.0, 1.0)
    X = X.to(torch.bfloat16)
    W = torch.cat([Wg, Wu]).to(torch.bfloat16)
    want = ref.gemm_epilogue(X, W, True, act=fact.ACT_SILU_GATE).bits
    assert set(np.unique(want[:, 0::2]).tolist()) == {0x8000} and set(np.unique(want[:, 1::2]).tolist()) == {0}
    for cfg in cfgs(1):
        got = G().gemm(X, W, 1, act=fact.ACT_SILU_GATE, cfg=cfg)
        assert np.array_equal(got, want), f"cfg {cfg}"


# ---- random inputs, the five configurations at reduced size -------------------------------------

def test_config1_full():
    c = wl.config1()
    r = ref.gemm_epilogue(c["A"], c["B"])
    got = G().gemm(c["A"], c["B"], 0)
    s = check.assert_close(got, r, what="config 1")
    assert s["bits_equal_frac"] >= 0.99, s
    for cfg in cfgs(0):
        check.assert_close(G().gemm(c["A"], c["B"], 0, cfg=cfg), r, what=f"config 1 cfg {cfg}")


def test_config2_reduced_with_bias():
    c = wl.config2(1024)
    r = ref.gemm_epilogue(c["A"], c["B"], bias=c["bias"])
    for cfg in cfgs(0):
        check.assert_close(G().gemm(c["A"], c["B"], 0, bias=c["bias"], cfg=cfg, group_m=1 + cfg % 5), r,
                           what=f"cfg {cfg}")


def test_batched_reduced_with_distinct_permutations():
    batch, n = 6, 256
    X = wl.uniform((batch, n, n), "gb.X")
    Pm = torch.stack([torch.eye(n, dtype=torch.bfloat16)[wl.permutation(n, f"gb.p{b}")] for b in range(batch)])
    Xd, Pd = X.cuda(), Pm.cuda()
    Cd = torch.zeros(batch, n, n, dtype=torch.bfloat16, device="cuda")
    fact.binding.check(fact.fact_gemm_batched(batch, n, n, n, Pd, n, n * n, Xd, n, n * n, 0, Cd, n, n * n, None))
    got = G().bits_of(Cd)
    for b in range(batch):
        want = wl.bits(X[b][wl.permutation(n, f"gb.p{b}")].contiguous())
        assert np.array_equal(got[b], want), f"batch {b}"
    # shared B (stride 0) and random data within tolerance
    c = wl.config3a(batch, n)
    Ad, Bd = c["A"].cuda(), c["B"].cuda()
    fact.binding.check(fact.fact_gemm_batched(batch, n, n, n, Ad, n, n * n, Bd, n, 0, 0, Cd, n, n * n, None))
    got = G().bits_of(Cd)
    for b in range(batch):
        check.assert_close(got[b], ref.gemm_epilogue(c["A"][b], c["B"][0]), what=f"batch {b}")


@pytest.mark.parametrize("trans_b", [0, 1])
def test_splitk_every_factor_is_exact_on_integers_and_deterministic(trans_b):
    M, N, K = 136, 264, 2048 + 72
    A = wl.small_int((M, K), -1, 1, "gs.A")
    B = wl.small_int((K, N), -1, 1, "gs.B")
    Bs = B if not trans_b else B.t().contiguous()
    bias = wl.small_int((N,), -2, 2, "gs.b")
    r = ref.gemm_epilogue(A, Bs, bool(trans_b), bias=bias)
    for split in (1, 2, 3, 5, 8, 33):
        got = G().gemm(A, Bs, trans_b, bias=bias, split=split)
        check.assert_bits_equal(got, r, what=f"split {split}")
    c = wl.config3b(128, 128, 8192)
    Bs = c["B"] if not trans_b else c["B"].t().contiguous()
    r = ref.gemm_epilogue(c["A"], Bs, bool(trans_b))
    first = G().gemm(c["A"], Bs, trans_b, split=16)
    check.assert_close(first, r, what="large-K reduced")
    for _ in range(3):
        assert np.array_equal(G().gemm(c["A"], Bs, trans_b, split=16), first)    # fixed reduction order
    check.assert_close(G().gemm(c["A"], Bs, trans_b, split=0), r, what="table's split")


@pytest.mark.parametrize("kind", ["gelu", "swiglu"])
def test_block_mlp_reduced(kind):
    T, d, dff = 520, 256, 768
    X = wl.normal((T, d), 1.0, "gm.X")
    W1 = wl.normal((dff, d), 0.05, "gm.W1")
    Wu = wl.normal((dff, d), 0.05, "gm.Wu")
    b1 = wl.normal((dff,), 0.05, "gm.b1")
    W2 = wl.normal((d, dff), 0.05, "gm.W2")
    b2 = wl.normal((d,), 0.05, "gm.b2")
    R = wl.normal((T, d), 1.0, "gm.R")
    gated = kind == "swiglu"
    act = fact.ACT_SILU_GATE if gated else fact.ACT_GELU_TANH
    Hd = G().poisoned(T, dff)
    Yd = G().poisoned(T, d)
    need = fact.fact_block_mlp_workspace_bytes(T, d, dff, act)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
    rc = fact.fact_block_mlp(T, d, dff, X.cuda(), W1.cuda(), Wu.cuda() if gated else None,
                             None if gated else b1.cuda(), act, W2.cuda(), None if gated else b2.cuda(),
                             R.cuda(), Hd, Yd, ws, need)
    fact.binding.check(rc, "fact_block_mlp")
    Hg, Yg = G().bits_of(Hd), G().bits_of(Yd)
    # end to end against the oracle's own H
    h, y = ref.block_mlp(X, W1, Wu if gated else None, None if gated else b1, act, W2,
                         None if gated else b2, R)
    check.assert_close(Hg, h, what="H")
    check.assert_close(Yg, y, what="Y end to end")
    # stage-wise strict: the oracle's second GEMM fed the GPU's H bits
    _, y2 = ref.block_mlp(X, W1, Wu if gated else None, None if gated else b1, act, W2,
                          None if gated else b2, R, H_bits=Hg)
    s = check.assert_close(Yg, y2, what="Y stage-wise")
    assert s["bits_equal_frac"] >= 0.99, s


def test_errors_launch_nothing():
    A = torch.zeros(64, 64, dtype=torch.bfloat16, device="cuda")
    C = G().poisoned(64, 64)
    assert fact.fact_gemm(64, 64, 64, A, 32, A, 64, 0, C, 64, None) == -2
    assert fact.fact_gemm_splitk(64, 64, 4096, A, 4096, A, 64, 0, C, 64, None, 4, None, 0) == -6
    assert fact.fact_gemm_ex(1, 64, 64, 64, A, 64, 0, A, 64, 0, 0, C, 64, 0, None, 99, 0, 0, None, 0) == -7
    assert (G().bits_of(C) == G().POISON).all()


# ---- tail split: the last, partly filled round of tiles shared along K ---------------------------

def _tail_timeouts(ws, *unused, **unused_kw):
    """1 if a work-group of a tail-split launch on this workspace gave up waiting for a partial tile
    (the helper pre-fills workspaces with 0xA5, which is no launch's identity)."""
    rc, gave_up = fact.fact_tail_timeouts(ws)
    assert rc == 0
    return gave_up


@pytest.mark.parametrize("trans_b", [0, 1])
@pytest.mark.parametrize("g", [2, 3])
def test_tail_split_every_tile_shared(trans_b, g):
    # fewer tiles than compute units: every tile is a tail tile, shared by g work-groups.
    # Ragged M and N (guarded epilogue path adds the partials), K not a multiple of the step.
    M, N, K = 264, 328, 1000
    A = wl.normal((M, K), 1.0, "ts.A")
    B = wl.normal((N, K) if trans_b else (K, N), 1.0, "ts.B")
    bias = wl.normal((N,), 1.0, "ts.b")
    res = wl.normal((M, N), 1.0, "ts.R")
    r = ref.gemm_epilogue(A, B, bool(trans_b), bias=bias, residual=res, act=fact.ACT_GELU_TANH)
    for cfg in (0, 3, 6, 11):
        keep = []
        got = G().gemm(A, B, trans_b, bias=bias, residual=res, act=fact.ACT_GELU_TANH, cfg=cfg, split=-g, return_ws=keep)
        s = check.assert_close(got, r, what=f"tail split g={g} cfg {cfg}")
        assert s["bits_equal_frac"] >= 0.97, s
        again = G().gemm(A, B, trans_b, bias=bias, residual=res, act=fact.ACT_GELU_TANH, cfg=cfg, split=-g)
        assert np.array_equal(got, again), "tail split is not bit-reproducible"
        assert _tail_timeouts(keep[0], cfg, M, N, K, g) == 0


def test_tail_split_interior_and_gated():
    # aligned shape (straight-line epilogue adds the partials); gated epilogue
    M, K, I = 512, 1024, 512
    X = wl.normal((M, K), 1.0, "tg.X")
    W = wl.normal((2 * I, K), 0.1, "tg.W")
    r = ref.gemm_epilogue(X, W, True, act=fact.ACT_SILU_GATE)
    for cfg in (0, 3, 12):
        for g in (2, 4):
            got = G().gemm(X, W, 1, act=fact.ACT_SILU_GATE, cfg=cfg, split=-g)
            s = check.assert_close(got, r, what=f"gated tail split g={g} cfg {cfg}")
            assert s["bits_equal_frac"] >= 0.97, s
    A = wl.normal((M, K), 1.0, "tg.A")
    B = wl.normal((K, I), 1.0, "tg.B")
    r = ref.gemm_epilogue(A, B, False)
    for cfg in (0, 1, 3):
        got = G().gemm(A, B, 0, cfg=cfg, split=-2)
        check.assert_close(got, r, what=f"plain tail split cfg {cfg}")


def test_tail_split_after_full_rounds():
    # more tiles than work-group slots: 576 tiles of 64 x 64 on 512 slots -> 512 whole tiles + 64 shared
    n, K = 1536, 512
    A = wl.uniform((n, K), "tf.A")
    B = wl.uniform((n, K), "tf.B")
    r = ref.gemm_epilogue(A, B, True)
    keep = []
    got = G().gemm(A, B, 1, cfg=6, split=-2, return_ws=keep)
    check.assert_close(got, r, what="tail split after full rounds")
    assert _tail_timeouts(keep[0], 6, n, n, K, 2) == 0
    plain = G().gemm(A, B, 1, cfg=6)
    whole = 512 * 64 * 64            # outputs of tiles computed whole are identical to the plain launch's
    assert (got != plain).sum() <= got.size - whole


def test_tail_split_wait_that_gives_up_is_reported_not_hidden():
    # The give-up branch, forced from the host (a negative poll budget makes the finishing work-groups
    # give up at once; every kernel still runs to its end): the shared tiles come out as NaN, whole
    # tiles are untouched, the workspace's status word reports it, and the next launch with the
    # normal budget is correct again on the same workspace.
    n, K = 1536, 512                 # 576 tiles of 64 x 64 on 512 slots -> 512 whole tiles + 64 shared by two work-groups
    A = wl.uniform((n, K), "tt.A")
    B = wl.uniform((n, K), "tt.B")
    plain = G().gemm(A, B, 1, cfg=6)
    keep = []
    try:
        fact.fact_test_tail_poll_budget(-1)
        got = G().gemm(A, B, 1, cfg=6, split=-2, return_ws=keep)
    finally:
        fact.fact_test_tail_poll_budget(1 << 20)
    ws = keep[0]
    nan = (got & 0x7FFF) > 0x7F80
    assert nan.sum() == 64 * 64 * 64, "exactly the 64 shared tiles are NaN"
    tiles = nan.reshape(n // 64, 64, n // 64, 64).transpose(0, 2, 1, 3).reshape(-1, 64 * 64)
    assert set(tiles.sum(1).tolist()) == {0, 64 * 64}, "a shared tile is NaN in every element, a whole tile in none"
    assert np.array_equal(got[~nan], plain[~nan])
    assert _tail_timeouts(ws) == 1
    # same workspace, normal budget: correct, and bit-identical to a run on a fresh workspace
    Ad, Bd = A.cuda(), B.cuda()
    C = G().poisoned(n, n)
    need = fact.fact_gemm_splitk_workspace_bytes(n, n, K, -2)
    fact.binding.check(fact.fact_gemm_ex(1, n, n, K, Ad, K, 0, Bd, K, 0, 1, C, n, 0, None, 6, -2, 0, ws, need))
    again = G().bits_of(C)
    fresh = G().gemm(A, B, 1, cfg=6, split=-2)
    assert np.array_equal(again, fresh) and not ((again & 0x7FFF) > 0x7F80).any()
    assert _tail_timeouts(ws) == 1            # the word is sticky until the caller clears the workspace
    ws.fill_(0)
    assert _tail_timeouts(ws) == 0
    assert fact.fact_tail_timeouts(None)[0] == -1 and fact.fact_tail_timeouts(ws.data_ptr() + 8)[0] == -3


def test_tail_split_refusals():
    A = wl.normal((256, 128), 1.0, "tr.A")
    B = wl.normal((256, 128), 1.0, "tr.B")
    with pytest.raises(Exception):
        G().gemm(A, B, 1, cfg=3, split=-2)        # 2 K steps: too little K per range


# ---- fp32 output (by the main kernel's epilogue; by the reduction pass when K is split) ------------------

def _f32_call(A, B, trans_b, split, bias=None, residual=None, act=fact.ACT_NONE, cfg=-1):
    M, K = A.shape
    N = B.shape[0] if trans_b else B.shape[1]
    nout = N // 2 if act == fact.ACT_SILU_GATE else N
    C = torch.full((M + 1, nout + 4), float("nan"), dtype=torch.float32, device="cuda")
    need = fact.fact_gemm_f32out_workspace_bytes(M, N, K, split)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda").fill_(0xA5)
    ep = fact.Epilogue(bias=G().to_dev(bias), residual=G().to_dev(residual), ldr=nout, act=act, out_f32=1)
    Ad, Bd = A.cuda(), B.cuda()
    if cfg >= 0:
        rc = fact.fact_gemm_ex(1, M, N, K, Ad, K, 0, Bd, B.shape[1], 0, trans_b, C, nout + 4, 0, ep, cfg, split, 0, ws, need)
    else:
        rc = fact.fact_gemm_splitk(M, N, K, Ad, K, Bd, B.shape[1], trans_b, C, nout + 4, ep, split, ws, need)
    fact.binding.check(rc, f"fp32-output GEMM split={split}")
    torch.cuda.synchronize()
    out = C.cpu().numpy()
    assert np.isnan(out[M]).all() and np.isnan(out[:, nout:]).all(), "wrote outside C"
    return out[:M, :nout].astype(np.float64)


def _assert_f32_close(got, r, what):
    # the paper's own criterion for an fp32 result (Section 5.1: rtol 1e-3, atol 1e-5), and far tighter in norm
    err = np.abs(got - r.z)
    assert (err <= 1e-5 + 1e-3 * np.abs(r.z)).all(), (what, float(err.max()))
    assert np.linalg.norm(got - r.z) <= 2e-6 * np.linalg.norm(r.z) + 1e-12, (what, float(np.linalg.norm(got - r.z) / np.linalg.norm(r.z)))


@pytest.mark.parametrize("split", [1, 4, 0])
def test_fp32_output_large_k(split):
    M, N, K = 256, 264, 16384
    A = wl.normal((M, K), K ** -0.5, "f32.A")
    B = wl.normal((K, N), K ** -0.5, "f32.B")
    r = ref.gemm_epilogue(A, B, False)
    _assert_f32_close(_f32_call(A, B, 0, split), r, f"fp32 out split {split}")


def test_fp32_output_with_epilogue_and_exact_integers():
    M, N, K = 200, 256, 512
    A = wl.small_int((M, K), -2, 2, "f32.Ai")
    W = wl.small_int((N, K), -2, 2, "f32.Wi")
    bias = wl.normal((N,), 1.0, "f32.b")
    res = wl.normal((M, N), 1.0, "f32.R")
    r = ref.gemm_epilogue(A, W, True, bias=bias, residual=res)
    got = _f32_call(A, W, 1, 2, bias=bias, residual=res, cfg=3)
    assert np.array_equal(got, r.z.astype(np.float32).astype(np.float64))      # integers + bf16 bias + bf16 residual: exact in fp32
    r = ref.gemm_epilogue(A, W, True, bias=bias, act=fact.ACT_GELU_TANH)
    _assert_f32_close(_f32_call(A, W, 1, 1, bias=bias, act=fact.ACT_GELU_TANH), r, "fp32 out GELU")
    assert np.abs(_f32_call(A, W, 1, 1, bias=bias, act=fact.ACT_GELU_TANH) - r.z).max() < 5e-4     # fast-math GELU, not a rounding to bf16


def test_fp32_output_without_workspace_plain_and_batched():
    # K whole: every entry point writes fp32 straight from its epilogue, ragged edges and every tile shape included
    M, N, K = 300, 264, 520
    A = wl.normal((M, K), 1.0, "f32d.A")
    W = wl.normal((N, K), 0.05, "f32d.W")
    bias = wl.normal((N,), 1.0, "f32d.b")
    r = ref.gemm_epilogue(A, W, True, bias=bias)
    ep = fact.Epilogue(bias=bias.cuda(), out_f32=1)
    for ldc in (N, N + 3):                       # 16-byte rows, and rows that only allow element stores
        C = torch.full((M + 1, ldc), float("nan"), dtype=torch.float32, device="cuda")
        fact.binding.check(fact.fact_gemm(M, N, K, A.cuda(), K, W.cuda(), K, 1, C, ldc, ep))
        out = C.cpu().numpy()
        assert np.isnan(out[M]).all() and np.isnan(out[:, N:]).all(), "wrote outside C"
        _assert_f32_close(out[:M, :N].astype(np.float64), r, f"fp32 out direct ldc {ldc}")
    for cfg in cfgs(1):
        C = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
        fact.binding.check(fact.fact_gemm_ex(1, M, N, K, A.cuda(), K, 0, W.cuda(), K, 0, 1, C, N, 0, ep, cfg, 1, 0, None, 0))
        _assert_f32_close(C.cpu().numpy().astype(np.float64), r, f"fp32 out direct cfg {cfg}")
    # batched: two problems, fp32 strides in fp32 elements
    A2 = wl.normal((2, 128, 256), 1.0, "f32d.A2")
    B2 = wl.normal((2, 256, 136), 1.0, "f32d.B2")
    C = torch.full((2, 128, 136), float("nan"), dtype=torch.float32, device="cuda")
    fact.binding.check(fact.fact_gemm_batched(2, 128, 136, 256, A2.cuda(), 256, 128 * 256, B2.cuda(), 136, 256 * 136, 0,
                                              C, 136, 128 * 136, fact.Epilogue(out_f32=1)))
    for b in range(2):
        _assert_f32_close(C[b].cpu().numpy().astype(np.float64), ref.gemm_epilogue(A2[b], B2[b], False), f"fp32 out batch {b}")


def test_fp32_output_refusals():
    A = torch.zeros(64, 4096, dtype=torch.bfloat16, device="cuda")
    B = torch.zeros(4096, 64, dtype=torch.bfloat16, device="cuda")
    C = torch.zeros(64, 64, dtype=torch.float32, device="cuda")
    ep = fact.Epilogue(out_f32=1)
    assert fact.fact_gemm_splitk(64, 64, 4096, A, 4096, B, 64, 0, C, 64, ep, 4, None, 0) == -6       # K split: partial planes need a workspace
    Codd = torch.zeros(64 * 64 + 1, dtype=torch.float32, device="cuda")
    assert fact.fact_gemm(64, 64, 4096, A, 4096, B, 64, 0, Codd.view(torch.uint8)[2:].data_ptr(), 64, ep) == -3   # fp32 C not 4-byte aligned
