"""GPU parity of persistent launches: a work-group walks several tiles, and the first operand stages of
its next tile are requested before the epilogue of the tile in hand runs.

Every case has more tiles than the GPU holds work-groups at once (checked through
fact_persistent_grid, so that no case silently runs the ordinary launch), several rounds and a ragged
last one, and edge tiles next to interior ones, so that one work-group mixes the register epilogue
(with the next tile's loads in flight) and the LDS-staged one.  Exact integer inputs must give the
oracle's bits in every 4-wave configuration; every other epilogue must give the bits of the ordinary
launch of the same problem (which the other parity tests hold to the oracle).
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
    fact.lib()
    before = fact.fact_tune_persistent(1)          # (off by default)
    yield
    fact.fact_tune_persistent(before)


def G():
    import gpu_util
    return gpu_util


def four_wave_configs(trans_b):
    out = []
    for c in range(fact.fact_num_configs()):
        bm, bn, wm, wn = fact.fact_config_info(c)[:4]
        if wm * wn <= 4 and (trans_b or 64 % (bn // 8) == 0):
            out.append(c)
    return out


def shape_for(cfg, gated=False):
    """More than two rounds of tiles plus a ragged one, a ragged last tile row and column."""
    bm, bn, wm, wn, lds = fact.fact_config_info(cfg)[:5]
    bn_out = bn // 2 if gated else bn
    occ = 2 if lds <= 80 * 1024 else 1
    need = 256 * occ * 2 + 37
    tiles_m = 9 if bm >= 128 else 17
    tiles_n = -(-need // tiles_m)
    return tiles_m * bm - 8, tiles_n * bn_out - 8          # output rows, output columns


@pytest.mark.parametrize("trans_b", [0, 1])
def test_integers_bit_exact_in_every_four_wave_config(trans_b):
    K = 192
    for cfg in four_wave_configs(trans_b):
        M, N = shape_for(cfg)
        assert fact.fact_persistent_grid(1, M, N, K, trans_b, fact.ACT_NONE, cfg) > 0, f"cfg {cfg}: not a persistent launch"
        A = wl.small_int((M, K), -2, 2, f"ps.A{cfg}")
        B = wl.small_int((K, N), -2, 2, f"ps.B{cfg}")
        Bs = B if not trans_b else B.t().contiguous()
        bias = wl.small_int((N,), -3, 3, "ps.bias")
        res = wl.small_int((M, N), -3, 3, f"ps.res{cfg}")
        r = ref.gemm_epilogue(A, Bs, bool(trans_b), bias=bias, residual=res)
        got = G().gemm(A, Bs, trans_b, bias=bias, residual=res, cfg=cfg, split=1)
        check.assert_bits_equal(got, r, what=f"persistent cfg {cfg} tb {trans_b} {M}x{N}x{K}")


def _both_modes(run):
    fact.fact_tune_persistent(1)
    a = run()
    fact.fact_tune_persistent(0)
    try:
        b = run()
    finally:
        fact.fact_tune_persistent(1)
    return a, b


@pytest.mark.parametrize("kind", ["plain", "gelu", "gelu_res", "gated", "gated_res", "f32"])
def test_same_bits_as_the_ordinary_launch(kind):
    K = 328                                            # a partial last K step
    gated = kind.startswith("gated")
    act = fact.ACT_SILU_GATE if gated else fact.ACT_GELU_TANH if kind.startswith("gelu") else fact.ACT_NONE
    for cfg in (0, 3, 13, 14):
        M, Nout = shape_for(cfg, gated)
        Ncontr = 2 * Nout if gated else Nout
        assert fact.fact_persistent_grid(1, M, Ncontr, K, 1, act, cfg) > 0
        X = wl.normal((M, K), 1.0, f"pm.X{cfg}{kind}")
        W = wl.normal((Ncontr, K), 0.05, f"pm.W{cfg}{kind}")
        bias = None if gated or kind == "plain" else wl.normal((Nout,), 1.0, "pm.bias")
        res = wl.normal((M, Nout), 1.0, f"pm.R{cfg}{kind}") if kind.endswith("res") else None
        if kind == "f32":
            from test_gpu_parity import _f32_call
            a, b = _both_modes(lambda: _f32_call(X, W, 1, 1, bias=bias, cfg=cfg))
        else:
            a, b = _both_modes(lambda: G().gemm(X, W, 1, bias=bias, residual=res, act=act, cfg=cfg, split=1))
        assert np.array_equal(a, b), f"{kind} cfg {cfg}: {int((a != b).sum())} elements differ"
    # and the persistent result against the oracle on a sample of rows, for the last configuration
    rows = np.unique(np.r_[np.arange(0, M, 97), M - 1])
    if kind != "f32":
        r = ref.gemm_epilogue(X, W, True, bias=bias, residual=res, act=act, rows=rows)
        check.assert_close(a[rows], r, what=f"persistent {kind}")


def test_batched_persistent_launch():
    # 6 batch entries x 100 tiles of 128 x 128 > 512 resident work-groups; distinct operands per entry
    cfg, batch, M, N, K = 3, 6, 10 * 128 - 8, 10 * 128, 136
    assert fact.fact_persistent_grid(batch, M, N, K, 0, fact.ACT_NONE, cfg) > 0
    A = wl.small_int((batch, M, K), -2, 2, "pb.A")
    B = wl.small_int((batch, K, N), -2, 2, "pb.B")
    C = G().poisoned(batch * M, N).view(batch, M, N)
    ep = fact.Epilogue()
    fact.binding.check(fact.fact_gemm_ex(batch, M, N, K, A.cuda(), K, M * K, B.cuda(), N, K * N, 0, C, N, M * N, ep, cfg, 1, 4, None, 0))
    out = G().bits_of(C)
    for b in range(batch):
        check.assert_bits_equal(out[b], ref.gemm_epilogue(A[b], B[b], False), what=f"batch entry {b}")
