"""The on-device sweep under test: a small case, three tile configurations, and the winner's output
held to the CPU oracle (the sweep itself gates on the product's guarded kernel and knows no oracle)."""
import numpy as np
import pytest
import torch

import paper_2604_26666_amd as fact
import workloads as wl
from oracle import check, ref
from paper_2604_26666_amd import registry, sweep, workbench

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    if not torch.cuda.is_available():
        pytest.fail("these tests need the GPU; none is visible")
    fact.lib()


def _case(trans_b, act=fact.ACT_NONE, bias=True):
    M, N, K = 640, 768, 512
    X = wl.normal((M, K), 1.0, "sw.X")
    W = wl.normal((N, K) if trans_b else (K, N), 0.05, "sw.W")
    b = wl.normal((N // 2 if act == fact.ACT_SILU_GATE else N,), 0.05, "sw.b") if bias else None
    c = workbench.Case("sw.case", M, N, K, trans_b, act=act, bias=bias, maker=lambda: {"A": X, "B": W, "bias": b})
    return c, X, W, b


@pytest.mark.parametrize("trans_b,act", [(0, fact.ACT_NONE), (1, fact.ACT_GELU_TANH), (1, fact.ACT_SILU_GATE)])
def test_sweep_picks_a_winner_that_matches_the_oracle(trans_b, act):
    gated = act == fact.ACT_SILU_GATE
    case, X, W, b = _case(trans_b, act, bias=not gated)
    res, fail = sweep.sweep_case(case, steps=5, warmup=3, groups=(2, 8), tails=(), configs=(0, 3, 8))
    assert len(res) == 6 and not fail, (res, fail)                # 3 configurations x 2 groups, nothing refused or rejected
    assert res == sorted(res, key=lambda r: r["ms"])
    best = res[0]
    case.t["C"].fill_(0)
    assert case.run(cfg=best["cfg"], split=best["split"], group_m=best["group_m"]) == 0
    torch.cuda.synchronize()
    r = ref.gemm_epilogue(X, W, bool(trans_b), bias=b, act=act)
    check.assert_close(wl.bits(case.t["C"].cpu()), r, what=f"sweep winner {best}")
    # the entries the sweep would persist: the winner, with provenance, in the registry's format
    ents = sweep.entries_for(case, res)
    assert len(ents) == 1 and (ents[0].config, ents[0].split_k, ents[0].group_m) == (best["cfg"], 1, best["group_m"])
    assert ents[0].gated == int(gated) and ents[0].build == f"v{fact.fact_version()}" and ents[0].tflops > 0
    assert registry.parse(registry.render(ents))[0].line() == ents[0].line()


def test_sweep_gate_rejects_a_wrong_reference_and_records_refusals():
    case, X, W, b = _case(0)
    # a configuration id the library does not have is a recorded launch failure, not an exception
    res, fail = sweep.sweep_case(case, steps=3, warmup=2, groups=(4,), tails=(), configs=(0, 9999))
    assert [r["cfg"] for r in res] == [0] and [f["cfg"] for f in fail] == [9999] and fail[0]["reason"] == "refused"
    # the guarded kernel's reference is what candidates are held to: the same inputs give the oracle's result within tolerance
    rows, ref_dev = sweep.guarded_reference(case)
    assert rows is None                                           # a small case: every row
    r = ref.gemm_epilogue(X, W, False, bias=b)
    check.assert_close(wl.bits(ref_dev.cpu()), r, what="guarded reference")
    # and the gate itself turns down a result that is off by one row
    good = case.t["C"].clone()
    assert sweep._close(good, ref_dev) and not sweep._close(torch.roll(good, 1, 0), ref_dev)


def test_guarded_reference_on_sampled_rows_of_a_large_shape(monkeypatch):
    # the sampling branch, forced on a shape the oracle still covers: blocks of rows, each from its own guarded launch
    monkeypatch.setattr(sweep, "REF_FLOPS_LIMIT", 2.0 * 256 * 384 * 256 * 3)
    M, N, K = 2048 + 24, 384, 256
    X = wl.normal((M, K), 1.0, "swr.X")
    W = wl.normal((N, K), 0.05, "swr.W")
    Rs = wl.normal((M, N), 1.0, "swr.R")
    case = workbench.Case("swr.case", M, N, K, 1, residual=True, maker=lambda: {"A": X, "B": W, "R": Rs})
    rows, out = sweep.guarded_reference(case)
    rows = rows.cpu().numpy()
    assert len(rows) == 3 * 256 and rows[0] == 0 and rows[-1] == M - 1 and len(set(rows.tolist())) == len(rows)
    r = ref.gemm_epilogue(X, W, True, residual=Rs, rows=rows)
    check.assert_close(wl.bits(out.cpu()), r, what="guarded reference, sampled rows")
    res, fail = sweep.sweep_case(case, steps=3, warmup=2, groups=(4,), tails=(), configs=(3,))
    assert len(res) == 1 and not fail
