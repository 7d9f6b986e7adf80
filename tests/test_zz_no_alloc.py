"""The entry point that allocates nothing (split-K partial sums in the library's static device array),
through the C ABI, against fact_gemm_splitk with a caller's workspace: equal bits, on two calls in
a row, the second with a smaller input (the array keeps the first call's contents)."""
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


def _bits(t):
    torch.cuda.synchronize()
    return wl.bits(t.cpu().contiguous())


def _both(M, N, K, trans_b, split, tag, ep_kw=None, oracle=True):
    A = wl.normal((M, K), 1.0, f"na.A{tag}")
    B = wl.normal((N, K) if trans_b else (K, N), K ** -0.5, f"na.B{tag}")
    bias = wl.normal((N,), 1.0, f"na.b{tag}")
    Ad, Bd, bd = A.cuda(), B.cuda(), bias.cuda()
    ldb = K if trans_b else N
    ep = fact.Epilogue(bias=bd, **(ep_kw or {}))
    need = fact.fact_gemm_splitk_workspace_bytes(M, N, K, split)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda").fill_(0x5A)
    C1 = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    C2 = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    fact.binding.check(fact.fact_gemm_splitk(M, N, K, Ad, K, Bd, ldb, trans_b, C1, N, ep, split, ws, need), "with workspace")
    fact.binding.check(fact.fact_gemm_splitk_static(M, N, K, Ad, K, Bd, ldb, trans_b, C2, N, ep, split), "static")
    b1, b2 = _bits(C1), _bits(C2)
    assert np.array_equal(b1, b2), f"{tag}: static-array result differs from the workspace result"
    if oracle:
        check.assert_close(b2, ref.gemm_epilogue(A, B, bool(trans_b), bias=bias), what=f"no-alloc {tag}")
    return need


def test_static_scratch_matches_workspace_twice_in_a_row_second_call_smaller():
    assert fact.fact_gemm_splitk_static_init() == 0
    cap = fact.fact_gemm_splitk_static_capacity()
    assert cap == 32 << 20
    # first call: 16 K ranges of a 512 x 384 problem; second: a smaller one, other split, other layout,
    # into the array that still holds the first call's partial sums
    n1 = _both(512, 384, 8192, 0, 16, "first")
    n2 = _both(264, 136, 4096, 1, 8, "second")
    assert 0 < n2 < n1 <= cap
    # and once more the first shape: the array now holds the second call's contents
    _both(512, 384, 8192, 0, 16, "first")
    # the table's own choice for the large-K configuration (64 ranges of 256 x 256 x 131072: 16 MiB of partial sums)
    c = wl.config3b()
    M, N, K = 256, 256, 131072
    A, B = c["A"].cuda(), c["B"].cuda()
    need = fact.fact_gemm_splitk_workspace_bytes(M, N, K, 0)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    C1 = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
    C2 = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
    fact.binding.check(fact.fact_gemm_splitk(M, N, K, A, K, B, N, 0, C1, N, None, 0, ws, need))
    fact.binding.check(fact.fact_gemm_splitk_static(M, N, K, A, K, B, N, 0, C2, N, None, 0))
    assert np.array_equal(_bits(C1), _bits(C2))


def test_static_scratch_refuses_what_does_not_fit_and_launches_nothing():
    M, N, K = 2048, 2048, 8192
    A = torch.zeros(M, K, dtype=torch.bfloat16, device="cuda")
    B = torch.zeros(K, N, dtype=torch.bfloat16, device="cuda")
    C = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    assert fact.fact_gemm_splitk_workspace_bytes(M, N, K, 4) > fact.fact_gemm_splitk_static_capacity()
    assert fact.fact_gemm_splitk_static(M, N, K, A, K, B, N, 0, C, N, None, 4) == -6
    assert "static array holds" in fact.fact_last_error()
    torch.cuda.synchronize()
    assert torch.isnan(C).all(), "a refused call wrote to C"
    # split_k = 1 needs no partial sums at all and is served whatever the size
    assert fact.fact_gemm_splitk_static(M, N, K, A, K, B, N, 0, C, N, None, 1) == 0
    torch.cuda.synchronize()
    assert (C == 0).all()
    assert fact.fact_gemm_splitk_static(M, N, K, A, K, B, N, 0, C, N, None, -2) == -7      # as fact_gemm_splitk: no forced tail split here
