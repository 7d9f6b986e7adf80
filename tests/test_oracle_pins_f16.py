"""Pins of the oracle's IEEE binary16 ("fp16") path against things other than itself (no GPU).

The fp16 path (the precision of the paper's own kernels: Listing 1, Sections 5.2.3 - 5.2.5) differs
from the bf16 one in three routines only: how a 16-bit pattern is widened, how an fp64 value is
rounded to 16 bits, and which of the two the contraction and the epilogue call.  Each test fails for
a plausible mistake in one of them: a wrong exponent bias or subnormal scale (closed-form values,
numpy's float16 as a library cross-check on all 65536 patterns), a wrong rounding mode, a double
rounding through fp32, a wrong overflow or subnormal boundary (ties, their fp64 neighbours, the
values around 65520 and 2^-25), the bf16 routine called where the fp16 one belongs (values both
formats hold give equal sums; values only fp16 holds give the exact integer sums).
"""
import math
from fractions import Fraction

import numpy as np
import pytest

from oracle import check, ref


def h(x):
    """Python float, exactly representable in binary16 -> bit pattern via numpy's float16."""
    a = np.array(x, dtype=np.float64)
    b = a.astype(np.float16)
    assert (b.astype(np.float64) == a).all(), "test value is not a binary16 number"
    return b.view(np.uint16)


# ---- conversions ----------------------------------------------------------------------------

def test_widen_closed_form_values():
    pats = np.array([0x3C00, 0xBC00, 0x0001, 0x03FF, 0x0400, 0x7BFF, 0x3555, 0x4248, 0x0000, 0x8000, 0x7C00, 0xFC00], dtype=np.uint16)
    want = [1.0, -1.0, 2.0 ** -24, 1023 * 2.0 ** -24, 2.0 ** -14, 65504.0, (1024 + 0x155) * 2.0 ** -12, (1024 + 0x248) * 2.0 ** -9,
            0.0, -0.0, math.inf, -math.inf]
    got = ref.widen(pats, "f16")
    assert (got == np.array(want)).all()
    assert np.signbit(got[9]) and not np.signbit(got[8])
    assert np.isnan(ref.widen(np.array([0x7E00, 0x7C01, 0xFFFF], dtype=np.uint16), "f16")).all()


def test_widen_matches_numpy_for_all_patterns():
    allb = np.arange(65536, dtype=np.uint16)
    ours = ref.widen(allb, "f16")
    theirs = allb.view(np.float16).astype(np.float64)
    assert ((ours == theirs) | (np.isnan(ours) & np.isnan(theirs))).all()
    assert (np.signbit(ours) == np.signbit(theirs))[~np.isnan(ours)].all()


def test_widen_differs_from_the_bf16_reading():
    # the same pattern read as bf16 is another number: a mix-up of the two cannot pass
    assert ref.widen(np.array([0x3C00], dtype=np.uint16), "bf16")[0] == 2.0 ** -7
    assert ref.widen(np.array([0x3F80], dtype=np.uint16), "f16")[0] == 1.875


def test_round_trip_is_identity_on_all_patterns():
    allb = np.arange(65536, dtype=np.uint16)
    v = ref.widen(allb, "f16")
    back = ref.round_f16(v)
    nan = np.isnan(v)
    assert (back[~nan] == allb[~nan]).all()
    assert (back[nan] == 0x7E00).all()


def test_round_ties_go_to_even_and_neighbours_to_the_nearer_value():
    lo = np.arange(0x0000, 0x7BFF, dtype=np.uint16)           # every positive finite value but the largest
    a, b = ref.widen(lo, "f16"), ref.widen(lo + 1, "f16")
    mid = (a + b) / 2                                          # exact in fp64
    even = np.where(lo & 1, lo + 1, lo)
    assert (ref.round_f16(mid) == even).all()
    assert (ref.round_f16(-mid) == (even | 0x8000)).all()
    assert (ref.round_f16(np.nextafter(mid, np.inf)) == lo + 1).all()
    assert (ref.round_f16(np.nextafter(mid, -np.inf)) == lo).all()


def test_round_is_a_single_rounding():
    # just above the midpoint of 1 and 1 + 2^-10: through fp32 it would first become the midpoint
    # itself (the 2^-40 is lost), then tie to even = 1.0
    x = 1.0 + 2.0 ** -11 + 2.0 ** -40
    assert np.float64(np.float32(x)) == 1.0 + 2.0 ** -11
    assert int(ref.round_f16(np.array([x]))[0]) == 0x3C01
    assert int(ref.round_f16(np.array([1.0 + 2.0 ** -11]))[0]) == 0x3C00
    assert int(ref.round_f16(np.array([1.0 + 3 * 2.0 ** -11]))[0]) == 0x3C02


def test_round_overflow_and_subnormal_boundaries():
    r = lambda x: int(ref.round_f16(np.array([x], dtype=np.float64))[0])
    assert r(65504.0) == 0x7BFF
    assert r(65519.999) == 0x7BFF
    assert r(65520.0) == 0x7C00                 # the tie between 65504 and 2^16 goes to the even side: infinity
    assert r(-65520.0) == 0xFC00
    assert r(1e300) == 0x7C00 and r(math.inf) == 0x7C00
    assert r(2.0 ** -24) == 0x0001
    assert r(2.0 ** -25) == 0x0000              # tie between 0 and the smallest subnormal: even = 0
    assert r(-(2.0 ** -25)) == 0x8000
    assert r(np.nextafter(2.0 ** -25, 1.0)) == 0x0001
    assert r(3 * 2.0 ** -25) == 0x0002          # tie between 1 and 2 quanta
    assert r(1023.5 * 2.0 ** -24) == 0x0400     # largest subnormal's upper tie rounds into the smallest normal
    assert r(1023.4999 * 2.0 ** -24) == 0x03FF
    assert r(2.0 ** -14) == 0x0400
    assert r(1e-300) == 0x0000 and r(-1e-300) == 0x8000
    assert r(math.nan) == 0x7E00


def test_round_matches_numpy_on_random_fp64_inputs():
    g = np.random.default_rng(11)
    x = g.standard_normal(300000)
    x = np.concatenate([x, x * 1e-4, x * 1e-6, x * 3e-8, x * 1e3, x * 3e4, x * 7e4])
    with np.errstate(over="ignore"):
        theirs = x.astype(np.float16).view(np.uint16)        # numpy rounds fp64 -> binary16 directly
    assert (ref.round_f16(x) == theirs).all()


# ---- the contraction ------------------------------------------------------------------------

def test_identity_and_permutation_in_both_layouts():
    g = np.random.default_rng(3)
    n = 48
    X = g.standard_normal((n, n)).astype(np.float16).view(np.uint16)
    I = h(np.eye(n))
    perm = g.permutation(n)
    P = h(np.eye(n)[perm])
    xv = ref.widen(X, "f16")
    acc, bound = ref.gemm(I, X, False, fmt="f16")
    assert (acc == xv).all() and (bound == np.abs(xv)).all()
    acc, _ = ref.gemm(P, X, False, fmt="f16")
    assert (acc == xv[perm]).all()
    acc, _ = ref.gemm(X, P, False, fmt="f16")                  # X P: column j of the result is column k of X where P[k][j] = 1
    assert (acc == xv @ np.eye(n)[perm]).all()
    acc, _ = ref.gemm(X, P, True, fmt="f16")                   # X P^T
    assert (acc == xv @ np.eye(n)[perm].T).all()


def test_exact_integers_against_int64_matmul_with_values_only_fp16_holds():
    # odd integers up to 2047 need 11 significant bits: bf16 (8 bits) cannot hold them, binary16 can
    g = np.random.default_rng(5)
    M, N, K = 37, 29, 301
    Ai = g.integers(-2047, 2048, size=(M, K))
    Bi = g.integers(-2047, 2048, size=(K, N))
    A, B = h(Ai.astype(np.float64)), h(Bi.astype(np.float64))
    want = Ai.astype(np.int64) @ Bi.astype(np.int64)
    acc, bound = ref.gemm(A, B, False, fmt="f16")
    assert (acc == want).all()
    assert (bound == np.abs(Ai).astype(np.int64) @ np.abs(Bi).astype(np.int64)).all()
    acc_t, _ = ref.gemm(A, np.ascontiguousarray(B.T), True, fmt="f16")
    assert (acc_t == want).all()
    rows = [36, 0, 17, 17]
    acc_r, _ = ref.gemm(A, B, False, rows=rows, fmt="f16")
    assert (acc_r == want[rows]).all()


def test_values_both_formats_hold_give_the_same_sums():
    g = np.random.default_rng(9)
    M, N, K = 16, 24, 130
    vals = g.integers(-15, 16, size=(M, K)) * 2.0 ** g.integers(-6, 5, size=(M, K))       # <= 4 significant bits
    wts = g.integers(-15, 16, size=(N, K)) * 2.0 ** g.integers(-6, 5, size=(N, K))
    import torch
    Ab = torch.tensor(vals, dtype=torch.float64).to(torch.bfloat16)
    Bb = torch.tensor(wts, dtype=torch.float64).to(torch.bfloat16)
    assert (Ab.to(torch.float64).numpy() == vals).all()
    a16, _ = ref.gemm(h(vals), h(wts), True, fmt="f16")
    ab, _ = ref.gemm(Ab, Bb, True, fmt="bf16")
    assert (a16 == ab).all()
    assert (a16 == vals @ wts.T).all()          # every partial sum is a multiple of 2^-12 below 2^20: exact in fp64


def test_exact_rationals_on_a_tiny_shape_with_subnormal_operands():
    g = np.random.default_rng(13)
    M, N, K = 3, 4, 7
    A = g.integers(0, 65536, size=(M, K)).astype(np.uint16)
    B = g.integers(0, 65536, size=(K, N)).astype(np.uint16)
    A[(A & 0x7C00) == 0x7C00] = 0x0203          # no infinities or NaNs; a subnormal instead
    B[(B & 0x7C00) == 0x7C00] = 0x8001
    A[0, 0], B[0, 0] = 0x0001, 0x03FF
    av, bv = A.view(np.float16).astype(np.float64), B.view(np.float16).astype(np.float64)
    acc, _ = ref.gemm(A, B, False, fmt="f16")
    for i in range(M):
        for j in range(N):
            exact = sum(Fraction(av[i, k]) * Fraction(bv[k, j]) for k in range(K))
            assert abs(Fraction(acc[i, j]) - exact) <= abs(exact) * Fraction(1, 2 ** 49) + Fraction(1, 2 ** 120)
    assert acc[0, 0] != 0.0


def test_long_k_against_fsum():
    g = np.random.default_rng(17)
    K = 20000
    a = g.standard_normal((1, K)).astype(np.float16)
    b = g.standard_normal((1, K)).astype(np.float16)
    acc, bound = ref.gemm(a.view(np.uint16), b.view(np.uint16), True, fmt="f16")
    prods = [float(x) * float(y) for x, y in zip(a[0].astype(np.float64), b[0].astype(np.float64))]   # each exact
    assert abs(acc[0, 0] - math.fsum(prods)) <= K * 2.0 ** -53 * math.fsum(abs(p) for p in prods)
    assert abs(bound[0, 0] - math.fsum(abs(p) for p in prods)) <= K * 2.0 ** -53 * bound[0, 0]


# ---- the epilogue in fp16 -------------------------------------------------------------------

def test_epilogue_wiring_and_single_rounding_at_k_1():
    # K = 1: acc = a b exactly.  z = acc + bias, then + residual, then ONE rounding to binary16.
    A = h(np.array([[1.0], [3.0]]))
    B = h(np.array([[1.0, 0.5]]))
    bias = h(np.array([2.0 ** -11, 0.0]))
    R = h(np.array([[2.0 ** -22, 1.0], [0.0, 2.0 ** -11]]))
    r = ref.gemm_epilogue(A, B, False, bias=bias, residual=R, fmt="f16")
    want_z = np.array([[1.0 + 2.0 ** -11 + 2.0 ** -22, 0.5 + 1.0], [3.0 + 2.0 ** -11, 1.5 + 2.0 ** -11]])
    assert (r.z == want_z).all() and r.fmt == "f16"
    # 1 + 2^-11 + 2^-22 is above the tie -> up; 3 + 2^-11 is below the tie of spacing 2^-9 -> down;
    # 1.5 + 2^-11 is the tie between 1.5 and 1.5 + 2^-10 -> even (1.5 = 0x3E00)
    assert [int(x) for x in r.bits.ravel()] == [0x3C01, 0x3E00, 0x4200, 0x3E00]
    assert (r.bound == np.array([[1.0 + 2.0 ** -11 + 2.0 ** -22, 1.5], [3.0 + 2.0 ** -11, 1.5 + 2.0 ** -11]])).all()


def test_epilogue_order_bias_before_and_residual_after_the_activation():
    A = h(np.array([[1.0]]))
    B = h(np.array([[0.5]]))
    bias = h(np.array([0.25]))
    R = h(np.array([[4.0]]))
    r = ref.gemm_epilogue(A, B, True, bias=bias, residual=R, act=ref.ACT_GELU_TANH, fmt="f16")
    z = 0.75
    want = 0.5 * z * (1.0 + math.tanh(math.sqrt(2.0 / math.pi) * (z + 0.044715 * z ** 3))) + 4.0
    assert abs(r.z[0, 0] - want) < 1e-15
    assert int(r.bits[0, 0]) == int(np.array([want]).astype(np.float16).view(np.uint16)[0])


def test_gated_epilogue_in_fp16_and_row_subset():
    g = np.random.default_rng(23)
    M, I, K = 9, 6, 20
    X = g.standard_normal((M, K)).astype(np.float16).view(np.uint16)
    W = g.standard_normal((2 * I, K)).astype(np.float16).view(np.uint16)
    Rm = g.standard_normal((M, I)).astype(np.float16).view(np.uint16)
    full = ref.gemm_epilogue(X, W, True, residual=Rm, act=ref.ACT_SILU_GATE, fmt="f16")
    xv, wv = X.view(np.float16).astype(np.float64), W.view(np.float16).astype(np.float64)
    gv, uv = xv @ wv[:I].T, xv @ wv[I:].T
    want = gv / (1.0 + np.exp(-gv)) * uv + Rm.view(np.float16).astype(np.float64)
    assert np.allclose(full.z, want, rtol=1e-13, atol=1e-13)
    rows = [8, 2, 2, 0]
    sub = ref.gemm_epilogue(X, W, True, residual=Rm, act=ref.ACT_SILU_GATE, rows=rows, fmt="f16")
    assert (sub.z == full.z[rows]).all() and (sub.bits == full.bits[rows]).all() and (sub.rows == np.array(rows)).all()


def test_check_uses_the_format_of_the_reference():
    A = h(np.array([[1.0, 2.0], [3.0, 4.0]]))
    B = h(np.array([[1.0, 0.0], [0.0, 1.0]]))
    r = ref.gemm_epilogue(A, B, False, fmt="f16")
    assert check.compare(r.bits, r)["ok"] and check.compare(r.bits, r)["max_abs_err"] == 0.0
    check.assert_bits_equal(r.bits, r)
    wrong = r.bits.copy()
    wrong[1, 0] = 0x4400                          # 4.0 where 3.0 belongs
    assert not check.compare(wrong, r)["ok"]
    with pytest.raises(AssertionError):
        check.assert_bits_equal(wrong, r)
    # the same bits read as bf16 would be tiny numbers: the comparison must not do that
    assert check.compare(r.bits, r)["bits_equal_frac"] == 1.0
    # one binary16 ulp off at 1.0 passes the element criterion (atol) and is reported as 1 ulp
    near = r.bits.copy()
    near[0, 0] = 0x3C01
    s = check.compare(near, r)
    assert abs(s["max_err_ulp"] - 1.0) < 1e-12


# ---- the two-GEMM block in fp16 ---------------------------------------------------------------

def test_block_mlp_stores_h_in_binary16_between_the_two_gemms():
    # X W1^T = 1 + 2^-10 and 1 + 2^-11 + 2^-13: the first is a binary16 number (bf16 would make it 1),
    # the second rounds to 1 + 2^-10 in binary16 (above the tie); Y = 4 H + R shows which H was used
    X = h(np.array([[1.0, 2.0 ** -10], [1.0, 2.0 ** -11 + 2.0 ** -13]]))
    W1 = h(np.array([[1.0, 1.0]]))
    W2 = h(np.array([[4.0], [0.5]]))
    R = h(np.array([[0.0, 1.0], [2.0, 0.0]]))
    rh, ry = ref.block_mlp(X, W1, None, None, ref.ACT_NONE, W2, None, R, fmt="f16")
    assert [int(b) for b in rh.bits.ravel()] == [0x3C01, 0x3C01] and rh.fmt == "f16" and ry.fmt == "f16"
    hv = 1.0 + 2.0 ** -10
    assert (ry.z == np.array([[4 * hv, 0.5 * hv + 1.0], [4 * hv + 2.0, 0.5 * hv]])).all()
    # rows: the second stage follows the first stage's row subset, the residual too
    rh1, ry1 = ref.block_mlp(X, W1, None, None, ref.ACT_NONE, W2, None, R, rows=[1], fmt="f16")
    assert (ry1.z == ry.z[[1]]).all() and (ry1.bits == ry.bits[[1]]).all() and (rh1.bits == rh.bits[[1]]).all()


def test_block_mlp_fp16_against_a_numpy_composition():
    g = np.random.default_rng(29)
    T, d, dff = 12, 16, 40
    f16 = lambda a: a.astype(np.float16)
    X, W1, W1u, W2 = f16(g.standard_normal((T, d))), f16(g.standard_normal((dff, d)) * 0.3), f16(g.standard_normal((dff, d)) * 0.3), f16(g.standard_normal((d, dff)) * 0.3)
    b1, b2, R = f16(g.standard_normal(dff) * 0.1), f16(g.standard_normal(d) * 0.1), f16(g.standard_normal((T, d)))
    u = lambda a: a.view(np.uint16)
    d64 = lambda a: a.astype(np.float64)
    # GELU block with biases and residual
    rh, ry = ref.block_mlp(u(X), u(W1), None, u(b1), ref.ACT_GELU_TANH, u(W2), u(b2), u(R), fmt="f16")
    z1 = d64(X) @ d64(W1).T + d64(b1)
    hz = 0.5 * z1 * (1.0 + np.tanh(np.sqrt(2.0 / np.pi) * (z1 + 0.044715 * z1 ** 3)))
    assert np.allclose(rh.z, hz, rtol=1e-13, atol=1e-14)
    H = d64(rh.z.astype(np.float16))                      # numpy's own fp64 -> binary16 rounding of the oracle's H
    assert (u(rh.z.astype(np.float16)) == rh.bits).all()
    assert np.allclose(ry.z, H @ d64(W2).T + d64(b2) + d64(R), rtol=1e-13, atol=1e-13)
    # gated block
    rh, ry = ref.block_mlp(u(X), u(W1), u(W1u), None, ref.ACT_SILU_GATE, u(W2), None, None, fmt="f16")
    gz, uz = d64(X) @ d64(W1).T, d64(X) @ d64(W1u).T
    assert np.allclose(rh.z, gz / (1.0 + np.exp(-gz)) * uz, rtol=1e-13, atol=1e-14)
    assert np.allclose(ry.z, d64(rh.z.astype(np.float16)) @ d64(W2).T, rtol=1e-13, atol=1e-13)
