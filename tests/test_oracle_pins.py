"""Pins of the CPU oracle against things other than itself (no GPU).

Each test fails for a plausible mistake in the oracle: a wrong index or
transposed operand (identity / permutation / padded-ld tests), a wrong rounding
mode or a double rounding (K = 1 ties), a dropped or repeated term (exact
integer products against int64 matmul, exact rationals, all-ones closed forms),
a wrong activation formula or epilogue order (closed-form points, odd-part
identities, library cross-checks, K = 1 wiring cases).
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import check, ref

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def bf(x):
    """Python float (exactly representable in bf16) -> bit pattern via torch's conversion."""
    t = torch.tensor(x, dtype=torch.float64)
    b = t.to(torch.bfloat16)
    assert (b.to(torch.float64) == t).all(), "test value is not a bf16 number"
    return wl.bits(b)


# ---- bf16 conversions ---------------------------------------------------------

def test_widen_matches_torch_for_all_patterns():
    allb = np.arange(65536, dtype=np.uint16)
    ours = ref.widen(allb)
    theirs = wl.from_bits(allb).to(torch.float64).numpy()
    same = (ours == theirs) | (np.isnan(ours) & np.isnan(theirs))
    assert same.all()
    assert (np.signbit(ours) == np.signbit(theirs))[~np.isnan(ours)].all()


def test_round_trip_is_identity_on_all_patterns():
    allb = np.arange(65536, dtype=np.uint16)
    v = ref.widen(allb)
    back = ref.round_bf16(v)
    nan = np.isnan(v)
    assert (back[~nan] == allb[~nan]).all()
    assert (back[nan] == 0x7FC0).all()


def test_round_matches_torch_on_fp32_inputs():
    g = torch.Generator().manual_seed(7)
    x = torch.randn(200000, generator=g, dtype=torch.float32)
    x = torch.cat([x, x * 1e-38, x * 1e-40, x * 1e30, x * 3e38])
    # every midpoint between adjacent positive bf16 numbers, and its fp32 neighbours
    hi = torch.arange(0x0001, 0x7F7F, dtype=torch.int32)
    mid = ((hi << 16) | 0x8000).view(torch.float32)
    x = torch.cat([x, mid, -mid, ((hi << 16) | 0x8001).view(torch.float32),
                   ((hi << 16) | 0x7FFF).view(torch.float32)])
    want = wl.bits(x.to(torch.bfloat16))
    got = ref.round_bf16(x.to(torch.float64).numpy())
    assert (got == want).all()


def test_round_ties_to_even_by_hand():
    # 1 + 2^-8 is halfway between 1 and 1 + 2^-7: even neighbour is 1.0 (0x3F80)
    assert ref.lib().orc_bf16_from_f64(1.0 + 2.0 ** -8) == 0x3F80
    # 1 + 3*2^-8 is halfway between 1+2^-7 (odd) and 1+2^-6 (even) -> up
    assert ref.lib().orc_bf16_from_f64(1.0 + 3 * 2.0 ** -8) == 0x3F82
    # not a tie
    assert ref.lib().orc_bf16_from_f64(1.0 + 2.0 ** -8 + 2.0 ** -20) == 0x3F81
    assert ref.lib().orc_bf16_from_f64(-(1.0 + 2.0 ** -8)) == 0xBF80


def test_round_is_a_single_rounding_from_fp64():
    # Just above a tie by less than fp32 can hold: rounding to fp32 first would
    # land exactly on the tie and then go to even (1.0); one rounding goes up.
    x = 1.0 + 2.0 ** -8 + 2.0 ** -40
    assert float(np.float32(x)) == 1.0 + 2.0 ** -8
    assert ref.lib().orc_bf16_from_f64(x) == 0x3F81


def test_round_specials():
    L = ref.lib()
    assert L.orc_bf16_from_f64(0.0) == 0x0000
    assert L.orc_bf16_from_f64(-0.0) == 0x8000
    assert L.orc_bf16_from_f64(float("inf")) == 0x7F80
    assert L.orc_bf16_from_f64(float("-inf")) == 0xFF80
    assert L.orc_bf16_from_f64(float("nan")) == 0x7FC0
    big = float.fromhex("0x1.fep127")            # largest bf16
    assert L.orc_bf16_from_f64(big) == 0x7F7F
    assert L.orc_bf16_from_f64(float.fromhex("0x1.ffp127")) == 0x7F80   # tie at the top -> inf
    assert L.orc_bf16_from_f64(float.fromhex("0x1.fefp127")) == 0x7F7F
    assert L.orc_bf16_from_f64(2.0 ** -133) == 0x0001                    # smallest subnormal
    assert L.orc_bf16_from_f64(2.0 ** -134) == 0x0000                    # tie -> even (zero)
    assert L.orc_bf16_from_f64(2.0 ** -134 * 1.5) == 0x0001
    assert L.orc_bf16_from_f64(2.0 ** -126) == 0x0080                    # smallest normal


# ---- indexing, layouts, leading dimensions ------------------------------------

@pytest.mark.parametrize("trans_b", [False, True])
def test_identity_and_permutation(trans_b):
    n, m = 48, 37
    X = wl.uniform((n, m), "pin.X")              # generic data
    eye = torch.eye(n, dtype=torch.bfloat16)
    # A = I  ->  C = B
    Bmat = X if not trans_b else X.t().contiguous()           # logical B is [n, m]
    acc, _ = ref.gemm(eye, Bmat, trans_b)
    assert (ref.round_bf16(acc) == wl.bits(X)).all()
    # A = P (row permutation) -> C rows are permuted rows of B
    p = wl.permutation(n, "pin.perm")
    P = eye[p]
    acc, _ = ref.gemm(P, Bmat, trans_b)
    assert (ref.round_bf16(acc) == wl.bits(X[p].contiguous())).all()
    # B = I -> C = A  (A is [m, n])
    A = X.t().contiguous()
    acc, _ = ref.gemm(A, eye, trans_b)
    assert (ref.round_bf16(acc) == wl.bits(A)).all()
    # B = column permutation: (A Q)[i][j] = A[i][q[j]] where Q[k][j] = 1 iff k == q[j]
    q = wl.permutation(n, "pin.perm2")
    Q = torch.zeros(n, n, dtype=torch.bfloat16)
    Q[q, torch.arange(n)] = 1
    acc, _ = ref.gemm(A, Q if not trans_b else Q.t().contiguous(), trans_b)
    assert (ref.round_bf16(acc) == wl.bits(A[:, q].contiguous())).all()


@pytest.mark.parametrize("trans_b", [False, True])
def test_leading_dimension_padding_is_ignored(trans_b):
    M, N, K = 9, 11, 13
    A = wl.small_int((M, K), -3, 3, "ld.A")
    B = wl.small_int((K, N), -3, 3, "ld.B")
    Bs = B if not trans_b else B.t().contiguous()
    base, _ = ref.gemm(A, Bs, trans_b)
    # same data inside wider buffers whose padding is poisoned with NaN patterns
    Ap = np.full((M, K + 5), 0x7FC0, dtype=np.uint16)
    Ap[:, :K] = wl.bits(A)
    Bp = np.full((Bs.shape[0], Bs.shape[1] + 3), 0x7FC0, dtype=np.uint16)
    Bp[:, : Bs.shape[1]] = wl.bits(Bs)
    acc, bound = ref.gemm(Ap[:, :K], Bp[:, : Bs.shape[1]], trans_b)
    assert np.array_equal(acc, base) and np.isfinite(bound).all()


def test_row_subset_equals_full_rows():
    A = wl.uniform((33, 20), "rs.A")
    B = wl.uniform((20, 17), "rs.B")
    full, fb = ref.gemm(A, B)
    rows = [32, 0, 7, 7, 15]
    sub, sb = ref.gemm(A, B, rows=rows)
    assert np.array_equal(sub, full[rows]) and np.array_equal(sb, fb[rows])


# ---- rounding at the store: K = 1 outer products on ties -----------------------

def test_k1_outer_product_ties():
    # products of two bf16 numbers are exact in fp32/fp64; only the final rounding acts
    a = [1.0078125, 1.0234375, 1.0078125, -1.0078125]
    b = [1.5, 1.25]
    A = bf(a).reshape(4, 1)
    B = bf(b).reshape(1, 2)
    r = ref.gemm_epilogue(A, B)
    want = np.array([
        [1.515625, 1.2578125],      # 1.51171875 tie -> even above;   1.259765625 -> nearest
        [1.53125, 1.28125],         # 1.53515625 tie -> even below;   1.279296875 -> nearest
        [1.515625, 1.2578125],
        [-1.515625, -1.2578125],
    ])
    assert np.array_equal(ref.widen(r.bits), want)
    assert r.z[0, 0] == 1.51171875 and r.z[1, 0] == 1.53515625     # un-rounded values kept


# ---- no dropped / repeated terms ------------------------------------------------

@pytest.mark.parametrize("trans_b", [False, True])
@pytest.mark.parametrize("shape", [(5, 7, 3), (64, 48, 200), (17, 130, 1031)])
def test_small_integers_match_int64_matmul(shape, trans_b):
    M, N, K = shape
    A = wl.small_int((M, K), -4, 4, f"int.A{shape}")
    B = wl.small_int((K, N), -4, 4, f"int.B{shape}")
    Ai = A.to(torch.int64).numpy()
    Bi = B.to(torch.int64).numpy()
    Bs = B if not trans_b else B.t().contiguous()
    acc, bound = ref.gemm(A, Bs, trans_b)
    assert np.array_equal(acc, (Ai @ Bi).astype(np.float64))
    assert np.array_equal(bound, (np.abs(Ai) @ np.abs(Bi)).astype(np.float64))


def test_all_ones_closed_forms():
    for K in (1, 3, 256, 1024, 4096):
        A = torch.ones(4, K, dtype=torch.bfloat16)
        B = torch.ones(K, 6, dtype=torch.bfloat16)
        acc, bound = ref.gemm(A, B)
        assert (acc == K).all() and (bound == K).all()
    K = 300
    A = torch.ones(3, K, dtype=torch.bfloat16)
    j = torch.arange(9)
    B = ((j % 3) - 1).to(torch.bfloat16).repeat(K, 1)
    acc, _ = ref.gemm(A, B)
    assert np.array_equal(acc, np.tile(K * ((np.arange(9) % 3) - 1.0), (3, 1)))


@pytest.mark.parametrize("trans_b", [False, True])
def test_tiny_shapes_against_exact_rationals(trans_b):
    for M in (1, 2, 3, 5):
        for N in (1, 2, 5):
            for K in (1, 2, 3, 5):
                A = wl.uniform((M, K), f"fr.A{M}{N}{K}")
                B = wl.uniform((K, N), f"fr.B{M}{N}{K}")
                a = A.to(torch.float64).tolist()
                b = B.to(torch.float64).tolist()
                Bs = B if not trans_b else B.t().contiguous()
                acc, bound = ref.gemm(A, Bs, trans_b)
                for i in range(M):
                    for jn in range(N):
                        exact = sum(Fraction(a[i][k]) * Fraction(b[k][jn]) for k in range(K))
                        exact_abs = sum(abs(Fraction(a[i][k]) * Fraction(b[k][jn])) for k in range(K))
                        assert abs(Fraction(acc[i, jn]) - exact) <= Fraction(2) ** -50 * max(exact_abs, Fraction(1, 10**9))
                        assert abs(Fraction(bound[i, jn]) - exact_abs) <= Fraction(2) ** -50 * exact_abs


def test_fp64_accumulation_is_adequate_on_long_k():
    M, N, K = 4, 4, 40000
    A = wl.normal((M, K), 1.0, "fs.A")
    B = wl.normal((K, N), 1.0, "fs.B")
    a = A.to(torch.float64).numpy()
    b = B.to(torch.float64).numpy()
    acc, bound = ref.gemm(A, B)
    for i in range(M):
        for j in range(N):
            exact = math.fsum((a[i] * b[:, j]).tolist())      # products exact, sum exactly rounded
            assert abs(acc[i, j] - exact) <= 2.0 ** -40 * bound[i, j]


# ---- activations ------------------------------------------------------------------

def _golden_points():
    pts = {"gelu_tanh": [], "silu": []}
    with open(os.path.join(GOLDEN, "activation_points.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, z, v = line.split()
            pts[name].append((float(z), float(v)))
    return pts


def test_activation_closed_form_points():
    pts = _golden_points()
    assert len(pts["gelu_tanh"]) >= 10 and len(pts["silu"]) >= 10
    # 1 + tanh(t) cancels for t << 0, so fp64 evaluation of the formula carries an
    # absolute error of about 1e-16 |z|; twelve orders below the 1e-3 tolerance floor
    for z, v in pts["gelu_tanh"]:
        assert ref.gelu_tanh(z) == pytest.approx(v, rel=1e-13, abs=2e-15)
    for z, v in pts["silu"]:
        assert ref.silu(z) == pytest.approx(v, rel=1e-13, abs=2e-15)


def test_activation_identities_and_limits():
    z = np.linspace(-12, 12, 4801)
    # tanh and the logistic's odd part: f(z) - f(-z) = z for both activations
    assert np.allclose(ref.gelu_tanh(z) - ref.gelu_tanh(-z), z, rtol=0, atol=1e-14)
    assert np.allclose(ref.silu(z) - ref.silu(-z), z, rtol=0, atol=1e-14)
    assert ref.gelu_tanh(0.0) == 0.0 and ref.silu(0.0) == 0.0
    assert ref.gelu_tanh(30.0) == 30.0 and abs(ref.gelu_tanh(-30.0)) == 0.0
    assert ref.silu(50.0) == pytest.approx(50.0, rel=1e-15) and abs(ref.silu(-800.0)) == 0.0
    # it is the tanh form, not the erf form: they differ by about 4e-4 at z = -3
    erf_form = 0.5 * -3.0 * (1 + math.erf(-3.0 / math.sqrt(2)))
    assert abs(ref.gelu_tanh(-3.0) - erf_form) > 3e-4


def test_activations_match_library_routines():
    z = torch.linspace(-9, 9, 3001, dtype=torch.float64)
    want_g = torch.nn.functional.gelu(z, approximate="tanh").numpy()
    want_s = torch.nn.functional.silu(z).numpy()
    assert np.allclose(ref.gelu_tanh(z.numpy()), want_g, rtol=1e-13, atol=1e-15)
    assert np.allclose(ref.silu(z.numpy()), want_s, rtol=1e-13, atol=1e-15)


# ---- epilogue wiring and order -------------------------------------------------------

def test_epilogue_order_bias_then_activation_then_residual():
    M, N = 3, 4
    A = bf([1.0] * M).reshape(M, 1)
    Bz = bf([0.0] * N).reshape(1, N)
    bias = bf([-1.0, 0.5, 1.0, 2.0])
    res = wl.small_int((M, N), -3, 3, "ep.R")
    r = wl.bits(res)
    pts = dict(_golden_points()["gelu_tanh"])
    gb = np.array([pts[-1.0], pts[0.5], pts[1.0], pts[2.0]])
    resv = res.to(torch.float64).numpy()
    # bias only / residual only / act only / all
    assert np.array_equal(ref.gemm_epilogue(A, Bz, bias=bias).z, np.tile([-1.0, 0.5, 1.0, 2.0], (M, 1)))
    assert np.array_equal(ref.gemm_epilogue(A, Bz, residual=r).z, resv)
    assert np.array_equal(ref.gemm_epilogue(A, Bz, act=ref.ACT_GELU_TANH).z, np.zeros((M, N)))
    z = ref.gemm_epilogue(A, Bz, bias=bias, residual=r, act=ref.ACT_GELU_TANH).z
    assert np.allclose(z, gb[None, :] + resv, rtol=1e-14, atol=1e-15)
    # the accumulator itself goes through the activation too: B = 1 -> gelu(1 + bias)
    B1 = bf([1.0] * N).reshape(1, N)
    z = ref.gemm_epilogue(A, B1, bias=bf([0.0, 1.0, 2.0, -1.5]), act=ref.ACT_GELU_TANH).z
    assert np.allclose(z[0], [pts[1.0], pts[2.0], pts[3.0], pts[-0.5]], rtol=1e-14)


def test_silu_gate_wiring():
    pts = dict(_golden_points()["silu"])
    # X = [1], gate weights g_j, up weights u_j  ->  out_j = SiLU(g_j) * u_j
    g = [1.0, -1.0, 2.0, 0.0, 3.0]
    u = [1.0, 1.0, 0.5, 7.0, -2.0]
    X = bf([1.0]).reshape(1, 1)
    W = bf(g + u).reshape(10, 1)                 # gate rows first, then up rows
    r = ref.gemm_epilogue(X, W, trans_b=True, act=ref.ACT_SILU_GATE)
    want = [pts[1.0], pts[-1.0], 0.5 * pts[2.0], 0.0, -2.0 * pts[3.0]]
    assert r.z.shape == (1, 5)
    assert np.allclose(r.z[0], want, rtol=1e-14, atol=0)
    # residual is added after the product
    res = bf([1.0, 2.0, 3.0, 4.0, 5.0]).reshape(1, 5)
    r2 = ref.gemm_epilogue(X, W, trans_b=True, residual=res, act=ref.ACT_SILU_GATE)
    assert np.allclose(r2.z[0], np.array(want) + [1, 2, 3, 4, 5], rtol=1e-14)
    with pytest.raises(ValueError):
        ref.gemm_epilogue(X, W, trans_b=True, bias=bf([0.0] * 5), act=ref.ACT_SILU_GATE)


def test_block_mlp_rounds_h_between_the_gemms():
    # H = 1.0078125 * 1.5 = 1.51171875 rounds to 1.515625 in bf16; Y = H - 1.5
    X = bf([1.0078125]).reshape(1, 1)
    W1 = bf([1.5]).reshape(1, 1)
    W2 = bf([1.0]).reshape(1, 1)
    b2 = bf([-1.5])
    h, y = ref.block_mlp(X, W1, None, None, ref.ACT_NONE, W2, b2, None)
    assert h.z[0, 0] == 1.51171875 and ref.widen(h.bits)[0, 0] == 1.515625
    assert y.z[0, 0] == 0.015625                  # from the rounded H, not 0.01171875
    # stage-wise variant consumes the H it is handed
    h2, y2 = ref.block_mlp(X, W1, None, None, ref.ACT_NONE, W2, b2, None, H_bits=bf([1.5]).reshape(1, 1))
    assert y2.z[0, 0] == 0.0


def test_block_mlp_gelu_and_swiglu_composition_against_torch_fp64():
    T, d, dff = 6, 8, 12
    X = wl.normal((T, d), 1.0, "bm.X")
    W1 = wl.normal((dff, d), 0.3, "bm.W1")
    Wu = wl.normal((dff, d), 0.3, "bm.Wu")
    b1 = wl.normal((dff,), 0.3, "bm.b1")
    W2 = wl.normal((d, dff), 0.3, "bm.W2")
    b2 = wl.normal((d,), 0.3, "bm.b2")
    R = wl.normal((T, d), 1.0, "bm.R")
    f = lambda t: t.to(torch.float64)
    # GELU block with torch's own fp64 operators (library cross-check of the composition)
    h, y = ref.block_mlp(X, W1, None, b1, ref.ACT_GELU_TANH, W2, b2, R)
    Ht = torch.nn.functional.gelu(f(X) @ f(W1).t() + f(b1), approximate="tanh")
    assert np.allclose(h.z, Ht.numpy(), rtol=1e-12, atol=1e-14)
    Hb = Ht.to(torch.bfloat16)
    Yt = f(Hb) @ f(W2).t() + f(b2) + f(R)
    assert np.allclose(y.z, Yt.numpy(), rtol=1e-12, atol=1e-13)
    # SwiGLU block
    h, y = ref.block_mlp(X, W1, Wu, None, ref.ACT_SILU_GATE, W2, None, R)
    Ht = torch.nn.functional.silu(f(X) @ f(W1).t()) * (f(X) @ f(Wu).t())
    assert np.allclose(h.z, Ht.numpy(), rtol=1e-12, atol=1e-14)
    Yt = f(Ht.to(torch.bfloat16)) @ f(W2).t() + f(R)
    assert np.allclose(y.z, Yt.numpy(), rtol=1e-12, atol=1e-13)


# ---- the checker itself ---------------------------------------------------------------

def test_checker_accepts_rounded_reference_and_rejects_a_planted_error():
    c = wl.config1(64)
    r = ref.gemm_epilogue(c["A"], c["B"])
    s = check.compare(r.bits, r)
    assert s["ok"] and s["bits_equal_frac"] == 1.0 and s["rel_frobenius"] < 3e-3
    bad = r.bits.copy()
    bad[5, 9] ^= 0x0040                       # flip a high fraction bit of one element
    r2 = ref.Ref(z=r.z, bound=np.zeros_like(r.bound), bits=r.bits, rows=r.rows)
    assert not check.compare(bad, r2)["ok"]
    # a transposed result must fail
    assert not check.compare(np.ascontiguousarray(r.bits.T), r)["ok"]
    with pytest.raises(AssertionError):
        check.assert_bits_equal(bad, r)


# ---- row subsets: residual selection, the block, and the checker's "full" mode -------------------

def test_residual_rows_follow_the_row_subset():
    # A = 0: the GEMM contributes nothing, so output row i is exactly residual row rows[i] (its own
    # bits: a bf16 value rounds to itself).  Every residual row is different, the subset is
    # unsorted and repeats a row, the residual is wider than the output.
    M, K, N = 9, 3, 5
    A = np.zeros((M, K), dtype=np.uint16)
    B = wl.bits(wl.uniform((K, N), "rr.B"))
    R = wl.bits(wl.normal((M, N + 3), 1.0, "rr.R"))
    assert len({R[i, :N].tobytes() for i in range(M)}) == M
    rows = [8, 2, 2, 0, 5]
    r = ref.gemm_epilogue(A, B, residual=R, rows=rows)
    assert np.array_equal(r.bits, R[rows, :N]) and np.array_equal(r.rows, rows)
    assert np.array_equal(r.bound, np.abs(ref.widen(R[rows, :N])))
    # and on a real product: the subset equals the same rows of the full result
    A = wl.uniform((M, K), "rr.A")
    full = ref.gemm_epilogue(A, B, bias=wl.uniform((N,), "rr.b"), residual=R, act=ref.ACT_GELU_TANH)
    sub = ref.gemm_epilogue(A, B, bias=wl.uniform((N,), "rr.b"), residual=R, act=ref.ACT_GELU_TANH, rows=rows)
    assert np.array_equal(sub.z, full.z[rows]) and np.array_equal(sub.bits, full.bits[rows]) and np.array_equal(sub.bound, full.bound[rows])
    # a planted row mistake (residual taken from rows 0..n-1 instead of the subset) is not the same
    wrong = ref.gemm_epilogue(A, B, bias=wl.uniform((N,), "rr.b"), residual=R[: len(rows)], act=ref.ACT_GELU_TANH,
                              rows=list(range(len(rows))))
    assert not np.array_equal(wrong.bits, sub.bits)


@pytest.mark.parametrize("gated", [False, True])
def test_block_mlp_rows_follow_the_row_subset(gated):
    T, d, dff = 10, 8, 16
    W1 = wl.normal((dff, d), 0.3, "br.W1")
    Wu = wl.normal((dff, d), 0.3, "br.Wu") if gated else None
    b1 = None if gated else wl.normal((dff,), 0.3, "br.b1")
    act = ref.ACT_SILU_GATE if gated else ref.ACT_GELU_TANH
    W2 = wl.normal((d, dff), 0.3, "br.W2")
    b2 = wl.normal((d,), 0.3, "br.b2")
    R = wl.normal((T, d), 1.0, "br.R")
    rows = [9, 4, 4, 1]
    # X = 0: H is the same in every row, so Y[i] - Y[j] = R[rows[i]] - R[rows[j]] exactly in fp64
    X0 = np.zeros((T, d), dtype=np.uint16)
    h, y = ref.block_mlp(X0, W1, Wu, b1, act, W2, b2, R, rows=rows)
    assert (h.bits == h.bits[0]).all()
    Rw = ref.widen(wl.bits(R))
    const = y.z - Rw[rows]
    assert np.abs(const - const[0]).max() < 1e-13 and np.array_equal(y.rows, rows)
    # real X: the subset equals the same rows of the whole block, in both modes
    X = wl.normal((T, d), 1.0, "br.X")
    hf, yf = ref.block_mlp(X, W1, Wu, b1, act, W2, b2, R)
    hs, ys = ref.block_mlp(X, W1, Wu, b1, act, W2, b2, R, rows=rows)
    assert np.array_equal(hs.bits, hf.bits[rows]) and np.array_equal(ys.z, yf.z[rows]) and np.array_equal(ys.bound, yf.bound[rows])
    # stage-wise mode: H handed in for ALL rows; the second stage must pick rows[] out of it
    Hgiven = wl.bits(wl.normal((T, dff), 0.5, "br.H"))
    _, yg = ref.block_mlp(X, W1, Wu, b1, act, W2, b2, R, rows=rows, H_bits=Hgiven)
    direct = ref.gemm_epilogue(Hgiven[rows], W2, True, bias=b2, residual=wl.bits(R)[rows])
    assert np.array_equal(yg.z, direct.z) and np.array_equal(yg.rows, rows)


def test_checker_full_mode_takes_the_reference_rows():
    c = wl.config1(64)
    rows = [63, 5, 17, 0]
    r = ref.gemm_epilogue(c["A"], c["B"], rows=rows)
    full = np.full((64, 64), 0x7FC0, dtype=np.uint16)          # NaN everywhere ...
    full[rows] = r.bits                                         # ... except the rows the reference names
    s = check.compare(full, r, rows="full")
    assert s["ok"] and s["bits_equal_frac"] == 1.0 and s["elements"] == len(rows) * 64
    check.assert_bits_equal(full, r, rows="full")
    # planted: the right values in the wrong rows (as if rows 0..3 of the output had been compared)
    wrong = np.full((64, 64), 0x7FC0, dtype=np.uint16)
    wrong[: len(rows)] = r.bits
    assert not check.compare(wrong, r, rows="full")["ok"]
    with pytest.raises(AssertionError):
        check.assert_bits_equal(wrong, r, rows="full")
    # planted: two of the named rows exchanged
    swapped = full.copy()
    swapped[[63, 5]] = swapped[[5, 63]]
    assert not check.compare(swapped, r, rows="full")["ok"]
    with pytest.raises(AssertionError):
        check.assert_bits_equal(swapped, r, rows="full")
    # without "full" the same array is taken row for row and has the wrong shape
    with pytest.raises(ValueError):
        check.compare(full, r)
