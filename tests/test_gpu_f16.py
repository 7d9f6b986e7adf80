"""GPU parity of the binary16 ("fp16") mode: fact_epilogue.f16 = 1 through the C ABI against the CPU
oracle's fp16 path, element by element.

Exact tests (integers, rounding ties, subnormal results) demand equal bits; tolerance tests demand the
per-element criterion |got - z| <= 1e-2 * bound + 1e-3 and a relative Frobenius error <= 1e-3
(oracle/check.py, the fp16 figures).
"""
import numpy as np
import pytest
import torch

import paper_2604_26666_amd as fact
import workloads as wl
from oracle import check, ref

pytestmark = pytest.mark.gpu

POISON = 0x7E01      # a binary16 NaN pattern the library never produces


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    if not torch.cuda.is_available():
        pytest.fail("these tests need the GPU; none is visible")
    import os
    assert os.path.exists(fact.lib_path()), "libfact_gemm.so is not built"
    fact.lib()


def cfgs(trans_b):
    return [c for c in range(fact.fact_num_configs()) if trans_b or 64 % (fact.fact_config_info(c)[1] // 8) == 0]


def poisoned(rows, cols):
    return torch.full((rows, cols), POISON, dtype=torch.int16).view(torch.float16).cuda()


def padded(t, pad):
    r, c = t.shape
    buf = poisoned(r, c + pad)
    buf[:, :c] = t.cuda()
    return buf, c + pad


def gemm16(A, B, trans_b, bias=None, residual=None, act=fact.ACT_NONE, cfg=-1, split=0, group_m=0, pad=0, out_f32=False):
    """One fp16 GEMM on the GPU; A, B, bias, residual are CPU float16 tensors.  Returns the uint16 output
    [M, Nout] (or the fp32 output) and checks that nothing outside it was written."""
    M, K = A.shape
    N = B.shape[0] if trans_b else B.shape[1]
    nout = N // 2 if act == fact.ACT_SILU_GATE else N
    Ab, lda = padded(A, pad)
    Bb, ldb = padded(B, pad)
    ldc = nout + pad + 8
    if out_f32:
        Cb = torch.full((M + 1, ldc), float("nan"), dtype=torch.float32, device="cuda")
    else:
        Cb = poisoned(M + 1, ldc)
    res_ptr, ldr = None, 0
    if residual is not None:
        res_ptr, ldr = padded(residual, pad)
    ep = fact.Epilogue(bias=None if bias is None else bias.cuda(), residual=res_ptr, ldr=ldr, act=act, out_f32=int(out_f32), f16=1)
    if out_f32:
        ws_bytes = max(fact.fact_gemm_f32out_workspace_bytes(M, N, K, split), 16)
    else:
        ws_bytes = max(fact.fact_gemm_splitk_workspace_bytes(M, N, K, split), 16) if split != 1 else 16
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda").fill_(0xA5)
    rc = fact.fact_gemm_ex(1, M, N, K, Ab, lda, 0, Bb, ldb, 0, trans_b, Cb, ldc, 0, ep, cfg, split, group_m, ws, ws_bytes)
    fact.binding.check(rc, f"fp16 M={M} N={N} K={K} tb={trans_b} act={act} cfg={cfg} split={split}")
    torch.cuda.synchronize()
    if out_f32:
        out = Cb.cpu().numpy()
        assert np.isnan(out[M, :]).all() and np.isnan(out[:, nout:]).all(), "wrote outside C"
        return out[:M, :nout].copy()
    out = wl.bits(Cb.cpu().contiguous())
    assert (out[M, :] == POISON).all() and (out[:, nout:] == POISON).all(), "wrote outside C"
    return out[:M, :nout].copy()


# ---- exact ------------------------------------------------------------------------------------

@pytest.mark.parametrize("trans_b", [0, 1])
@pytest.mark.parametrize("shape", [(300, 264, 200), (520, 776, 1096), (257, 520, 72)])
def test_integers_bit_exact_every_config(shape, trans_b):
    # |a| <= 20; sums stay below 2^24, so fp32 accumulation is exact in any order and
    # the only rounding is the store's (sums above 2048 are not all binary16 numbers)
    M, N, K = shape
    A = wl.small_int_f16((M, K), -20, 20, f"h.A{shape}")
    B = wl.small_int_f16((K, N), -20, 20, f"h.B{shape}")
    Bs = B if not trans_b else B.t().contiguous()
    r = ref.gemm_epilogue(A, Bs, bool(trans_b), fmt="f16")
    assert np.abs(r.z).max() < 2 ** 24 and np.abs(r.z).max() > 2048 and np.abs(r.z).max() < 65504
    for cfg in cfgs(trans_b):
        got = gemm16(A, Bs, trans_b, cfg=cfg, pad=8 if cfg % 2 else 0)
        check.assert_bits_equal(got, r, what=f"cfg {cfg} {shape} tb {trans_b}")


def test_eleven_bit_operands_are_multiplied_exactly():
    # odd integers up to 2047 use all 11 significant bits of binary16 (bf16 holds 8); K = 2 products of
    # up to 22 bits are exact in the fp32 accumulator, their sums too
    M, N, K = 128, 128, 64
    A = torch.zeros(M, K, dtype=torch.float16)
    B = torch.zeros(K, N, dtype=torch.float16)
    A[:, :2] = wl.small_int_f16((M, 2), -2047, 2047, "h11.A")
    B[:2, :] = wl.small_int_f16((2, N), -2047, 2047, "h11.B")
    got = gemm16(A, B, 0, out_f32=True, split=1)
    want = A.double().numpy() @ B.double().numpy()
    assert np.abs(want).max() > 2 ** 21
    assert (got.astype(np.float64) == want).all()
    r = ref.gemm_epilogue(A, B, False, fmt="f16")
    assert (r.z == want).all()
    check.assert_bits_equal(gemm16(A, B, 0), r, what="rounded store, overflow to infinity included")
    assert (r.bits == 0x7C00).any() or (r.bits == 0xFC00).any()         # some |sums| exceed 65520


def test_rounding_ties_overflow_and_subnormal_results():
    # K = 1 products through the MFMA path (K padded with zeros to one step) and the guarded kernel
    a = torch.tensor([1.0 + 2.0 ** -10, 1.0 + 3 * 2.0 ** -10, 255.0, 2.0 ** -12, 2.0 ** -14, -(2.0 ** -13)] * 11, dtype=torch.float32)[:64]
    b = torch.tensor([1.5, 1.25, 257.0, 2.0 ** -11, 3 * 2.0 ** -11] * 13, dtype=torch.float32)[:64]
    for K, entry in ((1, "fallback"), (64, "mfma")):
        A = torch.zeros(64, K)
        A[:, 0] = a
        B = torch.zeros(K, 64)
        B[0, :] = b
        A, B = A.to(torch.float16), B.to(torch.float16)
        assert (A.float()[:, 0] == a).all() and (B.float()[0, :] == b).all()
        r = ref.gemm_epilogue(A, B, fmt="f16")
        rc, cfg, _ = fact.fact_select_config(1, 64, 64, K, 0, 0)
        assert (cfg < 0) == (entry == "fallback")
        got = gemm16(A, B, 0)
        check.assert_bits_equal(got, r, what=entry)
        w = ref.widen(got, "f16")
        assert w[0, 0] == 1.5 + 2.0 ** -9                   # 1.5 (1 + 2^-10) = 1.5 + 1.5 * 2^-10: tie -> even
        assert w[2, 2] == np.inf                             # 255 * 257 = 65535 -> infinity
        assert w[3, 3] == 2.0 ** -23 and w[4, 4] == 2.0 ** -24 * 2      # 2^-14 * 3 * 2^-11 = 1.5 * 2^-24: tie -> 2 quanta
        assert w[5, 3] == -(2.0 ** -24)


def test_subnormal_operands_count():
    # binary16 subnormals (below 2^-14) as operands: the matrix instruction must not flush them
    M = N = K = 64
    A = torch.zeros(M, K, dtype=torch.float16)
    B = torch.zeros(K, N, dtype=torch.float16)
    A[:, 0] = torch.tensor([float(i + 1) * 2.0 ** -24 for i in range(M)], dtype=torch.float64).to(torch.float16)
    B[0, :] = torch.tensor([float(2 ** (j % 6 + 8)) for j in range(N)], dtype=torch.float64).to(torch.float16)
    r = ref.gemm_epilogue(A, B, fmt="f16")
    assert (r.z != 0).all()
    check.assert_bits_equal(gemm16(A, B, 0), r, what="subnormal operands")


# ---- tolerance: every epilogue, split-K, batches ---------------------------------------------

@pytest.mark.parametrize("trans_b", [0, 1])
def test_normal_inputs_every_epilogue_table_choice_and_every_config(trans_b):
    M, N, K = 520, 776, 1096
    A = wl.normal_f16((M, K), 1.0, "hn.A")
    B = wl.normal_f16((K, N), 1.0, "hn.B")
    Bs = B if not trans_b else B.t().contiguous()
    bias = wl.normal_f16((N,), 1.0, "hn.bias")
    res = wl.normal_f16((M, N), 1.0, "hn.res")
    cases = [dict(), dict(bias=bias), dict(bias=bias, act=fact.ACT_GELU_TANH), dict(bias=bias, residual=res),
             dict(bias=bias, act=fact.ACT_GELU_TANH, residual=res)]
    for kw in cases:
        okw = {k: v for k, v in kw.items()}
        r = ref.gemm_epilogue(A, Bs, bool(trans_b), fmt="f16", **okw)
        for cfg in [-1] + cfgs(trans_b):
            check.assert_close(gemm16(A, Bs, trans_b, cfg=cfg, **kw), r, what=f"cfg {cfg} {sorted(kw)}")


def test_gated_epilogue_every_config():
    M, I, K = 300, 264, 512
    X = wl.normal_f16((M, K), 1.0, "hg.X")
    W = wl.normal_f16((2 * I, K), 0.05, "hg.W")
    res = wl.normal_f16((M, I), 1.0, "hg.res")
    r = ref.gemm_epilogue(X, W, True, residual=res, act=ref.ACT_SILU_GATE, fmt="f16")
    for cfg in [-1] + cfgs(1):
        check.assert_close(gemm16(X, W, 1, residual=res, act=fact.ACT_SILU_GATE, cfg=cfg), r, what=f"gated cfg {cfg}")


def test_split_k_rounded_and_fp32_output():
    M, N, K = 256, 264, 8192
    A = wl.normal_f16((M, K), K ** -0.5, "hs.A")
    B = wl.normal_f16((K, N), 1.0, "hs.B")
    bias = wl.normal_f16((N,), 1.0, "hs.bias")
    r = ref.gemm_epilogue(A, B, False, bias=bias, fmt="f16")
    for split in (2, 5, 16):
        check.assert_close(gemm16(A, B, 0, bias=bias, split=split), r, what=f"split {split}")
        got = gemm16(A, B, 0, bias=bias, split=split, out_f32=True)
        assert np.abs(got - r.z).max() <= 1e-3 * np.abs(r.z).max() and np.linalg.norm(got - r.z) <= 5e-6 * np.linalg.norm(r.z)
    Ai = wl.small_int_f16((M, K), -3, 3, "hs.Ai")
    Bi = wl.small_int_f16((K, N), -3, 3, "hs.Bi")
    ri = ref.gemm_epilogue(Ai, Bi, False, fmt="f16")
    for split in (1, 3, 8):
        check.assert_bits_equal(gemm16(Ai, Bi, 0, split=split), ri, what=f"integers, split {split}")


def test_batched_entries_and_guarded_kernel():
    batch, M, N, K = 3, 128, 136, 256
    A = wl.normal_f16((batch, M, K), 1.0, "hb.A")
    B = wl.normal_f16((batch, K, N), 1.0, "hb.B")
    C = poisoned(batch * M, N).view(batch, M, N)
    ep = fact.Epilogue(f16=1)
    fact.binding.check(fact.fact_gemm_batched(batch, M, N, K, A.cuda(), K, M * K, B.cuda(), N, K * N, 0, C, N, M * N, ep))
    torch.cuda.synchronize()
    for z in range(batch):
        check.assert_close(wl.bits(C[z].cpu().contiguous()), ref.gemm_epilogue(A[z], B[z], False, fmt="f16"), what=f"batch {z}")
    for (m, n, k) in [(5, 7, 3), (33, 20, 100)]:                       # K % 8 != 0: the guarded kernel
        a = wl.small_int_f16((m, k), -40, 40, f"hf.A{m}")
        b = wl.small_int_f16((k, n), -40, 40, f"hf.B{m}")
        bias = wl.small_int_f16((n,), -3, 3, "hf.bias")
        res = wl.small_int_f16((m, n), -3, 3, "hf.res")
        r = ref.gemm_epilogue(a, b, False, bias=bias, residual=res, fmt="f16")
        check.assert_bits_equal(gemm16(a, b, 0, bias=bias, residual=res, pad=3), r, what=f"guarded {(m, n, k)}")


def test_bf16_calls_are_untouched_by_the_field():
    import gpu_util
    A = wl.normal((256, 512), 1.0, "hx.A")
    B = wl.normal((512, 256), 1.0, "hx.B")
    r = ref.gemm_epilogue(A, B, False)
    check.assert_close(gpu_util.gemm(A, B, 0), r, what="bf16 beside fp16")
    bad = fact.Epilogue(f16=2)
    d = A.cuda()
    out = torch.empty(256, 256, dtype=torch.bfloat16, device="cuda")
    assert fact.fact_gemm(256, 256, 512, d, 512, B.cuda(), 256, 0, out, 256, bad) == -5          # FACT_ERR_EPILOGUE


# ---- full size ----------------------------------------------------------------------------------

def test_square_8192_bias_fp16_one_row_of_every_eight():
    # (the fp16 widening of the oracle is branchy and takes 4-5 times the bf16 one: one row out of every
    # group of 8, at a position that walks through the group, instead of every row as in the bf16 test of
    # the same launch; every tile, wave and 16-row MFMA tile of the 1024-tile launch is sampled)
    n = 8192
    c = wl.config2_f16(n)
    C = torch.empty(n, n, dtype=torch.float16, device="cuda")
    ep = fact.Epilogue(bias=c["bias"].cuda(), f16=1)
    fact.binding.check(fact.fact_gemm(n, n, n, c["A"].cuda(), n, c["B"].cuda(), n, 0, C, n, ep))
    torch.cuda.synchronize()
    got = wl.bits(C.cpu().contiguous())
    i = np.arange(n // 8)
    rows = 8 * i + (5 * i) % 8
    for part in np.array_split(rows, 4):
        r = ref.gemm_epilogue(c["A"], c["B"], False, bias=c["bias"], rows=part, fmt="f16")
        s = check.assert_close(got, r, rows="full", what=f"fp16 8192^3 rows {part[0]}..")
        assert s["bits_equal_frac"] > 0.9, s         # fp32 accumulation moves few results across a rounding boundary


# ---- the two-GEMM block in fp16 ---------------------------------------------------------------

@pytest.mark.parametrize("kind", ["gelu", "swiglu"])
def test_block_mlp_fp16_reduced(kind):
    T, d, dff = 520, 256, 768
    X = wl.normal_f16((T, d), 1.0, "hm.X")
    W1 = wl.normal_f16((dff, d), 0.05, "hm.W1")
    Wu = wl.normal_f16((dff, d), 0.05, "hm.Wu")
    b1 = wl.normal_f16((dff,), 0.05, "hm.b1")
    W2 = wl.normal_f16((d, dff), 0.05, "hm.W2")
    b2 = wl.normal_f16((d,), 0.05, "hm.b2")
    R = wl.normal_f16((T, d), 1.0, "hm.R")
    gated = kind == "swiglu"
    act = fact.ACT_SILU_GATE if gated else fact.ACT_GELU_TANH
    Hd, Yd = poisoned(T, dff), poisoned(T, d)
    need = fact.fact_block_mlp_workspace_bytes(T, d, dff, act)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
    rc = fact.fact_block_mlp_f16(T, d, dff, X.cuda(), W1.cuda(), Wu.cuda() if gated else None,
                                 None if gated else b1.cuda(), act, W2.cuda(), None if gated else b2.cuda(),
                                 R.cuda(), Hd, Yd, ws, need)
    fact.binding.check(rc, "fact_block_mlp_f16")
    torch.cuda.synchronize()
    Hg, Yg = wl.bits(Hd.cpu().contiguous()), wl.bits(Yd.cpu().contiguous())
    args = (X, W1, Wu if gated else None, None if gated else b1, act, W2, None if gated else b2, R)
    h, y = ref.block_mlp(*args, fmt="f16")
    check.assert_close(Hg, h, what="fp16 H")
    check.assert_close(Yg, y, what="fp16 Y end to end")
    _, y2 = ref.block_mlp(*args, H_bits=Hg, fmt="f16")                   # the oracle's second GEMM fed the GPU's H bits
    s = check.assert_close(Yg, y2, what="fp16 Y stage-wise")
    assert s["bits_equal_frac"] >= 0.97, s


def test_block_mlp_fp16_paper_gpt_shape_sampled_rows():
    # the MLP of the paper's GPT block (Section 5.2.4: 768 -> 3072 -> 768, GELU) at 8192 tokens, in its precision
    T, d, dff = 8192, 768, 3072
    X = wl.normal_f16((T, d), 1.0, "hp.X")
    W1 = wl.normal_f16((dff, d), 0.02, "hp.W1")
    b1 = wl.normal_f16((dff,), 0.02, "hp.b1")
    W2 = wl.normal_f16((d, dff), 0.02, "hp.W2")
    b2 = wl.normal_f16((d,), 0.02, "hp.b2")
    R = wl.normal_f16((T, d), 1.0, "hp.R")
    Hd = torch.empty(T, dff, dtype=torch.float16, device="cuda")
    Yd = torch.empty(T, d, dtype=torch.float16, device="cuda")
    need = fact.fact_block_mlp_workspace_bytes(T, d, dff, fact.ACT_GELU_TANH)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
    fact.binding.check(fact.fact_block_mlp_f16(T, d, dff, X.cuda(), W1.cuda(), None, b1.cuda(), fact.ACT_GELU_TANH, W2.cuda(), b2.cuda(),
                                               R.cuda(), Hd, Yd, ws, need))
    torch.cuda.synchronize()
    Hg, Yg = wl.bits(Hd.cpu().contiguous()), wl.bits(Yd.cpu().contiguous())
    rows = wl.choice_rows(T, 200, "hp.rows", edges=(0, 127, 128, 255, 256, T - 1))
    h, y = ref.block_mlp(X, W1, None, b1, fact.ACT_GELU_TANH, W2, b2, R, rows=rows, H_bits=Hg, fmt="f16")
    check.assert_close(Hg, h, rows="full", what="fp16 GPT MLP H")
    check.assert_close(Yg, y, rows="full", what="fp16 GPT MLP Y")
