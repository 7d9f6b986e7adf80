"""GPU parity of fact_attention against the fp64 attention oracle, through the C ABI.

Tolerance (same form as the GEMM contract): per element |got - z| <= 1e-2 * bound + 1e-3 with
bound = sum_j P_ij |V_jd|, and relative Frobenius error <= 5e-3.  The kernel rounds the
probabilities to bf16 before the second contraction (each term of the sum off by at most 2^-9 of
its magnitude), accumulates in fp32 and rounds the output once (2^-9 |o| <= 2^-9 bound): about
4e-3 * bound in the worst case, 1e-3 relative in the Frobenius norm."""
import numpy as np
import pytest
import torch

import paper_2604_26666_amd as fact
import workloads as wl
from oracle import attention as att
from oracle import check, ref

pytestmark = pytest.mark.gpu

POISON = 0x7FC1


def run_packed(B, T, Hq, Hkv, D, causal, std=1.0, name="ga", scale=0.0):
    """Q, K, V as slices of one packed projection output [B, T, (Hq + 2 Hkv) D]; O dense with a
    guard row per batch entry.  Returns (got bits [B*T*Hq, D], reference)."""
    W = (Hq + 2 * Hkv) * D
    packed = wl.normal((B, T, W), std, f"{name}.qkv.{B}.{T}.{Hq}.{Hkv}.{D}")
    pb = wl.bits(packed)
    Qv = pb[:, :, : Hq * D].reshape(B, T, Hq, D)
    Kv = pb[:, :, Hq * D: (Hq + Hkv) * D].reshape(B, T, Hkv, D)
    Vv = pb[:, :, (Hq + Hkv) * D:].reshape(B, T, Hkv, D)
    r = att.attention(Qv, Kv, Vv, causal=bool(causal), scale=None if scale <= 0 else scale)
    dev = packed.cuda()
    O = torch.full((B, T + 1, Hq * D), POISON, dtype=torch.int16).view(torch.bfloat16).cuda()
    base = dev.data_ptr()
    strides = (T * W, W, D)
    rc = fact.fact_attention(B, T, Hq, Hkv, D, base, strides, base + 2 * Hq * D, strides,
                             base + 2 * (Hq + Hkv) * D, strides, O, ((T + 1) * Hq * D, Hq * D, D), causal, scale)
    fact.binding.check(rc, f"fact_attention B={B} T={T} Hq={Hq} Hkv={Hkv} D={D} causal={causal}")
    torch.cuda.synchronize()
    ob = wl.bits(O.cpu())
    assert (ob[:, T, :] == POISON).all(), "wrote outside O"
    return np.ascontiguousarray(ob[:, :T, :]).reshape(B * T * Hq, D), r


@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("causal", [1, 0])
def test_small_ragged_lengths(D, causal):
    # shorter than one key block, one block and a bit, several blocks with a ragged tail
    for T in (1, 7, 64, 65, 100, 300):
        got, r = run_packed(2, T, 4, 2, D, causal, name=f"sm{causal}")
        s = check.assert_close(got, r, what=f"attention T={T} D={D} causal={causal}")
        assert s["rel_frobenius"] < 3e-3, s


@pytest.mark.parametrize("Hq,Hkv", [(3, 3), (8, 2), (4, 1)])
def test_head_grouping(Hq, Hkv):
    got, r = run_packed(2, 200, Hq, Hkv, 128, 1, name="hg")
    check.assert_close(got, r, what=f"attention heads {Hq}/{Hkv}")


def test_many_query_blocks_ragged_length():
    # several query blocks per head, T not a multiple of anything (the 256-query work-groups that
    # long sequences of 128-wide heads get are covered by the full-size tests)
    got, r = run_packed(2, 1000, 16, 4, 128, 1, std=1.28, name="qb4")
    check.assert_close(got, r, what="attention 2 x 1000 tokens, 16/4 heads of 128")
    got, r = run_packed(1, 1000, 4, 4, 64, 1, std=0.55, name="qb2")
    check.assert_close(got, r, what="attention 1000 tokens, 4 heads of 64")


def test_explicit_scale_and_peaked_scores():
    # a large scale makes the softmax nearly one-hot: the running maximum does the work
    got, r = run_packed(1, 257, 2, 1, 128, 1, std=1.0, name="sc", scale=1.0)
    check.assert_close(got, r, what="attention scale 1.0")
    got, r = run_packed(1, 257, 2, 1, 64, 0, std=1.0, name="sc0", scale=0.01)
    check.assert_close(got, r, what="attention scale 0.01 (nearly uniform)")


@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("causal", [1, 0])
def test_constructed_score_patterns(D, causal):
    """Inputs built so that the running reference of the softmax is exercised: scores that grow
    along the keys (every key block raises the reference and rescales the sums), scores that fall
    (the first block's reference stays for good), and all-equal scores (uniform probabilities:
    each output is the mean of the values it may see)."""
    B, T, H = 1, 330, 2
    V = wl.normal((B, T, H, D), 1.0, f"cs.V.{D}")
    ramp = torch.arange(T, dtype=torch.float32).view(1, T, 1, 1) / 8.0           # + 8 per key block of 64 at scale 1 / D
    for name, qv, kv in (("growing", 1.0, ramp), ("falling", 1.0, -ramp), ("equal", 0.0, ramp)):
        Q = torch.full((B, T, H, D), qv).to(torch.bfloat16)
        K = (kv * torch.ones(B, T, H, D)).to(torch.bfloat16)
        r = att.attention(wl.bits(Q), wl.bits(K), wl.bits(V), causal=bool(causal), scale=1.0 / D)
        O = torch.empty((B, T, H, D), dtype=torch.bfloat16, device="cuda")
        st = (T * H * D, H * D, D)
        fact.binding.check(fact.fact_attention(B, T, H, H, D, Q.cuda(), st, K.cuda(), st, V.cuda(), st, O, st, causal, 1.0 / D), name)
        torch.cuda.synchronize()
        got = wl.bits(O.cpu()).reshape(B * T * H, D)
        check.assert_close(got, r, what=f"attention, {name} scores, D={D} causal={causal}")
        if name == "equal":
            v = V.float().numpy()
            i = T - 1
            mean = v[0, : i + 1].mean(axis=0) if causal else v[0].mean(axis=0)
            assert np.abs(ref.widen(got.reshape(T, H, D)[i]) - mean).max() < 2e-2


def test_dense_head_major_layout():
    # Q, K, V, O as separate [B, H, T, D] tensors (token stride D, head stride T*D)
    B, T, Hq, Hkv, D = 2, 150, 4, 2, 64
    Q = wl.normal((B, Hq, T, D), 1.0, "hm.Q"); K = wl.normal((B, Hkv, T, D), 1.0, "hm.K"); V = wl.normal((B, Hkv, T, D), 1.0, "hm.V")
    r = att.attention(wl.bits(Q).transpose(0, 2, 1, 3), wl.bits(K).transpose(0, 2, 1, 3), wl.bits(V).transpose(0, 2, 1, 3))
    O = torch.empty((B, Hq, T, D), dtype=torch.bfloat16, device="cuda")
    rc = fact.fact_attention(B, T, Hq, Hkv, D, Q.cuda(), (Hq * T * D, D, T * D), K.cuda(), (Hkv * T * D, D, T * D),
                             V.cuda(), (Hkv * T * D, D, T * D), O, (Hq * T * D, D, T * D), 1, 0.0)
    fact.binding.check(rc, "fact_attention head-major")
    torch.cuda.synchronize()
    got = np.ascontiguousarray(wl.bits(O.cpu()).transpose(0, 2, 1, 3)).reshape(B * T * Hq, D)
    check.assert_close(got, r, what="attention head-major layout")


def test_refusals_launch_nothing():
    x = torch.zeros(4 * 64 * 3 * 64, dtype=torch.bfloat16, device="cuda")
    O = torch.full((64 * 64,), POISON, dtype=torch.int16).view(torch.bfloat16).cuda()
    st = (64 * 192, 192, 64)
    ok = dict(batch=1, T=64, n_q_heads=1, n_kv_heads=1, head_dim=64)
    call = lambda **kw: fact.fact_attention(kw.get("batch", 1), kw.get("T", 64), kw.get("hq", 1), kw.get("hkv", 1), kw.get("D", 64),
                                            kw.get("Q", x), kw.get("qs", st), x.data_ptr() + 128, st, x.data_ptr() + 256, st,
                                            O, (64 * 64, 64, 64), kw.get("causal", 1), 0.0)
    assert call(D=96) == -7
    assert call(hq=3, hkv=2) == -2
    assert call(Q=None) == -1
    assert call(Q=x.data_ptr() + 2) == -3
    assert call(qs=(64 * 192, 32, 64)) == -2
    assert call(causal=2) == -4
    torch.cuda.synchronize()
    assert (wl.bits(O.cpu()) == POISON).all()
    assert call() == 0
