"""Pins of the attention oracle (CPU only).  None of them re-types the oracle's formula with the
same library calls: closed forms, invariants, a pure-Python brute force, and a library routine
as a special-case reference (torch's fp64 attention with expanded key/value heads)."""
import math

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import attention as att
from oracle import ref


def bits(x):
    """fp64/fp32 array -> bf16 bit patterns (values chosen exactly representable where it matters)."""
    return ref.round_bf16(np.asarray(x, dtype=np.float64))


def vals(b):
    return ref.widen(b)


def out4(r, B, T, H, D):
    return r.z.reshape(B, T, H, D)


def test_equal_keys_give_the_running_mean_of_v():
    # every key identical -> every allowed score equal -> uniform weights over keys 0..i
    B, T, H, D = 2, 37, 3, 8
    Q = wl.bits(wl.normal((B, T, H, D), 1.0, "ap.Q1"))
    krow = wl.bits(wl.normal((1, 1, 1, D), 1.0, "ap.k1"))
    K = np.broadcast_to(krow, (B, T, H, D)).copy()
    V = wl.bits(wl.normal((B, T, H, D), 1.0, "ap.V1"))
    v = vals(V)
    o = out4(att.attention(Q, K, V, causal=True), B, T, H, D)
    want = np.cumsum(v, axis=1) / np.arange(1, T + 1).reshape(1, T, 1, 1)
    assert np.abs(o - want).max() < 1e-13
    o = out4(att.attention(Q, K, V, causal=False), B, T, H, D)
    want = np.broadcast_to(v.mean(axis=1, keepdims=True), v.shape)
    assert np.abs(o - want).max() < 1e-13


def test_single_token_returns_v():
    B, T, Hq, Hkv, D = 3, 1, 4, 2, 16
    Q = wl.bits(wl.normal((B, T, Hq, D), 1.0, "ap.Q2"))
    K = wl.bits(wl.normal((B, T, Hkv, D), 1.0, "ap.K2"))
    V = wl.bits(wl.normal((B, T, Hkv, D), 1.0, "ap.V2"))
    r = att.attention(Q, K, V)
    o = r.bits.reshape(B, T, Hq, D)
    for h in range(Hq):
        assert np.array_equal(o[:, 0, h], V[:, 0, h // 2])      # bit for bit: weight exactly 1


def test_two_keys_closed_form_and_default_scale():
    # T = 2, D = 4: query 1 sees keys 0 and 1; weights are a logistic function of the score gap
    D = 4
    q = np.zeros((1, 2, 1, D)); k = np.zeros((1, 2, 1, D)); v = np.zeros((1, 2, 1, D))
    q[0, 1, 0] = [1.0, 2.0, 0.0, -1.0]
    k[0, 0, 0] = [0.5, 0.25, 3.0, 1.0]        # q.k0 = 0.5 + 0.5 - 1 = 0
    k[0, 1, 0] = [2.0, 1.0, -1.0, 0.0]        # q.k1 = 2 + 2 = 4
    v[0, 0, 0] = [1.0, -2.0, 0.5, 8.0]
    v[0, 1, 0] = [3.0, 2.0, -0.5, 0.0]
    o = out4(att.attention(bits(q), bits(k), bits(v)), 1, 2, 1, D)
    w1 = 1.0 / (1.0 + math.exp(-(4.0 - 0.0) / 2.0))              # default scale 1/sqrt(4)
    assert np.allclose(o[0, 0, 0], v[0, 0, 0], atol=0, rtol=0)
    assert np.abs(o[0, 1, 0] - ((1 - w1) * v[0, 0, 0] + w1 * v[0, 1, 0])).max() < 1e-14
    o = out4(att.attention(bits(q), bits(k), bits(v), scale=0.125), 1, 2, 1, D)
    w1 = 1.0 / (1.0 + math.exp(-4.0 * 0.125))
    assert np.abs(o[0, 1, 0] - ((1 - w1) * v[0, 0, 0] + w1 * v[0, 1, 0])).max() < 1e-14
    # printed value: logistic(2) = 0.8807970779778823
    assert abs(1.0 / (1.0 + math.exp(-2.0)) - 0.8807970779778823) < 1e-15


def test_a_dominant_key_selects_its_value_row():
    B, T, H, D = 1, 20, 1, 8
    Q = np.zeros((B, T, H, D)); K = np.zeros((B, T, H, D))
    Q[..., 0] = 16.0
    K[0, 7, 0, 0] = 64.0                                            # score gap 16*64/sqrt(8) = 362
    V = wl.bits(wl.normal((B, T, H, D), 1.0, "ap.V4"))
    o = out4(att.attention(bits(Q), bits(K), V), B, T, H, D)
    v = vals(V)
    for i in range(7, T):
        assert np.abs(o[0, i, 0] - v[0, 7, 0]).max() < 1e-100 + 1e-15
    for i in range(7):                                              # before key 7 exists: uniform
        assert np.abs(o[0, i, 0] - v[0, : i + 1, 0].mean(axis=0)).max() < 1e-14


def test_future_tokens_do_not_change_earlier_outputs():
    B, T, Hq, Hkv, D = 1, 33, 4, 2, 8
    Q = wl.bits(wl.normal((B, T, Hq, D), 1.0, "ap.Q5"))
    K = wl.bits(wl.normal((B, T, Hkv, D), 1.0, "ap.K5"))
    V = wl.bits(wl.normal((B, T, Hkv, D), 1.0, "ap.V5"))
    a = att.attention(Q, K, V).bits.reshape(B, T, Hq, D)
    K2, V2 = K.copy(), V.copy()
    K2[:, 20:] = wl.bits(wl.normal((B, T - 20, Hkv, D), 3.0, "ap.K5b"))
    V2[:, 20:] = wl.bits(wl.normal((B, T - 20, Hkv, D), 3.0, "ap.V5b"))
    b = att.attention(Q, K2, V2).bits.reshape(B, T, Hq, D)
    assert np.array_equal(a[:, :20], b[:, :20])
    assert not np.array_equal(a[:, 20:], b[:, 20:])
    # and without the mask the change reaches every row
    c = att.attention(Q, K, V, causal=False).bits.reshape(B, T, Hq, D)
    d = att.attention(Q, K2, V2, causal=False).bits.reshape(B, T, Hq, D)
    assert not np.array_equal(c[:, 0], d[:, 0])


def test_adding_a_vector_to_every_key_changes_nothing():
    # scores of one query all move by the same amount q.c: the weights do not change
    B, T, H, D = 1, 19, 2, 8
    Q = wl.bits(wl.small_int((B, T, H, D), -3, 3, "ap.Q6"))
    K = wl.bits(wl.small_int((B, T, H, D), -3, 3, "ap.K6"))
    V = wl.bits(wl.normal((B, T, H, D), 1.0, "ap.V6"))
    c = np.array([2.0, -1.0, 0.0, 4.0, 1.0, -2.0, 3.0, 0.0])
    K2 = bits(vals(K) + c)                                          # small integers: exact in bf16
    for causal in (True, False):
        a = att.attention(Q, K, V, causal=causal).z
        b = att.attention(Q, K2, V, causal=causal).z
        assert np.abs(a - b).max() < 1e-12


@pytest.mark.parametrize("causal", [True, False])
def test_brute_force_python_loops(causal):
    B, T, Hq, Hkv, D = 2, 6, 4, 2, 3
    Q = wl.bits(wl.normal((B, T, Hq, D), 1.0, "ap.Q7"))
    K = wl.bits(wl.normal((B, T, Hkv, D), 1.0, "ap.K7"))
    V = wl.bits(wl.normal((B, T, Hkv, D), 1.0, "ap.V7"))
    q, k, v = vals(Q).tolist(), vals(K).tolist(), vals(V).tolist()
    r = att.attention(Q, K, V, causal=causal, scale=0.7)
    o = out4(r, B, T, Hq, D)
    bd = r.bound.reshape(B, T, Hq, D)
    for b in range(B):
        for h in range(Hq):
            g = h // (Hq // Hkv)
            for i in range(T):
                last = i if causal else T - 1
                sc = [0.7 * sum(q[b][i][h][d] * k[b][j][g][d] for d in range(D)) for j in range(last + 1)]
                mx = max(sc)
                w = [math.exp(x - mx) for x in sc]
                tot = math.fsum(w)
                for d in range(D):
                    want = math.fsum(w[j] * v[b][j][g][d] for j in range(last + 1)) / tot
                    wantb = math.fsum(w[j] * abs(v[b][j][g][d]) for j in range(last + 1)) / tot
                    assert abs(o[b, i, h, d] - want) < 1e-13
                    assert abs(bd[b, i, h, d] - wantb) < 1e-13


@pytest.mark.parametrize("causal", [True, False])
def test_library_attention_with_expanded_kv_heads(causal):
    # the grouped form must equal ordinary multi-head attention on key/value heads repeated in place
    B, T, Hq, Hkv, D = 2, 70, 8, 2, 16
    Q = wl.normal((B, T, Hq, D), 1.0, "ap.Q8")
    K = wl.normal((B, T, Hkv, D), 1.0, "ap.K8")
    V = wl.normal((B, T, Hkv, D), 1.0, "ap.V8")
    r = att.attention(wl.bits(Q), wl.bits(K), wl.bits(V), causal=causal)
    q = Q.double().permute(0, 2, 1, 3)
    k = K.double().repeat_interleave(Hq // Hkv, dim=2).permute(0, 2, 1, 3)
    v = V.double().repeat_interleave(Hq // Hkv, dim=2).permute(0, 2, 1, 3)
    want = torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=causal).permute(0, 2, 1, 3)
    assert np.abs(out4(r, B, T, Hq, D) - want.numpy()).max() < 1e-12
    # a wrong grouping (interleaved instead of consecutive heads) is not the same thing
    k2 = K.double().repeat(1, 1, Hq // Hkv, 1).permute(0, 2, 1, 3)
    v2 = V.double().repeat(1, 1, Hq // Hkv, 1).permute(0, 2, 1, 3)
    other = torch.nn.functional.scaled_dot_product_attention(q, k2, v2, is_causal=causal).permute(0, 2, 1, 3)
    assert np.abs(out4(r, B, T, Hq, D) - other.numpy()).max() > 1e-3


def test_bound_equals_output_for_nonnegative_v_and_bits_are_the_rounded_z():
    B, T, H, D = 1, 12, 2, 8
    Q = wl.bits(wl.normal((B, T, H, D), 1.0, "ap.Q9"))
    K = wl.bits(wl.normal((B, T, H, D), 1.0, "ap.K9"))
    V = bits(np.abs(vals(wl.bits(wl.normal((B, T, H, D), 1.0, "ap.V9")))))
    r = att.attention(Q, K, V)
    assert np.array_equal(r.z, r.bound)
    assert np.array_equal(r.bits, ref.round_bf16(r.z))
    assert np.abs(vals(r.bits) - r.z).max() <= 2.0 ** -8 * np.abs(r.z).max()


def test_strided_views_are_read_as_logical_arrays():
    # a packed [B, T, (Hq + 2 Hkv) * D] projection output, sliced into Q, K, V views
    B, T, Hq, Hkv, D = 2, 9, 4, 2, 8
    packed = wl.bits(wl.normal((B, T, (Hq + 2 * Hkv) * D), 1.0, "ap.P10"))
    Q = packed[:, :, : Hq * D].reshape(B, T, Hq, D)
    K = packed[:, :, Hq * D: (Hq + Hkv) * D].reshape(B, T, Hkv, D)
    V = packed[:, :, (Hq + Hkv) * D:].reshape(B, T, Hkv, D)
    a = att.attention(Q, K, V).bits
    b = att.attention(Q.copy(), K.copy(), V.copy()).bits
    assert np.array_equal(a, b)
