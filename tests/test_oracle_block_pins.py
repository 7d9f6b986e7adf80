"""Pins of the block oracle's norm / rotary pieces and of its wiring (CPU only)."""
import math

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import block as blk
from oracle import ref


def bits(x):
    return ref.round_bf16(np.asarray(x, dtype=np.float64))


def test_layernorm_output_has_zero_mean_unit_variance_and_matches_library():
    X = wl.normal((9, 96), 3.0, "bp.X1")
    ones, zeros = bits(np.ones(96)), bits(np.zeros(96))
    z = blk.layernorm(wl.bits(X), ones, zeros, eps=0.0).z
    assert np.abs(z.mean(axis=1)).max() < 1e-13 and np.abs((z * z).mean(axis=1) - 1).max() < 1e-12
    g, b = wl.normal((96,), 1.0, "bp.g1"), wl.normal((96,), 1.0, "bp.b1")
    want = torch.nn.functional.layer_norm(X.double(), (96,), g.double(), b.double(), eps=1e-5).numpy()
    assert np.abs(blk.layernorm(wl.bits(X), wl.bits(g), wl.bits(b)).z - want).max() < 1e-12
    # a constant row has no variance: the output is beta (eps keeps the division finite)
    c = blk.layernorm(bits(np.full((1, 96), 2.5)), wl.bits(g), wl.bits(b)).z
    assert np.abs(c - ref.widen(wl.bits(b))).max() < 1e-12


def test_rmsnorm_closed_forms_and_library():
    g = wl.normal((64,), 1.0, "bp.g2")
    gv = ref.widen(wl.bits(g))
    x = np.full((1, 64), -4.0)                       # rms = 4 -> x / rms = -1
    assert np.abs(blk.rmsnorm(bits(x), wl.bits(g), eps=0.0).z + gv).max() < 1e-15
    x = np.zeros((1, 64)); x[0, 5] = 8.0             # rms = 8 / sqrt(64) = 1
    z = blk.rmsnorm(bits(x), wl.bits(g), eps=0.0).z
    assert abs(z[0, 5] - 8.0 * gv[5]) < 1e-14 and np.abs(np.delete(z[0], 5)).max() == 0
    X = wl.normal((7, 64), 2.0, "bp.X2")
    xd = X.double()
    want = (xd * torch.rsqrt((xd * xd).mean(-1, keepdim=True) + 1e-5) * g.double()).numpy()
    assert np.abs(blk.rmsnorm(wl.bits(X), wl.bits(g)).z - want).max() < 1e-12
    # scale invariance up to eps: rmsnorm(4 x) = rmsnorm(x)
    a = blk.rmsnorm(wl.bits(X), wl.bits(g), eps=0.0).z
    b = blk.rmsnorm(bits(4.0 * ref.widen(wl.bits(X))), wl.bits(g), eps=0.0).z
    assert np.abs(a - b).max() < 1e-12


def test_rotary_is_a_rotation_by_position_times_frequency():
    # D = 2: one pair, frequency base^0 = 1: token t is rotated by t radians
    x = np.zeros((1, 4, 1, 2)); x[0, :, 0, 0] = 1.0; x[0, :, 0, 1] = 0.5
    z = blk.rotary(bits(x), base=10000.0).z.reshape(4, 2)
    for t in range(4):
        assert abs(z[t, 0] - (math.cos(t) - 0.5 * math.sin(t))) < 1e-15
        assert abs(z[t, 1] - (0.5 * math.cos(t) + math.sin(t))) < 1e-15
    # D = 4, base 16: pair 0 = (x0, x2) at frequency 1, pair 1 = (x1, x3) at frequency 16^(-1/2) = 1/4
    x = np.zeros((1, 3, 1, 4)); x[0, 2, 0] = [1.0, 2.0, 0.0, 0.0]
    z = blk.rotary(bits(x), base=16.0).z.reshape(3, 4)
    assert np.allclose(z[2], [math.cos(2.0), 2 * math.cos(0.5), math.sin(2.0), 2 * math.sin(0.5)], atol=1e-15, rtol=0)


def test_rotary_invariants():
    B, T, H, D = 2, 17, 3, 16
    X = wl.bits(wl.normal((B, T, H, D), 1.0, "bp.X3"))
    x = ref.widen(X)
    z = blk.rotary(X).z.reshape(B, T, H, D)
    assert np.array_equal(z[:, 0], x[:, 0])                                   # position 0: identity
    half = D // 2
    assert np.abs((z[..., :half] ** 2 + z[..., half:] ** 2) - (x[..., :half] ** 2 + x[..., half:] ** 2)).max() < 1e-12
    # the score of a rotated query and key depends on their distance only
    q = np.broadcast_to(x[0, 0, 0], (1, T, 1, D)); k = np.broadcast_to(x[1, 3, 1], (1, T, 1, D))
    zq = blk.rotary(bits(q), base=100.0).z.reshape(T, D); zk = blk.rotary(bits(k), base=100.0).z.reshape(T, D)
    s = zq @ zk.T
    for d in range(-3, 4):
        diag = np.diagonal(s, offset=d)
        assert np.abs(diag - diag[0]).max() < 1e-11


def _params(kind, B=1, T=24):
    if kind == "llama":
        Hq, Hkv, D, d, dff = 4, 2, 16, 64, 96
    else:
        Hq, Hkv, D, d, dff = 4, 4, 16, 64, 128
    n = (Hq + 2 * Hkv) * D
    w = lambda shape, std, name: wl.bits(wl.normal(shape, std, f"bp.{kind}.{name}"))
    p = {"batch": B, "tokens": T, "q_heads": Hq, "kv_heads": Hkv, "head_dim": D, "d_ff": dff, "eps": 1e-5,
         "rms": kind == "llama", "rope": kind == "llama", "rope_base": 500000.0,
         "act": ref.ACT_SILU_GATE if kind == "llama" else ref.ACT_GELU_TANH,
         "norm1_g": w((d,), 1.0, "n1g"), "norm2_g": w((d,), 1.0, "n2g"),
         "Wqkv": w((n, d), 0.1, "Wqkv"), "Wo": w((d, Hq * D), 0.1, "Wo"), "W1": w((dff, d), 0.1, "W1"), "W2": w((d, dff), 0.1, "W2")}
    if kind == "llama":
        p["W1u"] = w((dff, d), 0.1, "W1u")
    else:
        p.update({"norm1_b": w((d,), 0.5, "n1b"), "norm2_b": w((d,), 0.5, "n2b"), "bqkv": w((n,), 0.1, "bqkv"),
                  "bo": w((d,), 0.1, "bo"), "b1": w((dff,), 0.1, "b1"), "b2": w((d,), 0.1, "b2")})
    return p, wl.bits(wl.normal((B * T, d), 1.0, f"bp.{kind}.X"))


@pytest.mark.parametrize("kind", ["gpt", "llama"])
def test_block_wiring_against_torch_fp64_without_intermediate_rounding(kind):
    """The same block written with torch fp64 library routines and NO rounding between stages
    agrees with the oracle to within the accumulated bf16 roundings of its eight stored tensors."""
    p, X = _params(kind)
    out = blk.block_forward(X, p)
    t = lambda a: torch.from_numpy(ref.widen(a))
    B, T, Hq, Hkv, D = p["batch"], p["tokens"], p["q_heads"], p["kv_heads"], p["head_dim"]
    x = t(X)
    if kind == "llama":
        norm = lambda v, g, b: v * torch.rsqrt((v * v).mean(-1, keepdim=True) + 1e-5) * t(g)
    else:
        norm = lambda v, g, b: torch.nn.functional.layer_norm(v, (v.shape[-1],), t(g), t(b), eps=1e-5)
    n1 = norm(x, p["norm1_g"], p.get("norm1_b"))
    qkv = n1 @ t(p["Wqkv"]).T + (t(p["bqkv"]) if "bqkv" in p else 0)
    q = qkv[:, : Hq * D].reshape(B, T, Hq, D); k = qkv[:, Hq * D: (Hq + Hkv) * D].reshape(B, T, Hkv, D)
    v = qkv[:, (Hq + Hkv) * D:].reshape(B, T, Hkv, D)
    if kind == "llama":
        def rot(u):
            half = D // 2
            inv = 500000.0 ** (-2.0 * torch.arange(half, dtype=torch.float64) / D)
            ang = torch.arange(T, dtype=torch.float64)[:, None] * inv[None, :]
            c, s = torch.cos(ang)[None, :, None, :], torch.sin(ang)[None, :, None, :]
            lo, hi = u[..., :half], u[..., half:]
            return torch.cat([lo * c - hi * s, hi * c + lo * s], -1)
        q, k = rot(q), rot(k)
    kk = k.repeat_interleave(Hq // Hkv, dim=2); vv = v.repeat_interleave(Hq // Hkv, dim=2)
    a = torch.nn.functional.scaled_dot_product_attention(q.transpose(1, 2), kk.transpose(1, 2), vv.transpose(1, 2), is_causal=True)
    a = a.transpose(1, 2).reshape(B * T, Hq * D)
    x1 = a @ t(p["Wo"]).T + (t(p["bo"]) if "bo" in p else 0) + x
    n2 = norm(x1, p["norm2_g"], p.get("norm2_b"))
    if kind == "llama":
        h = torch.nn.functional.silu(n2 @ t(p["W1"]).T) * (n2 @ t(p["W1u"]).T)
    else:
        h = torch.nn.functional.gelu(n2 @ t(p["W1"]).T + t(p["b1"]), approximate="tanh")
    y = h @ t(p["W2"]).T + (t(p["b2"]) if "b2" in p else 0) + x1
    err = np.abs(out["Y"].z - y.numpy()).max() / np.abs(y.numpy()).max()
    assert err < 2e-2, err
    # stage by stage the definitions are exact: feed each oracle stage torch's UNROUNDED input and compare
    assert np.abs(out["N1"].z - n1.numpy()).max() < 1e-12


def test_given_inputs_replace_the_oracles_own():
    p, X = _params("gpt")
    out = blk.block_forward(X, p)
    other = out["N1"].bits.copy(); other[0, 0] ^= 0x0100
    out2 = blk.block_forward(X, p, given={"N1": other})
    assert not np.array_equal(out["QKV"].bits[0], out2["QKV"].bits[0])
    assert np.array_equal(out["QKV"].bits[1:], out2["QKV"].bits[1:])
