"""Reference results for the pieces around attention and the feed-forward network in a
transformer block, and for the whole block, in fp64.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this module.  It
shares nothing with the HIP path and imports nothing from the product package.

The paper evaluates two blocks (Section 5.1): a GPT-style block with LayerNorm and a GELU
feed-forward network, and a Llama-3-8B decoder block with RMSNorm, grouped-query attention and a
SwiGLU feed-forward network.  Its method replaces the attention and feed-forward sub-graphs
(Sections 5.2.4, 5.2.5) and leaves the rest to the framework; here the rest is written out too,
in the usual pre-norm arrangement (the paper does not spell the block out - readings below):

    N1  = norm(X)                                   LayerNorm (gamma, beta) or RMSNorm (gamma)
    QKV = N1 Wqkv^T + bqkv                          per token: query heads | key heads | value heads
    q, k <- rotary(q, k)                            Llama-style blocks only
    A   = attention(QKV), causal                    oracle.attention
    X1  = A Wo^T + bo + X
    N2  = norm(X1)
    H   = act(N2 W1^T + b1)                         GELU(tanh), or SiLU(N2 Wg^T) * (N2 Wu^T)
    Y   = H W2^T + b2 + X1

Every tensor named on the left lives in memory as bf16, so it is rounded (nearest even) where
it is produced, and the next stage reads the rounded values: the same rule as for H in the
two-GEMM block.

Definitions (fp64, on the widened bf16 inputs):
  LayerNorm: y = (x - mean(x)) / sqrt(var(x) + eps) * gamma + beta, var = mean((x - mean)^2).
  RMSNorm:   y = x / sqrt(mean(x^2) + eps) * gamma.
  Rotary embedding, "rotate-half" pairing (the Llama convention): within a head of width D, for
  i < D/2 and token position t (0-based inside its sequence), angle = t * base^(-2 i / D):
      y_i       = x_i cos(angle) - x_{i + D/2} sin(angle)
      y_{i+D/2} = x_{i + D/2} cos(angle) + x_i sin(angle).
Readings: pre-norm residual arrangement; eps 1e-5; rotary base 500000 (the Llama-3 value) unless
given; positions restart at 0 in every batch entry.
"""
import numpy as np

from . import attention as _att
from . import ref as _ref


def layernorm(X, gamma, beta=None, eps=1e-5):
    """X: bf16 bits [T, d]; gamma, beta: bf16 bits [d].  Returns ref.Ref ([T, d])."""
    x = _ref.widen(np.ascontiguousarray(_ref.as_bits(X)))
    g = _ref.widen(_ref.as_bits(gamma)).reshape(1, -1)
    mean = x.mean(axis=1, keepdims=True)
    xc = x - mean
    var = (xc * xc).mean(axis=1, keepdims=True)
    z = xc / np.sqrt(var + eps) * g
    bound = np.abs(z)
    if beta is not None:
        b = _ref.widen(_ref.as_bits(beta)).reshape(1, -1)
        z = z + b
        bound = bound + np.abs(b)
    return _ref.Ref(z=z, bound=bound, bits=_ref.round_bf16(z), rows=np.arange(x.shape[0], dtype=np.int64))


def rmsnorm(X, gamma, eps=1e-5):
    x = _ref.widen(np.ascontiguousarray(_ref.as_bits(X)))
    g = _ref.widen(_ref.as_bits(gamma)).reshape(1, -1)
    z = x / np.sqrt((x * x).mean(axis=1, keepdims=True) + eps) * g
    return _ref.Ref(z=z, bound=np.abs(z), bits=_ref.round_bf16(z), rows=np.arange(x.shape[0], dtype=np.int64))


def rotary(X, base=500000.0):
    """X: bf16 bits [B, T, H, D] (any strides).  Returns ref.Ref with z / bits [B*T*H, D]."""
    x = _ref.widen(np.ascontiguousarray(_ref.as_bits(X)))
    B, T, H, D = x.shape
    half = D // 2
    i = np.arange(half, dtype=np.float64)
    ang = np.arange(T, dtype=np.float64).reshape(T, 1) * (float(base) ** (-2.0 * i / D)).reshape(1, half)
    c, s = np.cos(ang).reshape(1, T, 1, half), np.sin(ang).reshape(1, T, 1, half)
    lo, hi = x[..., :half], x[..., half:]
    z = np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=-1)
    bound = np.concatenate([np.abs(lo * c) + np.abs(hi * s), np.abs(hi * c) + np.abs(lo * s)], axis=-1)
    z2 = z.reshape(B * T * H, D)
    return _ref.Ref(z=z2, bound=bound.reshape(B * T * H, D), bits=_ref.round_bf16(z2), rows=np.arange(B * T * H, dtype=np.int64))


def block_forward(X, p, given=None):
    """The whole block.  X: bf16 bits [B*T, d].  p: dict with batch, tokens, q_heads, kv_heads, head_dim,
    d_ff, rms (bool), rope (bool), rope_base, eps, act, and bf16-bit arrays norm1_g, norm1_b, Wqkv
    [(Hq + 2 Hkv) D, d], bqkv, Wo [d, Hq D], bo, norm2_g, norm2_b, W1 [d_ff, d], W1u, b1, W2 [d, d_ff], b2
    (absent / None where the block has none).
    given: optional dict of bf16-bit tensors another implementation produced for the stage names
    below; a stage whose INPUT is in `given` consumes that instead of the oracle's own (the
    stage-wise strict check).  Returns a dict stage name -> ref.Ref, stages
    N1, QKV, QKVR (after rotary; equals QKV without), A, X1, N2, H, Y."""
    given = given or {}
    B, T, Hq, Hkv, D = p["batch"], p["tokens"], p["q_heads"], p["kv_heads"], p["head_dim"]
    eps = p.get("eps", 1e-5)
    Xb = np.ascontiguousarray(_ref.as_bits(X))
    out = {}

    def have(name):
        return np.ascontiguousarray(_ref.as_bits(given[name])) if name in given else out[name].bits

    norm = (lambda x, g, b: rmsnorm(x, g, eps)) if p["rms"] else (lambda x, g, b: layernorm(x, g, b, eps))
    out["N1"] = norm(Xb, p["norm1_g"], p.get("norm1_b"))
    out["QKV"] = _ref.gemm_epilogue(have("N1"), p["Wqkv"], True, bias=p.get("bqkv"))
    qkv = have("QKV").reshape(B, T, (Hq + 2 * Hkv) * D)
    if p.get("rope"):
        qk = qkv[:, :, : (Hq + Hkv) * D].reshape(B, T, Hq + Hkv, D)
        r = rotary(qk, p.get("rope_base", 500000.0))
        zfull = np.concatenate([r.z.reshape(B, T, (Hq + Hkv) * D), _ref.widen(qkv[:, :, (Hq + Hkv) * D:])], axis=2)
        bfull = np.concatenate([r.bound.reshape(B, T, (Hq + Hkv) * D), np.abs(_ref.widen(qkv[:, :, (Hq + Hkv) * D:]))], axis=2)
        z2 = zfull.reshape(B * T, -1)
        out["QKVR"] = _ref.Ref(z=z2, bound=bfull.reshape(B * T, -1), bits=_ref.round_bf16(z2), rows=np.arange(B * T, dtype=np.int64))
    else:
        out["QKVR"] = out["QKV"] if "QKV" not in given else _ref.Ref(z=_ref.widen(have("QKV")), bound=np.abs(_ref.widen(have("QKV"))), bits=have("QKV"), rows=np.arange(B * T, dtype=np.int64))
    qkvr = have("QKVR").reshape(B, T, (Hq + 2 * Hkv) * D)
    q = qkvr[:, :, : Hq * D].reshape(B, T, Hq, D)
    k = qkvr[:, :, Hq * D: (Hq + Hkv) * D].reshape(B, T, Hkv, D)
    v = qkvr[:, :, (Hq + Hkv) * D:].reshape(B, T, Hkv, D)
    a = _att.attention(q, k, v, causal=True)
    out["A"] = _ref.Ref(z=a.z.reshape(B * T, Hq * D), bound=a.bound.reshape(B * T, Hq * D), bits=a.bits.reshape(B * T, Hq * D),
                        rows=np.arange(B * T, dtype=np.int64))
    out["X1"] = _ref.gemm_epilogue(have("A"), p["Wo"], True, bias=p.get("bo"), residual=Xb)
    out["N2"] = norm(have("X1"), p["norm2_g"], p.get("norm2_b"))
    if p["act"] == _ref.ACT_SILU_GATE:
        W = np.concatenate([_ref.as_bits(p["W1"]), _ref.as_bits(p["W1u"])], axis=0)
        out["H"] = _ref.gemm_epilogue(have("N2"), W, True, act=_ref.ACT_SILU_GATE)
    else:
        out["H"] = _ref.gemm_epilogue(have("N2"), p["W1"], True, bias=p.get("b1"), act=p["act"])
    out["Y"] = _ref.gemm_epilogue(have("H"), p["W2"], True, bias=p.get("b2"), residual=have("X1"))
    return out
