"""Reference result for fused multi-head attention, in fp64.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
module.  It shares nothing with the HIP path and imports nothing from the
product package.

What is computed: the attention sub-graph that the paper's first block pattern
replaces with one fused kernel (Section 5.2.4 pattern p1, multi-head causal
self-attention; Section 5.2.5 pattern p1, the grouped-query form with fewer
key/value heads than query heads).  The fused
kernel is a re-tiling of the plain definition (Section 2.1: tiling that keeps
the intermediate results on chip), so the oracle is that definition written out, per
batch entry b and query head h:

    g       = h // (Hq / Hkv)                       the key/value head that query head h reads
    S[i][j] = scale * sum_d Q[b,i,h,d] K[b,j,g,d]   fp64
    S[i][j] = -inf  where j > i                     causal mask (a query sees itself and the past)
    P[i][j] = exp(S[i][j] - max_j S[i][j]) / sum_j exp(S[i][j] - max_j S[i][j])
    O[b,i,h,:] = sum_j P[i][j] V[b,j,g,:]
    out     = RNE_bf16(O)                           one rounding, at the store

Readings where the paper is silent.  Head grouping: the paper's block expands
the 8 key/value heads to 32 by repeating each one 4 times in place, so
consecutive query heads share a key/value head (g = h // 4); the oracle indexes
instead of expanding.  Scale: 1 / sqrt(head_dim) unless given.  Inputs are bf16
bit patterns widened exactly; nothing is rounded before the final store.

bound[i][d] = sum_j P[i][j] |V[j][d]| is returned for the tolerance: the fused
kernel rounds P to bf16 before the second contraction, which perturbs each term
of that sum by at most 2^-9 of its magnitude.
"""
import numpy as np

from . import ref as _ref


def attention(Q, K, V, causal=True, scale=None):
    """Q: bf16 bits [B, T, Hq, D]; K, V: bf16 bits [B, T, Hkv, D] (any strides).
    Returns a ref.Ref whose z / bound / bits are [B*T*Hq, D] (rows in [b][t][h] order)."""
    q = _ref.widen(np.ascontiguousarray(_ref.as_bits(Q)))
    k = _ref.widen(np.ascontiguousarray(_ref.as_bits(K)))
    v = _ref.widen(np.ascontiguousarray(_ref.as_bits(V)))
    B, T, Hq, D = q.shape
    Bk, Tk, Hkv, Dk = k.shape
    if (Bk, Tk, Dk) != (B, T, D) or v.shape != k.shape or Hq % Hkv:
        raise ValueError("shapes do not describe grouped-query self-attention")
    if scale is None:
        scale = 1.0 / np.sqrt(float(D))
    group = Hq // Hkv
    z = np.empty((B, T, Hq, D), dtype=np.float64)
    bound = np.empty_like(z)
    future = np.triu(np.ones((T, T), dtype=bool), k=1)          # [i][j] True where j > i
    for b in range(B):
        for h in range(Hq):
            g = h // group
            s = scale * (q[b, :, h, :] @ k[b, :, g, :].T)
            if causal:
                s = np.where(future, -np.inf, s)
            e = np.exp(s - s.max(axis=1, keepdims=True))
            p = e / e.sum(axis=1, keepdims=True)
            z[b, :, h, :] = p @ v[b, :, g, :]
            bound[b, :, h, :] = p @ np.abs(v[b, :, g, :])
    z2 = z.reshape(B * T * Hq, D)
    return _ref.Ref(z=z2, bound=bound.reshape(B * T * Hq, D), bits=_ref.round_bf16(z2),
                    rows=np.arange(B * T * Hq, dtype=np.int64))
