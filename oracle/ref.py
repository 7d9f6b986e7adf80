"""Reference results for bf16 (or fp16) GEMM + fused epilogue, in fp64.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this module.  It shares nothing with the HIP path and imports nothing from the
product package.

What is computed, in the order the paper's patterns apply it (Section 5.2.4,
pattern "MLP with GELU": a linear projection with an activation epilogue then a
linear projection with a standard epilogue; Section 5.2.5, pattern "SwiGLU
MLP": gate projection with SiLU, up projection, elementwise product, then the
down projection):

    acc = A x B                       fp64 sum over ascending k (fact_oracle.c)
    z   = acc + bias[j]               bias before the activation
    z   = act(z)                      none | GELU (tanh form) | SiLU(gate) * up
    z   = z + residual[i][j]          residual after the activation
    out = RNE_bf16(z)                 one rounding, at the store

Readings where the paper is silent: the paper says only "GELU"; the tanh form
is used (fixed by the workload definition).  The paper never mentions bias or
residual; the order above is the transformer-block convention.  Inputs are
bf16 (the paper uses tf32/fp16); accumulation here is fp64.

The contraction and the bf16 conversions are in fact_oracle.c; the epilogue is
written out below with numpy fp64 operations.

fmt="f16" everywhere below means that every 16-bit pattern (A, B, bias,
residual, the output) is IEEE binary16, the precision of the paper's own kernels
(Listing 1; Sections 5.2.3 - 5.2.5), instead of bf16; nothing else changes.
"""
import ctypes
import os
from dataclasses import dataclass

import numpy as np

from . import build as _build

ACT_NONE = 0
ACT_GELU_TANH = 1
ACT_SILU_GATE = 2

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path):
            _build.build(force=True)
        L = ctypes.CDLL(path)
        i64, p = ctypes.c_int64, ctypes.c_void_p
        L.orc_gemm_f64.argtypes = [i64, i64, i64, p, i64, p, i64, ctypes.c_int, p, i64, p, p]
        L.orc_gemm_f64.restype = ctypes.c_int
        L.orc_bf16_from_f64.argtypes = [ctypes.c_double]
        L.orc_bf16_from_f64.restype = ctypes.c_uint16
        L.orc_bf16_to_f64.argtypes = [ctypes.c_uint16]
        L.orc_bf16_to_f64.restype = ctypes.c_double
        L.orc_bf16_from_f64_array.argtypes = [p, p, i64]
        L.orc_bf16_from_f64_array.restype = None
        L.orc_bf16_to_f64_array.argtypes = [p, p, i64]
        L.orc_bf16_to_f64_array.restype = None
        L.orc_gemm_f64_f16.argtypes = L.orc_gemm_f64.argtypes
        L.orc_gemm_f64_f16.restype = ctypes.c_int
        L.orc_f16_from_f64.argtypes = [ctypes.c_double]
        L.orc_f16_from_f64.restype = ctypes.c_uint16
        L.orc_f16_to_f64.argtypes = [ctypes.c_uint16]
        L.orc_f16_to_f64.restype = ctypes.c_double
        L.orc_f16_from_f64_array.argtypes = [p, p, i64]
        L.orc_f16_from_f64_array.restype = None
        L.orc_f16_to_f64_array.argtypes = [p, p, i64]
        L.orc_f16_to_f64_array.restype = None
        L.orc_num_threads.argtypes = []
        L.orc_num_threads.restype = ctypes.c_int
        _lib = L
    return _lib


def num_threads():
    return int(lib().orc_num_threads())


# ---- bf16 bit patterns ------------------------------------------------------

def _check_fmt(fmt):
    if fmt not in ("bf16", "f16"):
        raise ValueError(f"unknown 16-bit format {fmt!r}")
    return fmt


def as_bits(x, fmt="bf16"):
    """View a 16-bit float array (numpy uint16, or a CPU torch tensor of the format's dtype) as numpy uint16."""
    _check_fmt(fmt)
    if isinstance(x, np.ndarray):
        if x.dtype != np.uint16:
            raise TypeError("16-bit float data must be given as uint16 bit patterns")
        return x
    import torch  # only to unwrap a tensor; no torch arithmetic is used here
    if isinstance(x, torch.Tensor):
        want = torch.bfloat16 if fmt == "bf16" else torch.float16
        if x.dtype != want or x.device.type != "cpu":
            raise TypeError(f"expected a CPU {want} tensor")
        return x.view(torch.int16).numpy().view(np.uint16)
    raise TypeError(type(x))


def widen(bits, fmt="bf16"):
    """16-bit patterns -> fp64 values (exact)."""
    b = np.ascontiguousarray(as_bits(bits, fmt))
    out = np.empty(b.shape, dtype=np.float64)
    f = lib().orc_bf16_to_f64_array if _check_fmt(fmt) == "bf16" else lib().orc_f16_to_f64_array
    f(b.ctypes.data, out.ctypes.data, b.size)
    return out


def round_bf16(z):
    """fp64 values -> bf16 bit patterns, round to nearest, ties to even, one rounding."""
    z = np.ascontiguousarray(z, dtype=np.float64)
    out = np.empty(z.shape, dtype=np.uint16)
    lib().orc_bf16_from_f64_array(z.ctypes.data, out.ctypes.data, z.size)
    return out


def round_f16(z):
    """fp64 values -> binary16 bit patterns, round to nearest, ties to even, one rounding."""
    z = np.ascontiguousarray(z, dtype=np.float64)
    out = np.empty(z.shape, dtype=np.uint16)
    lib().orc_f16_from_f64_array(z.ctypes.data, out.ctypes.data, z.size)
    return out


def round_to(z, fmt="bf16"):
    return round_bf16(z) if _check_fmt(fmt) == "bf16" else round_f16(z)


def _ld(a):
    """Leading dimension in elements of a 2-D uint16 array with unit inner stride."""
    if a.ndim != 2 or (a.shape[1] > 1 and a.strides[1] != 2):
        raise ValueError("matrix must be 2-D, row-major, inner stride 1")
    if a.shape[0] == 1:          # numpy leaves the stride of a length-1 axis arbitrary
        return a.shape[1]
    if a.strides[0] % 2 or a.strides[0] < 2 * a.shape[1]:
        raise ValueError("matrix must be 2-D, row-major, inner stride 1")
    return a.strides[0] // 2


# ---- the contraction --------------------------------------------------------

def gemm(A, B, trans_b=False, rows=None, fmt="bf16"):
    """acc[r][j] = sum_k A[rows[r]][k] * B[k][j] and bound = sum_k |a||b|, both fp64.

    A is [M, K].  B is [K, N] (trans_b False) or [N, K] (trans_b True).  rows is
    an optional 1-D list of row indices; default all rows.  Returns (acc, bound),
    each [len(rows), N].
    """
    A = as_bits(A, fmt)
    B = as_bits(B, fmt)
    M, K = A.shape
    if trans_b:
        N, Kb = B.shape
    else:
        Kb, N = B.shape
    if Kb != K:
        raise ValueError("inner dimensions differ")
    if rows is None:
        rows_arr, nrows, rows_ptr = None, M, None
    else:
        rows_arr = np.ascontiguousarray(rows, dtype=np.int64)
        nrows, rows_ptr = rows_arr.size, rows_arr.ctypes.data
    acc = np.empty((nrows, N), dtype=np.float64)
    bound = np.empty((nrows, N), dtype=np.float64)
    f = lib().orc_gemm_f64 if _check_fmt(fmt) == "bf16" else lib().orc_gemm_f64_f16
    rc = f(M, N, K, A.ctypes.data, _ld(A), B.ctypes.data, _ld(B),
          1 if trans_b else 0, rows_ptr, nrows,
          acc.ctypes.data, bound.ctypes.data)
    if rc != 0:
        raise ValueError("orc_gemm_f64 rejected its arguments")
    return acc, bound


# ---- activations, fp64 ------------------------------------------------------

def gelu_tanh(z):
    """0.5 z (1 + tanh( sqrt(2/pi) (z + 0.044715 z^3) ))."""
    z = np.asarray(z, dtype=np.float64)
    return 0.5 * z * (1.0 + np.tanh(np.sqrt(2.0 / np.pi) * (z + 0.044715 * z ** 3)))


def silu(z):
    """z / (1 + exp(-z))."""
    z = np.asarray(z, dtype=np.float64)
    with np.errstate(over="ignore"):
        return z / (1.0 + np.exp(-z))


# ---- GEMM + epilogue --------------------------------------------------------

@dataclass
class Ref:
    z: np.ndarray        # fp64 result before the final rounding, [nrows, Nout]
    bound: np.ndarray    # fp64 magnitude bound the tolerance scales with, same shape
    bits: np.ndarray     # uint16: RNE(z) in the output format
    rows: np.ndarray     # which rows of the full output these are
    fmt: str = "bf16"    # the 16-bit format of bits


def gemm_epilogue(A, B, trans_b=False, bias=None, residual=None, act=ACT_NONE, rows=None, fmt="bf16"):
    """One fused GEMM: acc -> +bias -> act -> +residual -> bf16.

    With ACT_SILU_GATE, B must be [2I, K] with trans_b True: rows 0..I-1 are the
    gate projection, rows I..2I-1 the up projection; the output has I columns and
    bias must be None.

    The returned bound is the magnitude that the per-element tolerance scales
    with: sum_k |a||b| of the GEMM feeding the element, plus |bias| and
    |residual|; for the gated product the product rule with |SiLU'| <= 1.1:
    1.1 bound_g |u| + |SiLU(g)| bound_u.
    """
    acc, bnd = gemm(A, B, trans_b, rows, fmt)
    M = as_bits(A, fmt).shape[0]
    rows_arr = np.arange(M, dtype=np.int64) if rows is None else np.asarray(rows, dtype=np.int64)

    if act == ACT_SILU_GATE:
        if bias is not None:
            raise ValueError("bias is not defined for the gated epilogue")
        if not trans_b or acc.shape[1] % 2:
            raise ValueError("gated epilogue needs B = [2I, K], trans_b")
        half = acc.shape[1] // 2
        g, u = acc[:, :half], acc[:, half:]
        bg, bu = bnd[:, :half], bnd[:, half:]
        sg = silu(g)
        z = sg * u
        bound = 1.1 * bg * np.abs(u) + np.abs(sg) * bu
    else:
        z = acc
        bound = bnd
        if bias is not None:
            b = widen(bias, fmt).reshape(1, -1)
            if b.shape[1] != z.shape[1]:
                raise ValueError("bias length")
            z = z + b
            bound = bound + np.abs(b)
        if act == ACT_GELU_TANH:
            z = gelu_tanh(z)
        elif act != ACT_NONE:
            raise ValueError("unknown activation")

    if residual is not None:
        r = widen(np.ascontiguousarray(as_bits(residual, fmt)[rows_arr, : z.shape[1]]), fmt)
        z = z + r
        bound = bound + np.abs(r)
    return Ref(z=z, bound=bound, bits=round_to(z, fmt), rows=rows_arr, fmt=fmt)


def block_mlp(X, W1, W1u, b1, act, W2, b2, R, rows=None, H_bits=None, fmt="bf16"):
    """Two-GEMM feed-forward block (Sections 5.2.4 and 5.2.5).

    H = act(X W1^T + b1), rounded to the 16-bit format (bf16, or binary16 with
    fmt="f16") because it is stored in it between the two GEMMs;  Y = H W2^T + b2 + R.  W1 is [d_ff, d]; with ACT_SILU_GATE W1
    is the gate weight and W1u the up weight, each [d_ff, d].  W2 is [d, d_ff].

    If H_bits is given (the bf16 H another implementation produced, all rows),
    the second stage consumes it instead of the oracle's own H: the stage-wise
    strict check.  Returns (ref_H, ref_Y).
    """
    W1 = as_bits(W1, fmt)
    if act == ACT_SILU_GATE:
        W = np.concatenate([W1, as_bits(W1u, fmt)], axis=0)
        ref_h = gemm_epilogue(X, W, True, None, None, ACT_SILU_GATE, rows, fmt)
    else:
        ref_h = gemm_epilogue(X, W1, True, b1, None, act, rows, fmt)
    if H_bits is None:
        H = ref_h.bits
        ref_y = gemm_epilogue(H, W2, True, b2, None, ACT_NONE, None, fmt)
        if R is not None:
            r = widen(np.ascontiguousarray(as_bits(R, fmt)[ref_h.rows, : ref_y.z.shape[1]]), fmt)
            z = ref_y.z + r
            ref_y = Ref(z=z, bound=ref_y.bound + np.abs(r), bits=round_to(z, fmt), rows=ref_h.rows, fmt=fmt)
        else:
            ref_y = Ref(z=ref_y.z, bound=ref_y.bound, bits=ref_y.bits, rows=ref_h.rows, fmt=fmt)
    else:
        ref_y = gemm_epilogue(as_bits(H_bits, fmt), W2, True, b2, R, ACT_NONE, ref_h.rows, fmt)
    return ref_h, ref_y
