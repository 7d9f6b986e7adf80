"""Tolerance check of a bf16 (or fp16) result against the fp64 reference.  TEST INFRASTRUCTURE ONLY.

Pass criteria (the workload definition's): for every element
    |got - z| <= 1e-2 * bound + 1e-3
and over the whole compared block
    ||got - z||_F / ||z||_F <= 5e-3,
where bound is the sum of |a||b| of the GEMM feeding the element (plus |bias|,
|residual|; see ref.gemm_epilogue).  The paper's own criterion (Section 5.1,
rtol 1e-3 / atol 1e-5 against a library result) cannot hold for a bf16 output,
whose half-ulp is 2^-9, and is not used.

A binary16 result (ref.fmt == "f16") is held to the same per-element criterion
and to a tighter norm: its rounding at the store is 2^-12 relative at most
(1.4e-4 in the Frobenius norm for uniformly spread rounding errors) and the
fp32 accumulation adds less than that at the K of the workloads, so
    ||got - z||_F / ||z||_F <= 1e-3.
"""
import numpy as np

from . import ref as _ref

RTOL_BOUND = 1e-2
ATOL = 1e-3
FRO_TOL = 5e-3
FRO_TOL_F16 = 1e-3


def compare(got_bits, ref, rows=None):
    """got_bits: uint16 [*, Nout] holding the rows named by ref.rows (or the full
    output, from which ref.rows are taken when rows == 'full').  Returns a dict."""
    g = _ref.as_bits(got_bits, ref.fmt)
    if rows == "full":
        g = g[ref.rows]
    g = np.ascontiguousarray(g[:, : ref.z.shape[1]])
    got = _ref.widen(g, ref.fmt)
    if got.shape != ref.z.shape:
        raise ValueError(f"shape {got.shape} vs reference {ref.z.shape}")
    err = np.abs(got - ref.z)
    tol = RTOL_BOUND * ref.bound + ATOL
    finite = np.isfinite(got).all()
    ratio = float((err / tol).max()) if err.size else 0.0
    zn = float(np.linalg.norm(ref.z))
    fro = float(np.linalg.norm(got - ref.z)) / zn if zn > 0 else float(np.linalg.norm(got - ref.z))
    # error in units of the output format's spacing at |z| (bf16: 2^-7, binary16: 2^-10 relative to
    # the power of two below |z|; subnormal spacing at the bottom)
    frac_bits, min_ulp = (7, 2.0 ** -133) if ref.fmt == "bf16" else (10, 2.0 ** -24)
    with np.errstate(divide="ignore", invalid="ignore"):
        ulp = np.where(ref.z != 0, np.maximum(2.0 ** (np.floor(np.log2(np.abs(ref.z) + 1e-300)) - frac_bits), min_ulp), min_ulp)
    fro_tol = FRO_TOL if ref.fmt == "bf16" else FRO_TOL_F16
    return {
        "finite": bool(finite),
        "max_abs_err": float(err.max()) if err.size else 0.0,
        "max_err_over_tol": ratio,
        "rel_frobenius": fro,
        "max_err_ulp": float((err / ulp).max()) if err.size else 0.0,
        "bits_equal_frac": float((g == ref.bits).mean()) if err.size else 1.0,
        "elements": int(err.size),
        "ok": bool(finite and ratio <= 1.0 and fro <= fro_tol),
    }


def assert_close(got_bits, ref, rows=None, what=""):
    s = compare(got_bits, ref, rows)
    assert s["ok"], f"{what}: outside tolerance: {s}"
    return s


def assert_bits_equal(got_bits, ref, rows=None, what=""):
    g = _ref.as_bits(got_bits, ref.fmt)
    if rows == "full":
        g = g[ref.rows]
    g = g[:, : ref.bits.shape[1]]
    bad = np.argwhere(g != ref.bits)
    assert bad.size == 0, (f"{what}: {len(bad)} of {ref.bits.size} elements differ in bits; first at "
                           f"{tuple(bad[0])}: got 0x{int(g[tuple(bad[0])]):04x} want 0x{int(ref.bits[tuple(bad[0])]):04x}")
