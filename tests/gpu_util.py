"""Helpers for the GPU parity tests: move seeded inputs to the device (PyTorch is used for
device memory and streams only), call the C ABI through the binding, bring bits back."""
import numpy as np
import torch

import paper_2604_26666_amd as fact
import workloads as wl

POISON = 0x7FC1      # a NaN pattern the library never produces


def to_dev(t):
    return None if t is None else t.cuda()


def bits_of(t):
    torch.cuda.synchronize()
    return wl.bits(t.cpu().contiguous())


def poisoned(rows, cols):
    """bf16 device matrix [rows, cols] filled with the poison pattern."""
    return torch.full((rows, cols), POISON, dtype=torch.int16).view(torch.bfloat16).cuda()


def padded(t, pad):
    """Device copy of a 2-D CPU tensor inside a buffer whose rows are `pad` elements longer,
    padding poisoned.  Returns (buffer, view, ld)."""
    r, c = t.shape
    buf = poisoned(r, c + pad)
    buf[:, :c] = t.cuda()
    return buf, buf[:, :c], c + pad


def gemm(A, B, trans_b, bias=None, residual=None, act=fact.ACT_NONE, cfg=-1, split=0, group_m=0,
         pad=0, entry="auto", in_place=False, return_ws=None):
    """Runs one GEMM on the GPU; A, B, bias, residual are CPU bf16 tensors.  Returns the
    uint16 output [M, Nout] and checks that nothing outside it was written."""
    M, K = A.shape
    N = B.shape[0] if trans_b else B.shape[1]
    nout = N // 2 if act == fact.ACT_SILU_GATE else N
    Ab, Av, lda = padded(A, pad)
    Bb, Bv, ldb = padded(B, pad)
    Cb = poisoned(M + 1, nout + pad + 8)          # one guard row, guard columns
    ldc = nout + pad + 8
    bias_d = to_dev(bias)
    if residual is not None:
        if in_place:
            Cb[:M, :nout] = residual.cuda()
            res_ptr, ldr = Cb, ldc
        else:
            Rb, Rv, ldr = padded(residual, pad)
            res_ptr = Rb
    else:
        res_ptr, ldr = None, 0
    ep = fact.Epilogue(bias=bias_d, residual=res_ptr, ldr=ldr, act=act)
    ws, ws_bytes = None, 0
    if entry == "auto":
        entry = "ex" if (cfg >= 0 or group_m > 0) else ("splitk" if split != 0 else "gemm")
    if entry in ("ex", "splitk") and split != 1:
        ws_bytes = max(fact.fact_gemm_splitk_workspace_bytes(M, N, K, split), 16)
        ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda").fill_(0xA5)      # contents are scratch: no clearing needed
    if entry == "gemm":
        rc = fact.fact_gemm(M, N, K, Ab, lda, Bb, ldb, trans_b, Cb, ldc, ep)
    elif entry == "splitk":
        rc = fact.fact_gemm_splitk(M, N, K, Ab, lda, Bb, ldb, trans_b, Cb, ldc, ep, split, ws, ws_bytes)
    else:
        rc = fact.fact_gemm_ex(1, M, N, K, Ab, lda, 0, Bb, ldb, 0, trans_b, Cb, ldc, 0, ep, cfg, split, group_m,
                               ws, ws_bytes)
    fact.binding.check(rc, f"{entry} M={M} N={N} K={K} tb={trans_b} act={act} cfg={cfg} split={split}")
    if return_ws is not None:
        return_ws.append(ws)
    out = bits_of(Cb)
    assert (out[M, :] == POISON).all() and (out[:, nout:] == POISON).all(), "wrote outside C"
    return out[:M, :nout].copy()
