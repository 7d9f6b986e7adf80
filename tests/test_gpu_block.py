"""GPU parity of fact_norm, fact_rope and fact_block_forward against the block oracle, through the
C ABI.  Tolerances as for the GEMMs (|err| <= 1e-2 bound + 1e-3 per element, Frobenius <= 5e-3), per
stage, each oracle stage fed the bf16 tensor the GPU produced for the stage before (stage-wise
strict); end to end against the oracle's own chain the roundings of eight stored tensors add up
and a flipped bf16 ulp early on moves everything after it, so that comparison is in the
Frobenius norm only (<= 2e-2)."""
import numpy as np
import pytest
import torch

import paper_2604_26666_amd as fact
import workloads as wl
from oracle import block as blk
from oracle import check, ref

pytestmark = pytest.mark.gpu
POISON = 0x7FC1


def dev(bits_or_tensor):
    t = bits_or_tensor if isinstance(bits_or_tensor, torch.Tensor) else wl.from_bits(bits_or_tensor)
    return t.cuda()


def host_bits(t):
    torch.cuda.synchronize()
    return wl.bits(t.cpu().contiguous())


@pytest.mark.parametrize("rms", [0, 1])
@pytest.mark.parametrize("d", [8, 200, 768, 4096, 8192])
def test_norm(rms, d):
    T, pad = 37, 16
    X = wl.normal((T, d), 2.0, f"gb.nX.{d}") + wl.normal((T, 1), 3.0, f"gb.nshift.{d}")        # rows with a mean
    g, b = wl.normal((d,), 1.0, f"gb.ng.{d}"), wl.normal((d,), 0.5, f"gb.nb.{d}")
    Xd = torch.full((T, d + pad), POISON, dtype=torch.int16).view(torch.bfloat16).cuda()
    Xd[:, :d] = X.cuda()
    Yd = torch.full((T + 1, d + pad), POISON, dtype=torch.int16).view(torch.bfloat16).cuda()
    rc = fact.fact_norm(T, d, Xd, d + pad, g.cuda(), None if rms else b.cuda(), 1e-5, rms, Yd, d + pad)
    fact.binding.check(rc, "fact_norm")
    out = host_bits(Yd)
    assert (out[T] == POISON).all() and (out[:, d:] == POISON).all()
    r = blk.rmsnorm(wl.bits(X), wl.bits(g)) if rms else blk.layernorm(wl.bits(X), wl.bits(g), wl.bits(b))
    s = check.assert_close(out[:T, :d], r, what=f"norm rms={rms} d={d}")
    assert s["bits_equal_frac"] > 0.9, s


def test_norm_refusals():
    x = torch.zeros(16, 64, dtype=torch.bfloat16, device="cuda")
    g = torch.ones(64, dtype=torch.bfloat16, device="cuda")
    assert fact.fact_norm(16, 60, x, 64, g, None, 1e-5, 1, x, 64) == -7
    assert fact.fact_norm(16, 64, x, 32, g, None, 1e-5, 1, x, 64) == -2
    assert fact.fact_norm(16, 64, x, 64, g, g, 1e-5, 1, x, 64) == -5
    assert fact.fact_norm(16, 64, None, 64, g, None, 1e-5, 1, x, 64) == -1


@pytest.mark.parametrize("D,base", [(64, 10000.0), (128, 500000.0)])
def test_rope_on_a_packed_buffer(D, base):
    B, T, Hq, Hkv = 2, 300, 4, 2
    W = (Hq + 2 * Hkv) * D
    packed = wl.normal((B, T, W), 1.0, f"gb.rope.{D}")
    d = packed.cuda()
    rc = fact.fact_rope(B, T, Hq + Hkv, D, d, (T * W, W, D), base)
    fact.binding.check(rc, "fact_rope")
    out = host_bits(d)
    pb = wl.bits(packed)
    assert np.array_equal(out[:, :, (Hq + Hkv) * D:], pb[:, :, (Hq + Hkv) * D:])           # the value heads are untouched
    r = blk.rotary(pb[:, :, : (Hq + Hkv) * D].reshape(B, T, Hq + Hkv, D), base)
    s = check.assert_close(np.ascontiguousarray(out[:, :, : (Hq + Hkv) * D]).reshape(-1, D), r, what=f"rope D={D}")
    assert s["bits_equal_frac"] > 0.97, s


def make_block(kind, B, T, d, Hq, Hkv, D, dff):
    n = (Hq + 2 * Hkv) * D
    w = lambda shape, std, name: wl.normal(shape, std, f"gb.{kind}.{name}.{d}")
    p = {"batch": B, "tokens": T, "q_heads": Hq, "kv_heads": Hkv, "head_dim": D, "d_ff": dff, "eps": 1e-5,
         "rms": kind == "llama", "rope": kind == "llama", "rope_base": 500000.0,
         "act": ref.ACT_SILU_GATE if kind == "llama" else ref.ACT_GELU_TANH}
    t = {"norm1_g": w((d,), 1.0, "n1g") , "norm2_g": w((d,), 1.0, "n2g"), "Wqkv": w((n, d), d ** -0.5, "Wqkv"),
         "Wo": w((d, Hq * D), (Hq * D) ** -0.5, "Wo"), "W1": w((dff, d), d ** -0.5, "W1"), "W2": w((d, dff), dff ** -0.5, "W2")}
    if kind == "llama":
        t["W1u"] = w((dff, d), d ** -0.5, "W1u")
    else:
        t.update({"norm1_b": w((d,), 0.5, "n1b"), "norm2_b": w((d,), 0.5, "n2b"), "bqkv": w((n,), 0.1, "bqkv"),
                  "bo": w((d,), 0.1, "bo"), "b1": w((dff,), 0.1, "b1"), "b2": w((d,), 0.1, "b2")})
    p.update({k: wl.bits(v) for k, v in t.items()})
    X = wl.normal((B * T, d), 1.0, f"gb.{kind}.X.{d}")
    return p, t, X


def run_block(p, t, X):
    B, T, Hq, Hkv, D, dff = p["batch"], p["tokens"], p["q_heads"], p["kv_heads"], p["head_dim"], p["d_ff"]
    d = X.shape[1]
    b = fact.Block(B, T, d, Hq, Hkv, D, dff, int(p["rms"]), p["act"], int(p["rope"]), 1e-5, p["rope_base"],
                   **{k: v.cuda() for k, v in t.items()})
    need = fact.fact_block_scratch_bytes(b)
    assert need > 0
    scratch = torch.full((need,), 0xA5, dtype=torch.uint8, device="cuda")
    Y = torch.empty(B * T, d, dtype=torch.bfloat16, device="cuda")
    fact.binding.check(fact.fact_block_forward(b, X.cuda(), Y, scratch, need), "fact_block_forward")
    torch.cuda.synchronize()
    offs = fact.fact_block_scratch_offsets(b)
    n = (Hq + 2 * Hkv) * D
    shapes = {"N1": (B * T, d), "QKVR": (B * T, n), "A": (B * T, Hq * D), "X1": (B * T, d), "N2": (B * T, d), "H": (B * T, dff)}
    raw = scratch.cpu().numpy()
    got = {}
    for name, off in zip(("N1", "QKVR", "A", "X1", "N2", "H"), offs):
        r, c = shapes[name]
        got[name] = raw[off: off + r * c * 2].view(np.uint16).reshape(r, c).copy()
    got["Y"] = host_bits(Y)
    return got


@pytest.mark.parametrize("kind,Hq,Hkv", [("gpt", 4, 4), ("llama", 4, 2)])
def test_small_block_stage_by_stage_and_end_to_end(kind, Hq, Hkv):
    p, t, X = make_block(kind, 2, 200, 256, Hq, Hkv, 64, 512)
    got = run_block(p, t, X)
    own = blk.block_forward(wl.bits(X), p)                                   # the oracle's own chain
    strict = blk.block_forward(wl.bits(X), p, given={k: got[k] for k in ("N1", "QKVR", "A", "X1", "N2", "H")})
    # QKV before the rotary step is not kept by the GPU path; with `given` QKVR the oracle's QKVR stage is
    # computed from given N1 through its own rounded QKV, which is what the GPU does
    for name in ("N1", "QKVR", "A", "X1", "N2", "H", "Y"):
        check.assert_close(got[name], strict[name], what=f"{kind} block stage {name}")
    z = own["Y"].z
    e2e = np.linalg.norm(ref.widen(got["Y"]) - z) / np.linalg.norm(z)
    assert e2e < 2e-2, e2e


def test_block_refusals():
    p, t, X = make_block("gpt", 1, 64, 256, 4, 4, 64, 512)
    w = {k: v.cuda() for k, v in t.items()}
    ok = fact.Block(1, 64, 256, 4, 4, 64, 512, 0, fact.ACT_GELU_TANH, **w)
    need = fact.fact_block_scratch_bytes(ok)
    sc = torch.empty(need, dtype=torch.uint8, device="cuda")
    Y = torch.full((64, 256), POISON, dtype=torch.int16).view(torch.bfloat16).cuda()
    Xd = X.cuda()
    assert fact.fact_block_forward(ok, Xd, Y, sc, need - 1) == -6
    assert fact.fact_block_forward(fact.Block(1, 64, 256, 4, 3, 64, 512, 0, fact.ACT_GELU_TANH, **w), Xd, Y, sc, need) == -2
    assert fact.fact_block_forward(fact.Block(1, 64, 256, 4, 4, 96, 512, 0, fact.ACT_GELU_TANH, **w), Xd, Y, sc, need) == -7
    assert fact.fact_block_forward(fact.Block(1, 64, 256, 4, 4, 64, 512, 0, fact.ACT_SILU_GATE, **w), Xd, Y, sc, need) == -5
    # what only a later stage would refuse is refused before the first launch: the scratch stays untouched
    sc.fill_(0x5A)
    long_seq = fact.Block(1, 1 << 21, 256, 4, 4, 64, 512, 0, fact.ACT_GELU_TANH, **w)      # rows of the packed projection past the attention kernel's 32-bit offsets
    assert fact.fact_block_scratch_bytes(long_seq) == 0 and fact.fact_block_forward(long_seq, Xd, Y, sc, need) == -7
    w_odd = dict(w)
    w_odd["norm2_g"] = torch.zeros(256 + 8, dtype=torch.bfloat16, device="cuda")[4:260]   # 8-byte aligned only: the second norm would refuse it
    assert fact.fact_block_forward(fact.Block(1, 64, 256, 4, 4, 64, 512, 0, fact.ACT_GELU_TANH, **w_odd), Xd, Y, sc, need) == -3
    torch.cuda.synchronize()
    assert (wl.bits(Y.cpu()) == POISON).all() and (sc == 0x5A).all()
    # the two-GEMM block: a workspace the second GEMM could not use is refused before the first GEMM runs
    T, d, dff = 2048, 4096, 14336
    needm = fact.fact_block_mlp_workspace_bytes(T, d, dff, fact.ACT_SILU_GATE)
    if needm > 0:
        z = lambda *shape: torch.zeros(*shape, dtype=torch.bfloat16, device="cuda")
        H = torch.full((T, dff), POISON, dtype=torch.int16).view(torch.bfloat16).cuda()
        wsm = torch.empty(needm + 16, dtype=torch.uint8, device="cuda")
        assert fact.fact_block_mlp(T, d, dff, z(T, d), z(dff, d), z(dff, d), None, fact.ACT_SILU_GATE, z(d, dff), None, None,
                                   H, z(T, d), wsm.data_ptr() + 8, needm) == -3
        torch.cuda.synchronize()
        assert (wl.bits(H.cpu()) == POISON).all()
    assert fact.fact_block_forward(ok, Xd, Y, sc, need) == 0
