"""Seeded synthetic inputs for the five benchmark configurations.

This module serves both the CPU oracle's tests and the GPU tests / benchmark.
It holds none of the method's arithmetic: it draws fp32 numbers from torch's
CPU generator and lets torch convert them to bfloat16 (a library routine).
Every tensor is a CPU torch.bfloat16 tensor; `bits()` views one as uint16.

The shapes and value distributions are those of the workload definition: the
three GEMM problems follow the paper's Section 5.1 "Benchmark problems"
(square, batched, large-K; here in bf16 and at the sizes the workload fixes),
the two block configurations take the layer shapes of Sections 5.2.4
(768 -> 3072 -> 768, GELU) and 5.2.5 (4096 -> 14336 -> 4096, SwiGLU, 32 query /
8 key-value heads of width 128).  They stand in for the benchmark-suite
problems and the model block the paper measured, none of which is available.
The seed is the paper's (Section 5.1: seed 42).
"""
import zlib

import numpy as np
import torch

SEED = 42


def _generator(name):
    g = torch.Generator(device="cpu")
    g.manual_seed((SEED * 1000003 + zlib.crc32(name.encode())) & 0x7FFFFFFFFFFFFFFF)
    return g


def uniform(shape, name):
    """fp32 uniform on [-1, 1), converted to bf16."""
    x = torch.rand(shape, generator=_generator(name), dtype=torch.float32) * 2.0 - 1.0
    return x.to(torch.bfloat16)


def normal(shape, std, name):
    """fp32 normal with the given standard deviation, converted to bf16."""
    x = torch.randn(shape, generator=_generator(name), dtype=torch.float32) * float(std)
    return x.to(torch.bfloat16)


def small_int(shape, lo, hi, name):
    """Integers in [lo, hi], exactly representable in bf16 (|v| <= 256)."""
    assert -256 <= lo <= hi <= 256
    x = torch.randint(lo, hi + 1, shape, generator=_generator(name), dtype=torch.int32)
    return x.to(torch.float32).to(torch.bfloat16)


def normal_f16(shape, std, name):
    """fp32 normal with the given standard deviation, converted to IEEE binary16 (torch.float16)."""
    x = torch.randn(shape, generator=_generator(name), dtype=torch.float32) * float(std)
    return x.to(torch.float16)


def small_int_f16(shape, lo, hi, name):
    """Integers in [lo, hi], exactly representable in binary16 (|v| <= 2048)."""
    assert -2048 <= lo <= hi <= 2048
    x = torch.randint(lo, hi + 1, shape, generator=_generator(name), dtype=torch.int32)
    return x.to(torch.float32).to(torch.float16)


def permutation(n, name):
    return torch.randperm(n, generator=_generator(name))


def choice_rows(M, count, name, edges=()):
    """Sorted sample of row indices: the given edge rows plus `count` random ones."""
    g = _generator(name)
    r = torch.randperm(M, generator=g)[: min(count, M)].tolist()
    s = sorted(set(int(e) for e in edges if 0 <= e < M) | set(r))
    return np.asarray(s, dtype=np.int64)


def bits(t):
    """uint16 numpy view of a CPU bfloat16 (or float16) tensor."""
    return t.view(torch.int16).numpy().view(np.uint16)


def from_bits(a):
    """CPU bfloat16 tensor sharing memory with a uint16 numpy array."""
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).view(torch.bfloat16)


# ---- the five configurations ------------------------------------------------

def config1(n=512):
    """Single GEMM C = A B, uniform[-1,1), no epilogue."""
    return {"A": uniform((n, n), "c1.A"), "B": uniform((n, n), "c1.B")}


def config2(n=8192):
    """Square GEMM, inputs ~ N(0,1), fused bias ~ N(0,1)."""
    return {"A": normal((n, n), 1.0, "c2.A"), "B": normal((n, n), 1.0, "c2.B"),
            "bias": normal((n,), 1.0, "c2.bias")}


def config2_f16(n=8192):
    """The square GEMM of config2 with every tensor in binary16 (the paper's own precision; same seeds'
    fp32 draws, rounded to fp16 instead of bf16)."""
    return {"A": normal_f16((n, n), 1.0, "c2.A"), "B": normal_f16((n, n), 1.0, "c2.B"),
            "bias": normal_f16((n,), 1.0, "c2.bias")}


def config3a(batch=128, n=512):
    """Batched GEMM, uniform[-1,1)."""
    return {"A": uniform((batch, n, n), "c3a.A"), "B": uniform((batch, n, n), "c3a.B")}


def config3b(m=256, n=256, k=131072):
    """Large-K GEMM, entries ~ N(0, variance 1/K)."""
    std = float(k) ** -0.5
    return {"A": normal((m, k), std, "c3b.A"), "B": normal((k, n), std, "c3b.B")}


def config4(tokens=8192, d=768, dff=3072):
    """GPT-small-shaped block GEMMs: weights and biases ~ N(0, std 0.02), activations ~ N(0,1)."""
    return {
        "X": normal((tokens, d), 1.0, "c4.X"),
        "Wqkv": normal((3 * d, d), 0.02, "c4.Wqkv"), "bqkv": normal((3 * d,), 0.02, "c4.bqkv"),
        "W1": normal((dff, d), 0.02, "c4.W1"), "b1": normal((dff,), 0.02, "c4.b1"),
        "W2": normal((d, dff), 0.02, "c4.W2"), "b2": normal((d,), 0.02, "c4.b2"),
        "R": normal((tokens, d), 1.0, "c4.R"),
    }


def config5(tokens=2048, d=4096, dff=14336, q_heads=32, kv_heads=8, head_dim=128):
    """Llama-3-8B-shaped block GEMMs: weights ~ N(0, std 0.02), no biases."""
    nqkv = (q_heads + 2 * kv_heads) * head_dim
    return {
        "X": normal((tokens, d), 1.0, "c5.X"),
        "Wqkv": normal((nqkv, d), 0.02, "c5.Wqkv"),
        "Wg": normal((dff, d), 0.02, "c5.Wg"), "Wu": normal((dff, d), 0.02, "c5.Wu"),
        "Wd": normal((d, dff), 0.02, "c5.Wd"),
        "R": normal((tokens, d), 1.0, "c5.R"),
    }


# ---- attention inputs of the two block configurations ---------------------------------------

def attention_qkv(batch, tokens, q_heads, kv_heads, head_dim, std, name):
    """A packed projection output [batch, tokens, (q_heads + 2 kv_heads) * head_dim]: per token the
    query heads, then the key heads, then the value heads.  Entries ~ N(0, std): a stand-in with
    the scale of X Wqkv^T for X ~ N(0,1) and weights ~ N(0, 0.02) (std = 0.02 sqrt(d_model))."""
    width = (q_heads + 2 * kv_heads) * head_dim
    return normal((batch, tokens, width), std, name)


def attention4(batch=8, tokens=1024):
    """GPT-small-shaped attention: 12 heads of 64 (d_model 768), batch x tokens = the 8192 tokens of
    configuration 4."""
    return {"qkv": attention_qkv(batch, tokens, 12, 12, 64, 0.02 * 768 ** 0.5, f"att4.qkv.{batch}.{tokens}"),
            "batch": batch, "tokens": tokens, "q_heads": 12, "kv_heads": 12, "head_dim": 64}


def attention5(batch=1, tokens=2048):
    """Llama-3-8B-shaped attention (Section 5.2.5): 32 query / 8 key-value heads of 128; batch 1 is
    configuration 5's 2048 tokens, batch 16 the block shape the paper measures."""
    return {"qkv": attention_qkv(batch, tokens, 32, 8, 128, 0.02 * 4096 ** 0.5, f"att5.qkv.{batch}.{tokens}"),
            "batch": batch, "tokens": tokens, "q_heads": 32, "kv_heads": 8, "head_dim": 128}


def split_qkv(w):
    """uint16 views (Q [B,T,Hq,D], K [B,T,Hkv,D], V [B,T,Hkv,D]) of a packed attention workload."""
    b = bits(w["qkv"])
    B, T, Hq, Hkv, D = w["batch"], w["tokens"], w["q_heads"], w["kv_heads"], w["head_dim"]
    q = b[:, :, : Hq * D].reshape(B, T, Hq, D)
    k = b[:, :, Hq * D: (Hq + Hkv) * D].reshape(B, T, Hkv, D)
    v = b[:, :, (Hq + Hkv) * D:].reshape(B, T, Hkv, D)
    return q, k, v


# ---- the paper's own problem shapes (Section 5.1 "Benchmark problems"), as a second workload -----
# Shapes only: the benchmark suite's files and the model's weights are not available and are not
# reconstructed; inputs are seeded draws as above, in bf16 (the paper runs them in tf32 / fp16).

def paper_square(n=4096):
    """Problem 1 of Section 5.1: C = A B, 4096 x 4096."""
    return {"A": normal((n, n), 1.0, f"p1.A.{n}"), "B": normal((n, n), 1.0, f"p1.B.{n}")}


def paper_batched(batch=128, m=512, k=1024, n=2048):
    """Problem 3: 128 x ([512, 1024] x [1024, 2048])."""
    return {"A": normal((batch, m, k), 1.0, "p3.A"), "B": normal((batch, k, n), 1.0, "p3.B")}


def paper_large_k(m=256, n=256, k=524288):
    """Problem 6: [256, 524288] x [524288, 256]; entries ~ N(0, variance 1/K) as in configuration 3b."""
    std = float(k) ** -0.5
    return {"A": normal((m, k), std, "p6.A"), "B": normal((k, n), std, "p6.B")}


def paper_block(kind):
    """Projection GEMMs of the two blocks at the token counts the paper measures: (128, 512, 768) and
    (16, 2048, 4096) with intermediate 14336.  Weights ~ N(0, 0.02), activations ~ N(0, 1)."""
    if kind == "gpt":
        t, d, dff, nqkv = 128 * 512, 768, 3072, 3 * 768
    else:
        t, d, dff, nqkv = 16 * 2048, 4096, 14336, 6144
    return {"tokens": t, "d": d, "dff": dff, "nqkv": nqkv,
            "X": normal((t, d), 1.0, f"pb.{kind}.X"), "Wqkv": normal((nqkv, d), 0.02, f"pb.{kind}.Wqkv"),
            "W1": normal((dff, d), 0.02, f"pb.{kind}.W1"), "Wu": normal((dff, d), 0.02, f"pb.{kind}.Wu") if kind != "gpt" else None,
            "W2": normal((d, dff), 0.02, f"pb.{kind}.W2"), "R": normal((t, d), 1.0, f"pb.{kind}.R"),
            "bqkv": normal((nqkv,), 0.02, f"pb.{kind}.bqkv"), "b1": normal((dff,), 0.02, f"pb.{kind}.b1"),
            "b2": normal((d,), 0.02, f"pb.{kind}.b2")}


# ---- whole blocks ---------------------------------------------------------------------------------

def block_weights(kind, batch, tokens):
    """Seeded weights and input of a whole block: "gpt" = GPT-small shape (d 768, 12 heads of 64, d_ff
    3072, LayerNorm, biases, GELU), "llama" = Llama-3-8B shape (d 4096, 32 query / 8 key-value heads of
    128, d_ff 14336, RMSNorm, rotary embedding, SwiGLU, no biases).  Projection weights ~ N(0, 0.02), norm
    gains ~ N(1, 0.1), biases ~ N(0, 0.02), input ~ N(0, 1).  Returns (description dict, tensors dict, X)."""
    if kind == "gpt":
        d, Hq, Hkv, D, dff = 768, 12, 12, 64, 3072
    else:
        d, Hq, Hkv, D, dff = 4096, 32, 8, 128, 14336
    n = (Hq + 2 * Hkv) * D
    tag = f"blk.{kind}"
    gain = lambda name: (normal((d,), 0.1, f"{tag}.{name}").float() + 1.0).to(torch.bfloat16)
    t = {"norm1_g": gain("n1g"), "norm2_g": gain("n2g"),
         "Wqkv": normal((n, d), 0.02, f"{tag}.Wqkv"), "Wo": normal((d, Hq * D), 0.02, f"{tag}.Wo"),
         "W1": normal((dff, d), 0.02, f"{tag}.W1"), "W2": normal((d, dff), 0.02, f"{tag}.W2")}
    if kind == "gpt":
        t.update({"norm1_b": normal((d,), 0.02, f"{tag}.n1b"), "norm2_b": normal((d,), 0.02, f"{tag}.n2b"),
                  "bqkv": normal((n,), 0.02, f"{tag}.bqkv"), "bo": normal((d,), 0.02, f"{tag}.bo"),
                  "b1": normal((dff,), 0.02, f"{tag}.b1"), "b2": normal((d,), 0.02, f"{tag}.b2")})
    else:
        t["W1u"] = normal((dff, d), 0.02, f"{tag}.W1u")
    desc = {"batch": batch, "tokens": tokens, "d_model": d, "q_heads": Hq, "kv_heads": Hkv, "head_dim": D, "d_ff": dff,
            "rms": kind != "gpt", "rope": kind != "gpt", "rope_base": 500000.0, "eps": 1e-5, "act_gated": kind != "gpt"}
    X = normal((batch * tokens, d), 1.0, f"{tag}.X.{batch}.{tokens}")
    return desc, t, X
