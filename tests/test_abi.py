"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol, and its
host logic (validation, shape -> configuration lookup) behaves.  No kernel is launched."""
import ctypes
import os
import re

import pytest

import paper_2604_26666_amd as fact

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module", autouse=True)
def _built():
    if not os.path.exists(fact.lib_path()):
        from paper_2604_26666_amd import build
        build.build()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "fact.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fact_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    syms = declared_symbols()
    assert {"fact_gemm", "fact_gemm_batched", "fact_gemm_splitk", "fact_block_mlp"} <= set(syms)
    L = ctypes.CDLL(fact.lib_path())
    for s in syms:
        assert hasattr(L, s), f"{s} is declared in fact.h but not exported"


def test_version_and_status_strings():
    assert fact.fact_version() >= 100
    assert fact.fact_status_string(0) == "ok"
    for rc in range(-8, 0):
        assert fact.fact_status_string(rc) not in ("ok", "unknown status")
    assert fact.fact_status_string(-99) == "unknown status"


def test_config_descriptions():
    n = fact.fact_num_configs()
    assert n >= 4
    for i in range(n):
        bm, bn, wm, wn, lds = fact.fact_config_info(i)
        assert bm % (32 * wm) == 0 and bn % (32 * wn) == 0
        assert 0 < lds <= 160 * 1024
    with pytest.raises(fact.FactError):
        fact.fact_config_info(n)


def test_validation_rejects_before_any_launch():
    p = 0x1000  # never dereferenced: validation fails first
    ok_args = dict(M=64, N=64, K=64, lda=64, ldb=64, ldc=64)
    g = lambda **kw: fact.fact_gemm(kw.get("M", 64), kw.get("N", 64), kw.get("K", 64), kw.get("A", p), kw.get("lda", 64),
                                    kw.get("B", p), kw.get("ldb", 64), kw.get("trans_b", 0), kw.get("C", p),
                                    kw.get("ldc", 64), kw.get("ep"), 0)
    assert g(A=None) == -1 and g(B=None) == -1 and g(C=None) == -1
    assert g(M=0) == -2 and g(N=-1) == -2 and g(K=0) == -2
    assert g(lda=63) == -2 and g(ldb=63) == -2 and g(ldc=63) == -2
    assert g(trans_b=2) == -4
    assert g(A=p + 1) == -3
    E = fact.Epilogue
    assert g(ep=E(act=7)) == -5
    assert g(ep=E(act=fact.ACT_SILU_GATE)) == -4                      # gated needs trans_b = 1
    assert g(ep=E(act=fact.ACT_SILU_GATE, bias=p), trans_b=1) == -5   # no bias with the gate
    assert g(ep=E(act=fact.ACT_SILU_GATE), trans_b=1, N=63, ldb=64) == -5
    assert g(ep=E(residual=p, ldr=63)) == -2
    # batched: C stride must hold a whole matrix
    assert fact.fact_gemm_batched(2, 64, 64, 64, p, 64, 0, p, 64, 0, 0, p, 64, 100, None, 0) == -2
    # split-K: workspace required and large enough
    assert fact.fact_gemm_splitk(256, 256, 4096, p, 4096, p, 256, 0, p, 256, None, 4, None, 0, 0) == -6
    need = fact.fact_gemm_splitk_workspace_bytes(256, 256, 4096, 4)
    assert need == 4 * 256 * 256 * 4
    assert fact.fact_gemm_splitk(256, 256, 4096, p, 4096, p, 256, 0, p, 256, None, 4, 0x2000, need - 1, 0) == -6
    assert fact.fact_gemm_splitk(256, 256, 4096, p, 4096, p, 256, 0, p, 256, None, -1, None, 0, 0) == -7
    # block: pointer and epilogue rules
    assert fact.fact_block_mlp(64, 64, 128, None, p, None, None, 0, p, None, None, p, p, None, 0, 0) == -1
    assert fact.fact_block_mlp(64, 64, 128, p, p, None, None, fact.ACT_SILU_GATE, p, None, None, p, p, None, 0, 0) == -1
    assert fact.fact_block_mlp(64, 64, 128, p, p, p, p, fact.ACT_SILU_GATE, p, None, None, p, p, None, 0, 0) == -5
    assert fact.fact_block_mlp(64, 64, 128, p, p, p, None, fact.ACT_GELU_TANH, p, None, None, p, p, None, 0, 0) == -5
    # forced configuration that does not exist / cannot take the shape
    n = fact.fact_num_configs()
    ex = lambda cfg, N=64, tb=0: fact.fact_gemm_ex(1, 64, N, 64, p, 64, 0, p, 64, 0, tb, p, 64, 0, None, cfg, 0, 0, None, 0, 0)
    assert ex(n) == -7
    assert ex(0, N=60) == -7          # N % 8 != 0 with trans_b = 0 cannot use the MFMA kernel
    wide192 = [c for c in range(n) if fact.fact_config_info(c)[1] == 192]
    assert wide192 and all(ex(c, tb=0) == -7 for c in wide192)       # 192-wide tiles stage B as [N][K] only


def test_select_config_host_logic():
    n = fact.fact_num_configs()
    shapes = [(1, 8192, 8192, 8192, 0, 0), (128, 512, 512, 512, 0, 0), (1, 256, 256, 131072, 0, 0),
              (1, 8192, 2304, 768, 1, 0), (1, 8192, 3072, 768, 1, 1), (1, 2048, 28672, 4096, 1, 2),
              (1, 2048, 4096, 14336, 1, 0), (1, 512, 512, 512, 0, 0)]
    for s in shapes:
        rc, cfg, split = fact.fact_select_config(*s)
        assert rc == 0 and 0 <= cfg < n and (split >= 1 or split <= -2), s      # -g: tail split of g K ranges
        if s[5] == fact.ACT_SILU_GATE:
            bm, bn, wm, wn, _ = fact.fact_config_info(cfg)
            assert (bn // wn // 16) % 2 == 0       # gate and up tiles pair up inside a wave
    # large K with few output tiles is split; a big square problem is not
    assert fact.fact_select_config(1, 256, 256, 131072, 0, 0)[2] > 1
    assert fact.fact_select_config(1, 8192, 8192, 8192, 0, 0)[2] == 1
    # unaligned dimensions go to the guarded kernel
    assert fact.fact_select_config(1, 5, 7, 3, 0, 0)[1] == -1
    assert fact.fact_select_config(1, 64, 60, 64, 0, 0)[1] == -1
    assert fact.fact_select_config(1, 64, 60, 64, 1, 0)[1] >= 0
    assert fact.fact_select_config(0, 1, 1, 1, 0, 0)[0] == -2
    assert fact.fact_select_config(1, 8, 9, 8, 1, 2)[0] == -5


def test_new_entry_points_validate_on_the_host_before_any_gpu_call():
    """Argument validation comes before anything touches the GPU, so it can be exercised here."""
    st = (64 * 192, 192, 64)
    p = 4096                                   # a non-NULL, 16-byte aligned number; never dereferenced
    att = lambda **k: fact.fact_attention(k.get("B", 1), k.get("T", 64), k.get("hq", 2), k.get("hkv", 1), k.get("D", 64),
                                          k.get("Q", p), k.get("qs", st), p, st, p, st, p, (64 * 128, 128, 64), k.get("causal", 1), 0.0, 0)
    assert att(D=96) == -7 and att(hq=3, hkv=2) == -2 and att(Q=None) == -1 and att(Q=p + 2) == -3
    assert att(qs=(64 * 192, 32, 64)) == -2 and att(causal=3) == -4 and att(T=0) == -2
    assert fact.fact_norm(16, 60, p, 64, p, None, 1e-5, 1, p, 64, 0) == -7
    assert fact.fact_norm(16, 64, p, 32, p, None, 1e-5, 1, p, 64, 0) == -2
    assert fact.fact_norm(16, 64, p, 64, p, p, 1e-5, 1, p, 64, 0) == -5
    assert fact.fact_norm(16, 16384, p, 16384, p, None, 1e-5, 0, p, 16384, 0) == -7
    assert fact.fact_rope(1, 64, 3, 24, p, st, 10000.0, 0) == -7
    assert fact.fact_rope(1, 64, 3, 64, p, st, 0.5, 0) == -2
    assert fact.fact_rope(1, 64, 3, 64, None, st, 10000.0, 0) == -1
    w = dict(norm1_g=p, norm2_g=p, Wqkv=p, Wo=p, W1=p, W2=p)
    ok = fact.Block(2, 128, 256, 4, 2, 64, 512, 1, fact.ACT_NONE, **w)
    n = fact.fact_block_scratch_bytes(ok)
    T, nqkv = 256, (4 + 2 * 2) * 64
    assert n >= 2 * (3 * T * 256 + T * nqkv + T * 256 + T * 512) and n % 256 == 0
    offs = fact.fact_block_scratch_offsets(ok)
    assert offs == sorted(offs) and all(o % 256 == 0 for o in offs) and offs[0] == 0
    assert fact.fact_block_scratch_bytes(fact.Block(2, 128, 256, 4, 3, 64, 512, 1, fact.ACT_NONE, **w)) == 0
    assert fact.fact_block_forward(ok, p, p, p, n - 1, 0) == -6
    assert fact.fact_block_forward(fact.Block(2, 128, 256, 4, 2, 64, 512, 1, fact.ACT_SILU_GATE, **w), p, p, p, n, 0) == -5
    assert fact.fact_gemm_f32out_workspace_bytes(256, 256, 4096, 1) == 0          # K whole: the main kernel writes fp32 itself
    assert fact.fact_gemm_f32out_workspace_bytes(256, 256, 4096, 4) == 4 * 256 * 256 * 4


def test_two_per_compute_unit_configuration_and_fp16_field_host_logic():
    """Configuration 15 (128 x 192, 2 stages) takes exactly half a compute unit's LDS, so two of its
    work-groups share one; it has no prefetch sink, hence no tail split.  The f16 field is validated
    before anything touches the GPU."""
    n = fact.fact_num_configs()
    assert n >= 16
    bm, bn, wm, wn, lds = fact.fact_config_info(15)
    assert (bm, bn, wm, wn) == (128, 192, 2, 2) and lds == 80 * 1024 and 2 * lds <= 160 * 1024
    bm14, bn14, _, _, lds14 = fact.fact_config_info(14)                 # the same tile on 3 stages, with the sink
    assert (bm14, bn14) == (128, 192) and lds14 == 3 * (128 + 192) * 128 + 4 * 256
    # every other configuration either fits twice with its sink or does not fit twice at all
    for c in range(n):
        l = fact.fact_config_info(c)[4]
        assert l <= 160 * 1024 and (l <= 80 * 1024 or l > 80 * 1024 + 2048 or c == 15), (c, l)
    p = 4096                                   # a non-NULL, 16-byte aligned number; never dereferenced
    # (832 tiles: a partly filled last round on 256 or 512 slots)  a tail split cannot use configuration 15;
    # the same request on configuration 14 only lacks a workspace
    ep = fact.Epilogue()
    assert fact.fact_gemm_ex(1, 8192, 2496, 4096, p, 4096, 0, p, 4096, 0, 1, p, 2496, 0, ep, 15, -2, 4, None, 0, 0) == -7
    assert fact.fact_gemm_ex(1, 8192, 2496, 4096, p, 4096, 0, p, 4096, 0, 1, p, 2496, 0, ep, 14, -2, 4, None, 0, 0) == -6
    assert fact.fact_gemm(64, 64, 64, p, 64, p, 64, 0, p, 64, fact.Epilogue(f16=2), 0) == -5
    assert fact.fact_gemm(64, 64, 64, p, 64, p, 64, 0, p, 64, fact.Epilogue(f16=-1), 0) == -5
