"""ctypes binding of include/fact.h.  Argument marshalling only.

Functions carry the C names and take the C arguments in the C order.  A pointer argument
may be an int (device address), None (NULL) or a torch tensor (its data_ptr() is passed);
`stream` may be None (torch's current stream), an int, or a torch.cuda.Stream.
Return codes are returned unchanged by the fact_* functions; `check()` raises on error.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
# FACT_GEMM_LIB selects another build of the same library (used to compare variants)
_LIB_PATH = os.environ.get("FACT_GEMM_LIB") or os.path.join(_HERE, "libfact_gemm.so")

ACT_NONE = 0
ACT_GELU_TANH = 1
ACT_SILU_GATE = 2
CONFIG_TABLE = -1        # config_id of fact_gemm_ex: the table's choice
CONFIG_GUARDED = -2      # config_id of fact_gemm_ex: the guarded one-thread-per-element kernel

_i64 = ctypes.c_int64
_int = ctypes.c_int
_ptr = ctypes.c_void_p
_size = ctypes.c_size_t


class FactError(RuntimeError):
    pass


class _CEpilogue(ctypes.Structure):
    _fields_ = [("bias", _ptr), ("residual", _ptr), ("ldr", _i64), ("stride_r", _i64), ("act", ctypes.c_int32),
                ("out_f32", ctypes.c_int32), ("f16", ctypes.c_int32)]


class _CBlock(ctypes.Structure):
    _fields_ = ([(n, _i64) for n in ("batch", "tokens", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ff")] +
                [("norm_rms", ctypes.c_int32), ("act", ctypes.c_int32), ("rope", ctypes.c_int32),
                 ("eps", ctypes.c_float), ("rope_base", ctypes.c_float)] +
                [(n, _ptr) for n in ("norm1_g", "norm1_b", "Wqkv", "bqkv", "Wo", "bo", "norm2_g", "norm2_b", "W1", "W1u", "b1", "W2", "b2")])


class Block:
    """Mirror of the C struct fact_block; pointer fields take tensors, ints or None."""
    _PTRS = ("norm1_g", "norm1_b", "Wqkv", "bqkv", "Wo", "bo", "norm2_g", "norm2_b", "W1", "W1u", "b1", "W2", "b2")

    def __init__(self, batch, tokens, d_model, n_q_heads, n_kv_heads, head_dim, d_ff, norm_rms, act, rope=0, eps=0.0,
                 rope_base=0.0, **weights):
        self.dims = (batch, tokens, d_model, n_q_heads, n_kv_heads, head_dim, d_ff)
        self.norm_rms, self.act, self.rope, self.eps, self.rope_base = norm_rms, act, rope, eps, rope_base
        unknown = set(weights) - set(self._PTRS)
        if unknown:
            raise TypeError(f"unknown block fields {sorted(unknown)}")
        self.weights = weights                      # keeps the tensors alive

    def _c(self):
        c = _CBlock(*[int(v) for v in self.dims], int(self.norm_rms), int(self.act), int(self.rope), float(self.eps),
                    float(self.rope_base))
        for n in self._PTRS:
            setattr(c, n, _addr(self.weights.get(n)))
        return c


class Epilogue:
    """Mirror of the C struct fact_epilogue."""

    def __init__(self, bias=None, residual=None, ldr=0, stride_r=0, act=ACT_NONE, out_f32=0, f16=0):
        self.bias, self.residual, self.ldr, self.stride_r, self.act, self.out_f32 = bias, residual, ldr, stride_r, act, out_f32
        self.f16 = f16

    def _c(self):
        return _CEpilogue(_addr(self.bias), _addr(self.residual), int(self.ldr), int(self.stride_r), int(self.act), int(self.out_f32), int(self.f16))


_lib = None


def lib_path():
    return _LIB_PATH


def lib():
    """The loaded shared library.  Raises if it has not been built: there is no fallback."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FactError(f"{_LIB_PATH} is missing: build it with `python -m paper_2604_26666_amd.build` "
                            "(or __graft_entry__.build()); there is no fallback path")
        L = ctypes.CDLL(_LIB_PATH)
        ep = ctypes.POINTER(_CEpilogue)
        L.fact_gemm.argtypes = [_i64, _i64, _i64, _ptr, _i64, _ptr, _i64, _int, _ptr, _i64, ep, _ptr]
        L.fact_gemm_batched.argtypes = [_i64, _i64, _i64, _i64, _ptr, _i64, _i64, _ptr, _i64, _i64, _int,
                                        _ptr, _i64, _i64, ep, _ptr]
        L.fact_gemm_splitk.argtypes = [_i64, _i64, _i64, _ptr, _i64, _ptr, _i64, _int, _ptr, _i64, ep,
                                       _int, _ptr, _size, _ptr]
        L.fact_gemm_splitk_workspace_bytes.argtypes = [_i64, _i64, _i64, _int]
        L.fact_gemm_splitk_workspace_bytes.restype = _size
        L.fact_gemm_f32out_workspace_bytes.argtypes = [_i64, _i64, _i64, _int]
        L.fact_gemm_f32out_workspace_bytes.restype = _size
        L.fact_block_mlp.argtypes = [_i64, _i64, _i64, _ptr, _ptr, _ptr, _ptr, _int, _ptr, _ptr, _ptr,
                                     _ptr, _ptr, _ptr, _size, _ptr]
        L.fact_block_mlp_f16.argtypes = L.fact_block_mlp.argtypes
        L.fact_block_mlp_workspace_bytes.argtypes = [_i64, _i64, _i64, _int]
        L.fact_block_mlp_workspace_bytes.restype = _size
        L.fact_gemm_ex.argtypes = [_i64, _i64, _i64, _i64, _ptr, _i64, _i64, _ptr, _i64, _i64, _int,
                                   _ptr, _i64, _i64, ep, _int, _int, _int, _ptr, _size, _ptr]
        i64p = ctypes.POINTER(_i64)
        L.fact_attention.argtypes = [_i64, _i64, _i64, _i64, _i64, _ptr, i64p, _ptr, i64p, _ptr, i64p, _ptr, i64p,
                                     _int, ctypes.c_float, _ptr]
        L.fact_attention.restype = _int
        L.fact_norm.argtypes = [_i64, _i64, _ptr, _i64, _ptr, _ptr, ctypes.c_float, _int, _ptr, _i64, _ptr]
        L.fact_norm.restype = _int
        L.fact_rope.argtypes = [_i64, _i64, _i64, _i64, _ptr, i64p, ctypes.c_float, _ptr]
        L.fact_rope.restype = _int
        bp = ctypes.POINTER(_CBlock)
        L.fact_block_scratch_bytes.argtypes = [bp]
        L.fact_block_scratch_bytes.restype = _size
        L.fact_block_scratch_offsets.argtypes = [bp, ctypes.POINTER(_size)]
        L.fact_block_scratch_offsets.restype = _int
        L.fact_block_forward.argtypes = [bp, _ptr, _ptr, _ptr, _size, _ptr]
        L.fact_block_forward.restype = _int
        L.fact_num_configs.argtypes = []
        ip = ctypes.POINTER(_int)
        L.fact_config_info.argtypes = [_int, ip, ip, ip, ip, ip]
        L.fact_select_config.argtypes = [_i64, _i64, _i64, _i64, _int, _int, ip, ip]
        L.fact_status_string.argtypes = [_int]
        L.fact_status_string.restype = ctypes.c_char_p
        L.fact_last_error.argtypes = []
        L.fact_last_error.restype = ctypes.c_char_p
        L.fact_version.argtypes = []
        L.fact_gemm_splitk_static.argtypes = [_i64, _i64, _i64, _ptr, _i64, _ptr, _i64, _int, _ptr, _i64, ep, _int, _ptr]
        L.fact_gemm_splitk_static.restype = _int
        L.fact_gemm_splitk_static_init.argtypes = []
        L.fact_gemm_splitk_static_init.restype = _int
        L.fact_gemm_splitk_static_capacity.argtypes = []
        L.fact_gemm_splitk_static_capacity.restype = _size
        L.fact_tail_timeouts.argtypes = [_ptr, _ptr, ctypes.POINTER(_int)]
        L.fact_tail_timeouts.restype = _int
        L.fact_test_tail_poll_budget.argtypes = [_int]
        L.fact_test_tail_poll_budget.restype = None
        L.fact_tune_persistent.argtypes = [_int]
        L.fact_tune_persistent.restype = _int
        L.fact_persistent_grid.argtypes = [_i64, _i64, _i64, _i64, _int, _int, _int]
        L.fact_persistent_grid.restype = _int
        L.fact_registry_load.argtypes = [ctypes.c_char_p]
        L.fact_registry_load.restype = _int
        L.fact_registry_clear.argtypes = []
        L.fact_registry_clear.restype = None
        L.fact_registry_size.argtypes = []
        L.fact_registry_size.restype = _int
        for name in ("fact_gemm", "fact_gemm_batched", "fact_gemm_splitk", "fact_block_mlp", "fact_block_mlp_f16", "fact_gemm_ex",
                     "fact_num_configs", "fact_config_info", "fact_select_config", "fact_version"):
            getattr(L, name).restype = _int
        _lib = L
    return _lib


def _addr(x):
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return int(x.data_ptr())       # torch tensor


def _stream(s):
    if s is None:
        import torch
        return int(torch.cuda.current_stream().cuda_stream)
    if isinstance(s, int):
        return s
    return int(s.cuda_stream)


def _ep(ep):
    return None if ep is None else ctypes.byref(ep._c())


def check(rc, what="fact call"):
    if rc != 0:
        raise FactError(f"{what} failed: {rc} ({fact_status_string(rc)}) {fact_last_error()}")
    return rc


def fact_gemm(M, N, K, A, lda, B, ldb, trans_b, C, ldc, ep=None, stream=None):
    return lib().fact_gemm(M, N, K, _addr(A), lda, _addr(B), ldb, int(trans_b), _addr(C), ldc, _ep(ep), _stream(stream))


def fact_gemm_batched(batch, M, N, K, A, lda, stride_a, B, ldb, stride_b, trans_b, C, ldc, stride_c,
                      ep=None, stream=None):
    return lib().fact_gemm_batched(batch, M, N, K, _addr(A), lda, stride_a, _addr(B), ldb, stride_b, int(trans_b),
                                   _addr(C), ldc, stride_c, _ep(ep), _stream(stream))


def fact_gemm_splitk(M, N, K, A, lda, B, ldb, trans_b, C, ldc, ep, split_k, ws, ws_bytes, stream=None):
    return lib().fact_gemm_splitk(M, N, K, _addr(A), lda, _addr(B), ldb, int(trans_b), _addr(C), ldc, _ep(ep),
                                  int(split_k), _addr(ws), int(ws_bytes), _stream(stream))


def fact_gemm_splitk_static(M, N, K, A, lda, B, ldb, trans_b, C, ldc, ep, split_k, stream=None):
    return lib().fact_gemm_splitk_static(M, N, K, _addr(A), lda, _addr(B), ldb, int(trans_b), _addr(C), ldc, _ep(ep),
                                         int(split_k), _stream(stream))


def fact_gemm_splitk_static_init():
    return int(lib().fact_gemm_splitk_static_init())


def fact_gemm_splitk_static_capacity():
    return int(lib().fact_gemm_splitk_static_capacity())


def fact_gemm_splitk_workspace_bytes(M, N, K, split_k):
    return int(lib().fact_gemm_splitk_workspace_bytes(M, N, K, int(split_k)))


def fact_gemm_f32out_workspace_bytes(M, N, K, split_k):
    return int(lib().fact_gemm_f32out_workspace_bytes(M, N, K, split_k))


def fact_block_mlp(T, d_model, d_ff, X, W1, W1u, b1, act, W2, b2, R, H, Y, ws, ws_bytes, stream=None):
    return lib().fact_block_mlp(T, d_model, d_ff, _addr(X), _addr(W1), _addr(W1u), _addr(b1), int(act),
                                _addr(W2), _addr(b2), _addr(R), _addr(H), _addr(Y), _addr(ws), int(ws_bytes),
                                _stream(stream))


def fact_block_mlp_f16(T, d_model, d_ff, X, W1, W1u, b1, act, W2, b2, R, H, Y, ws, ws_bytes, stream=None):
    return lib().fact_block_mlp_f16(T, d_model, d_ff, _addr(X), _addr(W1), _addr(W1u), _addr(b1), int(act),
                                    _addr(W2), _addr(b2), _addr(R), _addr(H), _addr(Y), _addr(ws), int(ws_bytes),
                                    _stream(stream))


def fact_block_mlp_workspace_bytes(T, d_model, d_ff, act):
    return int(lib().fact_block_mlp_workspace_bytes(T, d_model, d_ff, int(act)))


def fact_gemm_ex(batch, M, N, K, A, lda, stride_a, B, ldb, stride_b, trans_b, C, ldc, stride_c, ep,
                 config_id, split_k, group_m, ws, ws_bytes, stream=None):
    return lib().fact_gemm_ex(batch, M, N, K, _addr(A), lda, stride_a, _addr(B), ldb, stride_b, int(trans_b),
                              _addr(C), ldc, stride_c, _ep(ep), int(config_id), int(split_k), int(group_m),
                              _addr(ws), int(ws_bytes), _stream(stream))


def fact_attention(batch, T, n_q_heads, n_kv_heads, head_dim, Q, q_strides, K, k_strides, V, v_strides,
                   O, o_strides, causal=1, scale=0.0, stream=None):
    """Strides are sequences of three element strides (batch entry, token, head)."""
    arr = lambda s: (_i64 * 3)(*[int(x) for x in s])
    return lib().fact_attention(batch, T, n_q_heads, n_kv_heads, head_dim, _addr(Q), arr(q_strides), _addr(K), arr(k_strides),
                                _addr(V), arr(v_strides), _addr(O), arr(o_strides), int(causal), float(scale), _stream(stream))


def fact_norm(T, d, X, ldx, gamma, beta, eps, rms, Y, ldy, stream=None):
    return lib().fact_norm(T, d, _addr(X), ldx, _addr(gamma), _addr(beta), float(eps), int(rms), _addr(Y), ldy, _stream(stream))


def fact_rope(batch, T, n_heads, head_dim, X, strides, base, stream=None):
    return lib().fact_rope(batch, T, n_heads, head_dim, _addr(X), (_i64 * 3)(*[int(x) for x in strides]), float(base), _stream(stream))


def fact_block_scratch_bytes(blk):
    return int(lib().fact_block_scratch_bytes(ctypes.byref(blk._c())))


def fact_block_scratch_offsets(blk):
    """Byte offsets of (N1, QKV, A, X1, N2, H, workspace) inside the scratch buffer."""
    offs = (_size * 7)()
    rc = lib().fact_block_scratch_offsets(ctypes.byref(blk._c()), offs)
    check(rc, "fact_block_scratch_offsets")
    return [int(v) for v in offs]


def fact_block_forward(blk, X, Y, scratch, scratch_bytes, stream=None):
    return lib().fact_block_forward(ctypes.byref(blk._c()), _addr(X), _addr(Y), _addr(scratch), int(scratch_bytes), _stream(stream))


def fact_num_configs():
    return int(lib().fact_num_configs())


def fact_config_info(cfg_id):
    """Returns (tile_m, tile_n, waves_m, waves_n, lds_bytes) or raises for a bad id."""
    v = [_int() for _ in range(5)]
    check(lib().fact_config_info(int(cfg_id), *[ctypes.byref(x) for x in v]), "fact_config_info")
    return tuple(x.value for x in v)


def fact_select_config(batch, M, N, K, trans_b, act):
    """Returns (status, config_id, split_k)."""
    c, s = _int(-2), _int(0)
    rc = lib().fact_select_config(batch, M, N, K, int(trans_b), int(act), ctypes.byref(c), ctypes.byref(s))
    return rc, c.value, s.value


def fact_tail_timeouts(ws, stream=None):
    """(status, gave_up) for a tail-split workspace; synchronizes the stream."""
    g = _int(-1)
    rc = lib().fact_tail_timeouts(_addr(ws), _stream(stream), ctypes.byref(g))
    return rc, g.value


def fact_test_tail_poll_budget(polls):
    lib().fact_test_tail_poll_budget(int(polls))


def fact_tune_persistent(mode):
    return lib().fact_tune_persistent(int(mode))


def fact_persistent_grid(batch, M, N, K, trans_b, act=ACT_NONE, cfg=-1):
    return lib().fact_persistent_grid(batch, M, N, K, int(trans_b), int(act), int(cfg))


def fact_registry_load(path):
    """Entries taken from the registry file (>= 0) or a negative status."""
    return int(lib().fact_registry_load(None if path is None else os.fsencode(path)))


def fact_registry_clear():
    lib().fact_registry_clear()


def fact_registry_size():
    return int(lib().fact_registry_size())


def fact_status_string(rc):
    return lib().fact_status_string(int(rc)).decode()


def fact_last_error():
    return lib().fact_last_error().decode()


def fact_version():
    return int(lib().fact_version())
