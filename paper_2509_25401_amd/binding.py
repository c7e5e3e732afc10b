"""ctypes binding of the C-ABI in include/sparse_attn.h -- argument marshalling only.

Every step of the attention path runs inside the HIP library; PyTorch is used for device
memory and the current stream.  There is no fallback: if the library has not been built the
calls raise.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libsparse_attn_hip.so")
_lib = None


class SparseAttnError(RuntimeError):
    def __init__(self, code, message):
        super().__init__(f"sparse_attn error {code}: {message}")
        self.code = code


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libsparse_attn_hip.so (built by paper_2509_25401_amd/build.py); raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2509_25401_amd.build` "
            "(there is no fallback path)")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32 = ctypes.c_void_p, ctypes.c_int
    fwd_args = [vp] * 7 + [i32] * 6
    lib.sparse_attn_fwd.argtypes = fwd_args
    lib.sparse_attn_fwd.restype = i32
    lib.sparse_attn_fwd_stream.argtypes = fwd_args + [vp]
    lib.sparse_attn_fwd_stream.restype = i32
    lib.sparse_attn_fwd_noalloc.argtypes = fwd_args + [vp]
    lib.sparse_attn_fwd_noalloc.restype = i32
    lib.sparse_attn_fwd_timed.argtypes = fwd_args + [vp, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_float)]
    lib.sparse_attn_fwd_timed.restype = i32
    lib.sparse_attn_fwd_workspace.argtypes = fwd_args + [vp, ctypes.c_size_t, vp]
    lib.sparse_attn_fwd_workspace.restype = i32
    lib.sparse_attn_release_scratch.argtypes = [vp]
    lib.sparse_attn_release_scratch.restype = i32
    lib.sparse_attn_workspace_bytes.argtypes = [i32] * 5
    lib.sparse_attn_workspace_bytes.restype = ctypes.c_size_t
    lib.sparse_attn_count_kept.argtypes = [vp, vp] + [i32] * 5 + [ctypes.POINTER(ctypes.c_ulonglong)] * 2
    lib.sparse_attn_count_kept.restype = i32
    lib.sparse_attn_pack_mask.argtypes = [vp, ctypes.c_longlong, i32, vp]
    lib.sparse_attn_pack_mask.restype = i32
    lib.sparse_gemm_q.argtypes = [vp] * 5 + [i32] * 6
    lib.sparse_gemm_q.restype = i32
    lib.sparse_gemm_q_stream.argtypes = [vp] * 5 + [i32] * 6 + [vp]
    lib.sparse_gemm_q_stream.restype = i32
    lib.sparse_attn_plan_create.argtypes = [vp, vp] + [i32] * 6 + [vp, ctypes.POINTER(vp)]
    lib.sparse_attn_plan_create.restype = i32
    lib.sparse_attn_plan_run.argtypes = [vp] * 6 + [i32, vp]
    lib.sparse_attn_plan_run.restype = i32
    lib.sparse_attn_plan_run_forecast.argtypes = [vp] * 6 + [i32, vp, i32, vp]
    lib.sparse_attn_plan_run_forecast.restype = i32
    lib.sparse_attn_plan_destroy.argtypes = [vp]
    lib.sparse_attn_plan_destroy.restype = i32
    lib.sparse_gemm_q_norm_rope.argtypes = [vp] * 4 + [ctypes.c_float] + [vp] * 4 + [i32] * 6 + [vp]
    lib.sparse_gemm_q_norm_rope.restype = i32
    lib.sparse_gemm_o.argtypes = [vp] * 4 + [i32, vp, vp] + [i32] * 6
    lib.sparse_gemm_o.restype = i32
    lib.sparse_gemm_o_stream.argtypes = [vp] * 4 + [i32, vp, vp] + [i32] * 6 + [vp]
    lib.sparse_gemm_o_stream.restype = i32
    lib.sparse_gemm_o_reuse.argtypes = [vp] * 4 + [vp, vp, i32, vp] + [i32] * 6 + [vp]
    lib.sparse_gemm_o_reuse.restype = i32
    f32 = ctypes.c_float
    lib.sparse_attn_fwd_forecast.argtypes = [vp] * 7 + [i32, vp] + [i32] * 6 + [vp]
    lib.sparse_attn_fwd_forecast.restype = i32
    lib.sparse_op_reuse.argtypes = [vp, vp, i32, vp, ctypes.c_ulonglong, vp]
    lib.sparse_op_reuse.restype = i32
    lib.sparse_taylor_update.argtypes = [vp, vp, i32, i32, f32, ctypes.c_ulonglong, vp]
    lib.sparse_taylor_update.restype = i32
    lib.sparse_taylor_coefficients.argtypes = [i32, f32, vp]
    lib.sparse_taylor_coefficients.restype = None
    lib.sparse_symbols_update.argtypes = [vp] * 4 + [i32] * 6 + [f32] * 3
    lib.sparse_symbols_update.restype = i32
    lib.sparse_symbols_update_stream.argtypes = [vp] * 4 + [i32] * 6 + [f32] * 3 + [vp]
    lib.sparse_symbols_update_stream.restype = i32
    lib.sparse_symbols_update_granular.argtypes = [vp] * 4 + [i32] * 8 + [f32] * 3 + [vp]
    lib.sparse_symbols_update_granular.restype = i32
    lib.sparse_attn_profile_begin.argtypes = [i32]
    lib.sparse_attn_profile_begin.restype = i32
    lib.sparse_attn_profile_end.argtypes = [ctypes.POINTER(i32), ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
    lib.sparse_attn_profile_end.restype = i32
    lib.sparse_attn_last_error.argtypes = []
    lib.sparse_attn_last_error.restype = ctypes.c_char_p
    lib.sparse_attn_version.argtypes = []
    lib.sparse_attn_version.restype = i32
    _lib = lib
    return lib


def sparse_attn_last_error() -> str:
    return load_library().sparse_attn_last_error().decode()


def sparse_attn_version() -> int:
    return int(load_library().sparse_attn_version())


def _raise(code):
    raise SparseAttnError(code, sparse_attn_last_error())


def _dev_ptr(t, name, allow_none=False):
    if t is None:
        if allow_none:
            return None
        raise ValueError(f"{name} must not be None")
    if not t.is_cuda:
        raise ValueError(f"{name} must live in device memory")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return ctypes.c_void_p(t.data_ptr())


def _stream_ptr(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _check(t, name, dtype, shape, allow_none=False):
    """Raises ValueError unless tensor `t` has exactly this dtype and shape (the kernels index by them: a mask packed
    for another block size, or an int32 flag tensor, would make them read past the allocation)."""
    if t is None:
        if allow_none:
            return
        raise ValueError(f"{name} must not be None")
    if t.dtype != dtype:
        raise ValueError(f"{name} must have dtype {dtype}, got {t.dtype}")
    if tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} must have shape {tuple(shape)}, got {tuple(t.shape)}")


def _same_device(tensors):
    devs = {str(t.device) for t in tensors if t is not None}
    if len(devs) > 1:
        raise ValueError(f"all tensors must live on one device, got {sorted(devs)}")


def _ceil_div(a, b):
    return -(-int(a) // int(b))


def _check_attn_tensors(Q, K, V, cache_flags, kv_mask, O_cache, O, block_q, block_k, granularity=1):
    """Shapes and dtypes of the attention call as include/sparse_attn.h documents them."""
    import torch
    if Q.dim() != 4:
        raise ValueError("Q must be [B, H, L, D]")
    B, H, L, D = (int(x) for x in Q.shape)
    if int(block_q) <= 0 or int(block_k) <= 0 or int(granularity) <= 0:
        raise ValueError("block sizes and granularity must be positive")
    Tq, Tkv = _ceil_div(L, block_q), _ceil_div(L, block_k)
    sTq, sTkv = _ceil_div(Tq, granularity), _ceil_div(Tkv, granularity)
    for name, t in (("Q", Q), ("K", K), ("V", V), ("O", O)):
        _check(t, name, torch.bfloat16, (B, H, L, D))
    _check(O_cache, "O_cache", torch.bfloat16, (B, H, L, D), allow_none=True)
    _check(cache_flags, "cache_flags", torch.uint8, (B, H, sTq), allow_none=True)
    _check(kv_mask, "kv_mask", torch.uint8, (B, H, sTq, _ceil_div(sTkv, 8)), allow_none=True)
    _same_device((Q, K, V, O, O_cache, cache_flags, kv_mask))
    return B, H, L, D


def _fwd_args(Q, K, V, cache_flags, kv_mask, O_cache, O, block_q, block_k):
    B, H, L, D = _check_attn_tensors(Q, K, V, cache_flags, kv_mask, O_cache, O, block_q, block_k)
    return [_dev_ptr(Q, "Q"), _dev_ptr(K, "K"), _dev_ptr(V, "V"),
            _dev_ptr(cache_flags, "cache_flags", True), _dev_ptr(kv_mask, "kv_mask", True),
            _dev_ptr(O_cache, "O_cache", True), _dev_ptr(O, "O"),
            int(B), int(H), int(L), int(D), int(block_q), int(block_k)]


def sparse_attn_fwd(Q, K, V, cache_flags, kv_mask, O_cache, O, block_q, block_k, stream=None):
    """Algorithm 1 on device tensors (bf16 [B,H,L,D]); enqueued on `stream` (default: torch's current stream).

    cache_flags: uint8 [B,H,Tq] or None; kv_mask: uint8 [B,H,Tq,ceil(Tkv/8)] (see sparse_attn_pack_mask) or None;
    O_cache: bf16 [B,H,L,D], None or O itself (cached blocks already in place).  O is written in place.
    """
    args = _fwd_args(Q, K, V, cache_flags, kv_mask, O_cache, O, block_q, block_k)
    rc = load_library().sparse_attn_fwd_stream(*args, _stream_ptr(stream))
    if rc != 0:
        _raise(rc)
    return O


def sparse_attn_fwd_noalloc(Q, K, V, cache_flags, kv_mask, O_cache, O, block_q, block_k, stream=None):
    """sparse_attn_fwd through the entry point that allocates nothing (fixed scratch inside the library)."""
    args = _fwd_args(Q, K, V, cache_flags, kv_mask, O_cache, O, block_q, block_k)
    rc = load_library().sparse_attn_fwd_noalloc(*args, _stream_ptr(stream))
    if rc != 0:
        _raise(rc)
    return O


def sparse_attn_fwd_workspace(Q, K, V, cache_flags, kv_mask, O_cache, O, block_q, block_k, workspace, stream=None):
    """sparse_attn_fwd with the scratch memory supplied by the caller: `workspace` is a device uint8 tensor of at
    least sparse_attn_workspace_bytes(B, H, L, block_q, block_k) bytes, 256-byte aligned."""
    import torch
    args = _fwd_args(Q, K, V, cache_flags, kv_mask, O_cache, O, block_q, block_k)
    if workspace.dtype != torch.uint8 or workspace.dim() != 1:
        raise ValueError("workspace must be a one-dimensional uint8 tensor")
    rc = load_library().sparse_attn_fwd_workspace(*args, _dev_ptr(workspace, "workspace"), int(workspace.numel()),
                                                  _stream_ptr(stream))
    if rc != 0:
        _raise(rc)
    return O


def sparse_attn_release_scratch(stream=None) -> None:
    """Frees the library's scratch buffer of `stream` (default: torch's current stream) after waiting for it."""
    rc = load_library().sparse_attn_release_scratch(_stream_ptr(stream))
    if rc != 0:
        _raise(rc)


def sparse_attn_fwd_timed(Q, K, V, cache_flags, kv_mask, O_cache, O, block_q, block_k, stream=None):
    """Same work, timed with HIP events inside the library.  Returns (plan_ms, attn_ms)."""
    args = _fwd_args(Q, K, V, cache_flags, kv_mask, O_cache, O, block_q, block_k)
    plan, attn = ctypes.c_float(0), ctypes.c_float(0)
    rc = load_library().sparse_attn_fwd_timed(*args, _stream_ptr(stream), ctypes.byref(plan), ctypes.byref(attn))
    if rc != 0:
        _raise(rc)
    return plan.value, attn.value


def sparse_gemm_q(X, W, bias, cache_flags, Q, block_q, stream=None):
    """Sparse query projection on device tensors: X bf16 [B,L,C], W bf16 [H*D,C], bias bf16 [H*D] or None,
    cache_flags uint8 [B,H,ceil(L/block_q)] or None, Q bf16 [B,H,L,D] written in place for the computed blocks."""
    B, L, C = X.shape
    _, H, _, D = Q.shape
    if tuple(W.shape) != (H * D, C) or Q.shape[0] != B or Q.shape[2] != L:
        raise ValueError("shapes of X [B,L,C], W [H*D,C] and Q [B,H,L,D] do not fit together")
    rc = load_library().sparse_gemm_q_stream(_dev_ptr(X, "X"), _dev_ptr(W, "W"), _dev_ptr(bias, "bias", True),
                                             _dev_ptr(cache_flags, "cache_flags", True), _dev_ptr(Q, "Q"),
                                             int(B), int(L), int(C), int(H), int(D), int(block_q), _stream_ptr(stream))
    if rc != 0:
        _raise(rc)
    return Q


class SparseAttnPlan:
    """Handle of sparse_attn_plan_create: the symbol pre-pass stored for the Dispatch steps that reuse the symbols."""

    def __init__(self, cache_flags, kv_mask, B, H, L, block_q, block_k, granularity=1, stream=None):
        import torch
        self._h = ctypes.c_void_p()
        self.shape = (int(B), int(H), int(L))
        self.blocks = (int(block_q), int(block_k))
        if int(block_q) <= 0 or int(block_k) <= 0 or int(granularity) <= 0:
            raise ValueError("block sizes and granularity must be positive")
        sTq = _ceil_div(_ceil_div(L, block_q), granularity)
        sTkv = _ceil_div(_ceil_div(L, block_k), granularity)
        _check(cache_flags, "cache_flags", torch.uint8, (int(B), int(H), sTq), allow_none=True)
        _check(kv_mask, "kv_mask", torch.uint8, (int(B), int(H), sTq, _ceil_div(sTkv, 8)), allow_none=True)
        _same_device((cache_flags, kv_mask))
        rc = load_library().sparse_attn_plan_create(_dev_ptr(cache_flags, "cache_flags", True),
                                                    _dev_ptr(kv_mask, "kv_mask", True), int(B), int(H), int(L),
                                                    int(block_q), int(block_k), int(granularity), _stream_ptr(stream),
                                                    ctypes.byref(self._h))
        if rc != 0:
            _raise(rc)

    def run(self, Q, K, V, O_cache, O, stream=None):
        B, H, L, D = _check_attn_tensors(Q, K, V, None, None, O_cache, O, *self.blocks)
        if (B, H, L) != self.shape:
            raise ValueError("Q does not have the shape the plan was made for")
        rc = load_library().sparse_attn_plan_run(self._h, _dev_ptr(Q, "Q"), _dev_ptr(K, "K"), _dev_ptr(V, "V"),
                                                 _dev_ptr(O_cache, "O_cache", True), _dev_ptr(O, "O"), int(D),
                                                 _stream_ptr(stream))
        if rc != 0:
            _raise(rc)
        return O

    def run_forecast(self, Q, K, V, O_terms, coef, O, stream=None):
        """run() with OP_reuse = sum_d coef[d] * O_terms[d] in the cache branch (see sparse_attn_fwd_forecast)."""
        import torch
        B, H, L, D = _check_attn_tensors(Q, K, V, None, None, None, O, *self.blocks)
        if (B, H, L) != self.shape:
            raise ValueError("Q does not have the shape the plan was made for")
        for n, t in enumerate(O_terms):
            _check(t, f"O_terms[{n}]", torch.bfloat16, (B, H, L, D))
        ptrs, cf = _term_arrays(O_terms, coef, "O_terms")
        rc = load_library().sparse_attn_plan_run_forecast(self._h, _dev_ptr(Q, "Q"), _dev_ptr(K, "K"), _dev_ptr(V, "V"),
                                                          ptrs, cf, len(O_terms), _dev_ptr(O, "O"), int(D),
                                                          _stream_ptr(stream))
        if rc != 0:
            _raise(rc)
        return O

    def destroy(self):
        if self._h:
            rc = load_library().sparse_attn_plan_destroy(self._h)
            self._h = ctypes.c_void_p()
            if rc != 0:
                _raise(rc)

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def sparse_gemm_q_norm_rope(X, W, bias, norm_weight, eps, rope_cos, rope_sin, cache_flags, Q, block_q, stream=None):
    """sparse_gemm_q with token-wise RMSNorm (norm_weight bf16 [D] or None, eps) and RoPE on adjacent channel pairs
    (rope_cos, rope_sin fp32 [L, D/2], or both None) fused into the epilogue (Equation 2)."""
    B, L, C = X.shape
    _, H, _, D = Q.shape
    if tuple(W.shape) != (H * D, C) or tuple(Q.shape) != (B, H, L, D):
        raise ValueError("shapes of X [B,L,C], W [H*D,C] and Q [B,H,L,D] do not fit together")
    import torch
    for t, name in ((rope_cos, "rope_cos"), (rope_sin, "rope_sin")):
        if t is not None and (t.dtype != torch.float32 or tuple(t.shape) != (L, D // 2)):
            raise ValueError(f"{name} must be float32 [L, D/2]")
    if norm_weight is not None and (norm_weight.dtype != torch.bfloat16 or norm_weight.numel() != D):
        raise ValueError("norm_weight must be bfloat16 [D]")
    rc = load_library().sparse_gemm_q_norm_rope(_dev_ptr(X, "X"), _dev_ptr(W, "W"), _dev_ptr(bias, "bias", True),
                                                _dev_ptr(norm_weight, "norm_weight", True), float(eps),
                                                _dev_ptr(rope_cos, "rope_cos", True), _dev_ptr(rope_sin, "rope_sin", True),
                                                _dev_ptr(cache_flags, "cache_flags", True), _dev_ptr(Q, "Q"),
                                                int(B), int(L), int(C), int(H), int(D), int(block_q), _stream_ptr(stream))
    if rc != 0:
        _raise(rc)
    return Q


def sparse_gemm_o(O, W, bias, cache_flags, select_cached, addend, Out, block_q, stream=None):
    """Sparse output projection on device tensors: O bf16 [B,H,L,D], W bf16 [C_out,H*D], bias bf16 [C_out] or None,
    cache_flags uint8 [B,H,ceil(L/block_q)] or None, addend bf16 [B,L,C_out] / None / Out, Out bf16 [B,L,C_out] (written).
    select_cached = 1 sums the heads whose flag is set (stage 1, the cached bias), 0 the others (stage 2)."""
    B, H, L, D = O.shape
    C_out = W.shape[0]
    if tuple(W.shape) != (C_out, H * D) or tuple(Out.shape) != (B, L, C_out):
        raise ValueError("shapes of O [B,H,L,D], W [C_out,H*D] and Out [B,L,C_out] do not fit together")
    if addend is not None and tuple(addend.shape) != (B, L, C_out):
        raise ValueError("addend must have the shape of Out")
    rc = load_library().sparse_gemm_o_stream(_dev_ptr(O, "O"), _dev_ptr(W, "W"), _dev_ptr(bias, "bias", True),
                                             _dev_ptr(cache_flags, "cache_flags", True), int(select_cached),
                                             _dev_ptr(addend, "addend", True), _dev_ptr(Out, "Out"),
                                             int(B), int(H), int(L), int(D), int(C_out), int(block_q), _stream_ptr(stream))
    if rc != 0:
        _raise(rc)
    return Out


def sparse_gemm_o_reuse(O, W, bias, cache_flags, terms, coef, Out, block_q, stream=None):
    """GEMM-O stage 2 with the output initialised by OP_reuse(B_c) in one call: Out = sum_d coef[d] * terms[d] (rounded
    to bf16 once) + bias + the heads whose flag is clear.  terms: list of device tensors bf16 [B,L,C_out] (a term may
    be Out); bit-identical to sparse_op_reuse followed by sparse_gemm_o with that result as the addend."""
    import torch
    B, H, L, D = (int(x) for x in O.shape)
    C_out = int(W.shape[0])
    _check(O, "O", torch.bfloat16, (B, H, L, D))
    _check(W, "W", torch.bfloat16, (C_out, H * D))
    _check(Out, "Out", torch.bfloat16, (B, L, C_out))
    _check(bias, "bias", torch.bfloat16, (C_out,), allow_none=True)
    _check(cache_flags, "cache_flags", torch.uint8, (B, H, _ceil_div(L, block_q)), allow_none=True)
    for n, t in enumerate(terms):
        _check(t, f"terms[{n}]", torch.bfloat16, (B, L, C_out))
    ptrs, cf = _term_arrays(terms, coef, "terms")
    rc = load_library().sparse_gemm_o_reuse(_dev_ptr(O, "O"), _dev_ptr(W, "W"), _dev_ptr(bias, "bias", True),
                                            _dev_ptr(cache_flags, "cache_flags", True), ptrs, cf, len(terms),
                                            _dev_ptr(Out, "Out"), B, H, L, D, C_out, int(block_q), _stream_ptr(stream))
    if rc != 0:
        _raise(rc)
    return Out


def _term_arrays(terms, coef, name):
    if len(terms) != len(coef) or not terms:
        raise ValueError("one coefficient per term, at least one term")
    ptrs = (ctypes.c_void_p * len(terms))(*[_dev_ptr(t, f"{name}[{d}]").value for d, t in enumerate(terms)])
    cf = (ctypes.c_float * len(coef))(*[float(c) for c in coef])
    return ptrs, cf


def sparse_attn_fwd_forecast(Q, K, V, cache_flags, kv_mask, O_terms, coef, O, block_q, block_k, stream=None):
    """Algorithm 1 with OP_reuse = sum_d coef[d] * O_terms[d] in the cache branch (Taylor forecast of cached blocks).
    O_terms: list of device tensors bf16 [B,H,L,D]; coef: list of floats (see sparse_taylor_coefficients)."""
    import torch
    B, H, L, D = _check_attn_tensors(Q, K, V, cache_flags, kv_mask, None, O, block_q, block_k)
    for n, t in enumerate(O_terms):
        _check(t, f"O_terms[{n}]", torch.bfloat16, (B, H, L, D))
    ptrs, cf = _term_arrays(O_terms, coef, "O_terms")
    rc = load_library().sparse_attn_fwd_forecast(_dev_ptr(Q, "Q"), _dev_ptr(K, "K"), _dev_ptr(V, "V"),
                                                 _dev_ptr(cache_flags, "cache_flags", True),
                                                 _dev_ptr(kv_mask, "kv_mask", True), ptrs, cf, len(O_terms),
                                                 _dev_ptr(O, "O"), int(B), int(H), int(L), int(D), int(block_q),
                                                 int(block_k), _stream_ptr(stream))
    if rc != 0:
        _raise(rc)
    return O


def sparse_op_reuse(terms, coef, out, stream=None):
    """out = sum_d coef[d] * terms[d], element-wise on device bf16 tensors of one shape (a term may be `out`)."""
    n = out.numel()
    for t in terms:
        if t.numel() != n:
            raise ValueError("every term must have as many elements as out")
    ptrs, cf = _term_arrays(terms, coef, "terms")
    rc = load_library().sparse_op_reuse(ptrs, cf, len(terms), _dev_ptr(out, "out"), int(n), _stream_ptr(stream))
    if rc != 0:
        _raise(rc)
    return out


def sparse_taylor_update(fresh, terms, n_valid, interval, stream=None):
    """Refresh the stored forecast terms in place from a freshly computed feature (backward finite differences over
    `interval` steps); n_valid = number of terms that were valid before this call."""
    n = fresh.numel()
    for t in terms:
        if t.numel() != n:
            raise ValueError("every term must have as many elements as fresh")
    ptrs = (ctypes.c_void_p * len(terms))(*[_dev_ptr(t, f"terms[{d}]").value for d, t in enumerate(terms)])
    rc = load_library().sparse_taylor_update(_dev_ptr(fresh, "fresh"), ptrs, len(terms), int(n_valid), float(interval),
                                             int(n), _stream_ptr(stream))
    if rc != 0:
        _raise(rc)
    return terms


def sparse_taylor_coefficients(order, steps):
    """[steps^d / d! for d = 0..order] as the library computes them (float32 values)."""
    buf = (ctypes.c_float * (int(order) + 1))()
    load_library().sparse_taylor_coefficients(int(order), float(steps), buf)
    return [float(x) for x in buf]


def sparse_symbols_update(Q, K, cache_flags, kv_mask, block, text_tokens, tau_c, tau_kv, s_q=0.0, stream=None,
                          block_k=None, granularity=1):
    """Symbol generation of an Update step on device tensors: Q, K bf16 [B,H,L,D]; writes cache_flags uint8 [B,H,Tq]
    (1 = cached) and kv_mask uint8 [B,H,Tq,ceil(Tk/8)] (bit = 1 keeps the pair, first block in bit 7), with
    Tq = ceil(L / (granularity * block)), Tk = ceil(L / (granularity * block_k)); block is b_q, block_k defaults to it."""
    import torch
    block_k = block if block_k is None else block_k
    if Q.dim() != 4:
        raise ValueError("Q must be [B, H, L, D]")
    B, H, L, D = (int(x) for x in Q.shape)
    if int(block) <= 0 or int(block_k) <= 0 or int(granularity) <= 0:
        raise ValueError("block sizes and granularity must be positive")
    Tq, Tk = _ceil_div(L, granularity * block), _ceil_div(L, granularity * block_k)
    _check(Q, "Q", torch.bfloat16, (B, H, L, D))
    _check(K, "K", torch.bfloat16, (B, H, L, D))
    _check(cache_flags, "cache_flags", torch.uint8, (B, H, Tq))
    _check(kv_mask, "kv_mask", torch.uint8, (B, H, Tq, _ceil_div(Tk, 8)))
    _same_device((Q, K, cache_flags, kv_mask))
    rc = load_library().sparse_symbols_update_granular(_dev_ptr(Q, "Q"), _dev_ptr(K, "K"),
                                                       _dev_ptr(cache_flags, "cache_flags"), _dev_ptr(kv_mask, "kv_mask"),
                                                       B, H, L, D, int(block), int(block_k), int(granularity),
                                                       int(text_tokens), float(tau_c), float(tau_kv), float(s_q),
                                                       _stream_ptr(stream))
    if rc != 0:
        _raise(rc)
    return cache_flags, kv_mask


def sparse_attn_profile_begin(max_calls: int) -> None:
    rc = load_library().sparse_attn_profile_begin(int(max_calls))
    if rc != 0:
        _raise(rc)


def sparse_attn_profile_end():
    """Returns (calls, plan_ms_total, attn_ms_total) of the calls recorded since profile_begin."""
    calls, plan, attn = ctypes.c_int(0), ctypes.c_double(0), ctypes.c_double(0)
    rc = load_library().sparse_attn_profile_end(ctypes.byref(calls), ctypes.byref(plan), ctypes.byref(attn))
    if rc != 0:
        _raise(rc)
    return calls.value, plan.value, attn.value


def sparse_attn_workspace_bytes(B, H, L, block_q, block_k) -> int:
    return int(load_library().sparse_attn_workspace_bytes(B, H, L, block_q, block_k))


def sparse_attn_count_kept(cache_flags, kv_mask, B, H, L, block_q, block_k):
    """(kept, total) pair counts from HOST numpy arrays (uint8), either may be None."""
    def host(a):
        if a is None:
            return None, None
        a = np.ascontiguousarray(a, dtype=np.uint8)
        return a, a.ctypes.data_as(ctypes.c_void_p)
    f, fp = host(cache_flags)
    m, mp = host(kv_mask)
    kept, total = ctypes.c_ulonglong(0), ctypes.c_ulonglong(0)
    rc = load_library().sparse_attn_count_kept(fp, mp, B, H, L, block_q, block_k, ctypes.byref(kept), ctypes.byref(total))
    if rc != 0:
        _raise(rc)
    return kept.value, total.value


def sparse_attn_pack_mask(logical):
    """Pack a HOST logical mask (numpy, last axis = key blocks, non-zero = keep) into kv_mask bytes."""
    a = np.ascontiguousarray(logical)
    a = (a != 0).astype(np.uint8)
    Tkv = a.shape[-1]
    rows = int(np.prod(a.shape[:-1])) if a.ndim > 1 else 1
    out = np.empty(a.shape[:-1] + ((Tkv + 7) // 8,), dtype=np.uint8)
    rc = load_library().sparse_attn_pack_mask(a.ctypes.data_as(ctypes.c_void_p), rows, Tkv,
                                              out.ctypes.data_as(ctypes.c_void_p))
    if rc != 0:
        _raise(rc)
    return out
