"""ctypes front-end of the C oracle, and the symbol packer of Section 3.3.

TEST INFRASTRUCTURE ONLY (see the package docstring).
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liboracle_sparse_attn.so")
_lib = None


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        from . import build as _build
        _build.build()
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64
    lib.oracle_sparse_attn.argtypes = [vp] * 6 + [i32] * 6 + [vp, vp]
    lib.oracle_sparse_attn.restype = i32
    lib.oracle_sparse_attn_blocks.argtypes = [vp] * 6 + [i32] * 6 + [vp, i64, vp, vp]
    lib.oracle_sparse_attn_blocks.restype = i32
    lib.oracle_count_pairs.argtypes = [vp, vp] + [i32] * 5 + [ctypes.POINTER(i64)] * 2
    lib.oracle_count_pairs.restype = i32
    lib.oracle_num_threads.argtypes = []
    lib.oracle_num_threads.restype = i32
    _lib = lib
    return lib


# --------------------------------------------------------------------------------------
# Section 3.3, "Sparse Symbols Compression": logical {0,1} masks -> uint8 symbols.
# Logical entry t goes to byte t // 8, bit 7 - t % 8 (most significant bit first); the
# last byte is padded with zeros.  The printed example [1,1,1,0] -> 0b11100000 = 224 is
# what fixes the bit order.
# --------------------------------------------------------------------------------------
def pack_symbols(bits, flat=False):
    """Pack logical mask entries along the last axis.

    flat=False: every row (all leading axes) is padded to whole bytes on its own; this is
    the layout the attention entry point takes for S_s.  flat=True: the whole array is one
    bit stream (the paper's J index (i/n)(T_kv/n) + j/n), padded once at the end.
    """
    bits = np.asarray(bits)
    if not np.isin(bits, (0, 1)).all():
        raise ValueError("logical masks hold only 0 and 1")
    bits = bits.astype(np.uint8)
    if flat:
        bits = bits.reshape(-1)
    n = bits.shape[-1]
    nbytes = (n + 7) // 8
    out = np.zeros(bits.shape[:-1] + (nbytes,), dtype=np.uint8)
    for t in range(n):
        out[..., t // 8] |= (bits[..., t] << (7 - t % 8)).astype(np.uint8)
    return out


def unpack_symbols(symbols, n):
    """Inverse of pack_symbols(flat=False): first n logical entries of every row."""
    symbols = np.asarray(symbols, dtype=np.uint8)
    out = np.zeros(symbols.shape[:-1] + (n,), dtype=np.uint8)
    for t in range(n):
        out[..., t] = (symbols[..., t // 8] >> (7 - t % 8)) & 1
    return out


def expand_granularity(cache_flags, M_s, n, Tq, Tkv):
    """Symbols at granularity n (one entry per n x n tiles, Section 3.3) -> one entry per tile, following the
    decoding functions of Section 3.4: tile (i, j) reads flag i // n and mask entry (i // n, j // n).
    cache_flags: [B,H,ceil(Tq/n)] or None; M_s: logical [B,H,ceil(Tq/n),ceil(Tkv/n)] or None."""
    f = None if cache_flags is None else np.repeat(np.asarray(cache_flags), n, axis=2)[:, :, :Tq]
    m = None if M_s is None else np.repeat(np.repeat(np.asarray(M_s), n, axis=2), n, axis=3)[:, :, :Tq, :Tkv]
    return f, m


def _u16(a, name):
    a = np.ascontiguousarray(a)
    if a.dtype != np.uint16:
        raise TypeError(f"{name} must hold bf16 bit patterns as uint16")
    return a


def _u8_or_none(a):
    if a is None:
        return None
    a = np.ascontiguousarray(a)
    if a.dtype != np.uint8:
        raise TypeError("symbols must be uint8")
    return a


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _check(Q, K, V, cache_flags, kv_mask, O_cache, block_q, block_k):
    B, H, L, D = Q.shape
    if K.shape != Q.shape or V.shape != Q.shape:
        raise ValueError("Q, K, V must share the shape [B, H, L, D]")
    Tq, Tkv = -(-L // block_q), -(-L // block_k)      # Definition 1: ceil(L / b) blocks, the last may be short
    if cache_flags is not None and cache_flags.shape != (B, H, Tq):
        raise ValueError("cache_flags must be [B, H, Tq]")
    if kv_mask is not None and kv_mask.shape != (B, H, Tq, (Tkv + 7) // 8):
        raise ValueError("kv_mask must be [B, H, Tq, ceil(Tkv/8)]")
    if O_cache is not None and O_cache.shape != Q.shape:
        raise ValueError("O_cache must have the shape of Q")
    return B, H, L, D, Tq, Tkv


def sparse_attention(Q, K, V, cache_flags, kv_mask, O_cache, block_q, block_k,
                     O_init_bits=None):
    """Algorithm 1 on whole tensors (bf16 bit patterns in, uint16 arrays [B,H,L,D]).

    Returns (O_f64, O_bits).  Computed blocks: fp64 result and its bf16 rounding.
    Cached blocks: O_cache's raw bits (and their widened value).  With O_cache None the
    cached blocks keep whatever O_init_bits holds (zeros if not given) -- the
    early-continue of the cache branch of Algorithm 1.
    """
    Q, K, V = _u16(Q, "Q"), _u16(K, "K"), _u16(V, "V")
    cache_flags, kv_mask = _u8_or_none(cache_flags), _u8_or_none(kv_mask)
    O_cache = None if O_cache is None else _u16(O_cache, "O_cache")
    B, H, L, D, _, _ = _check(Q, K, V, cache_flags, kv_mask, O_cache, block_q, block_k)
    if O_init_bits is None:
        O_bits = np.zeros(Q.shape, dtype=np.uint16)
    else:
        O_bits = _u16(O_init_bits, "O_init_bits").copy()
    O_f64 = (O_bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    rc = _load().oracle_sparse_attn(_ptr(Q), _ptr(K), _ptr(V), _ptr(cache_flags), _ptr(kv_mask),
                                    _ptr(O_cache), B, H, L, D, block_q, block_k,
                                    _ptr(O_f64), _ptr(O_bits))
    if rc != 0:
        raise RuntimeError(f"oracle_sparse_attn failed with {rc}")
    return O_f64, O_bits


def sparse_attention_blocks(Q, K, V, cache_flags, kv_mask, O_cache, block_q, block_k, items):
    """Algorithm 1 on selected query blocks only.

    items: flattened indices (b*H + h)*Tq + i.  Returns (O_f64, O_bits) of shape
    [len(items), block_q, D]; rows of cached items with O_cache None stay zero.
    """
    Q, K, V = _u16(Q, "Q"), _u16(K, "K"), _u16(V, "V")
    cache_flags, kv_mask = _u8_or_none(cache_flags), _u8_or_none(kv_mask)
    O_cache = None if O_cache is None else _u16(O_cache, "O_cache")
    B, H, L, D, Tq, _ = _check(Q, K, V, cache_flags, kv_mask, O_cache, block_q, block_k)
    items = np.ascontiguousarray(items, dtype=np.int64)
    if items.ndim != 1 or (items.size and (items.min() < 0 or items.max() >= B * H * Tq)):
        raise ValueError("items out of range")
    O_f64 = np.zeros((items.size, block_q, D), dtype=np.float64)
    O_bits = np.zeros((items.size, block_q, D), dtype=np.uint16)
    rc = _load().oracle_sparse_attn_blocks(_ptr(Q), _ptr(K), _ptr(V), _ptr(cache_flags),
                                           _ptr(kv_mask), _ptr(O_cache), B, H, L, D, block_q,
                                           block_k, _ptr(items), items.size, _ptr(O_f64),
                                           _ptr(O_bits))
    if rc != 0:
        raise RuntimeError(f"oracle_sparse_attn_blocks failed with {rc}")
    return O_f64, O_bits


def count_pairs(cache_flags, kv_mask, B, H, L, block_q, block_k):
    """(kept, total) pair counts of Section 4.1: kept = computed (Q_i K_j^T, P_ij V_j) pairs."""
    cache_flags, kv_mask = _u8_or_none(cache_flags), _u8_or_none(kv_mask)
    kept, total = ctypes.c_int64(0), ctypes.c_int64(0)
    rc = _load().oracle_count_pairs(_ptr(cache_flags), _ptr(kv_mask), B, H, L, block_q, block_k,
                                    ctypes.byref(kept), ctypes.byref(total))
    if rc != 0:
        raise RuntimeError(f"oracle_count_pairs failed with {rc}")
    return kept.value, total.value


def sparsity(cache_flags, kv_mask, B, H, L, block_q, block_k):
    """Sparsity = skip / total (Section 4.1)."""
    kept, total = count_pairs(cache_flags, kv_mask, B, H, L, block_q, block_k)
    return (total - kept) / total


def num_threads():
    return int(_load().oracle_num_threads())
