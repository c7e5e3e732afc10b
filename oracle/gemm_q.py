"""CPU oracle of the sparse query projection (GEMM-Q, Section 3.5, Observation 2 / Equation 2).

TEST INFRASTRUCTURE ONLY.  What is computed: for every (batch b, head h, query block i) whose
cache flag is clear, the block of the query tensor is the plain projection
    Q[b, h, i*bq:(i+1)*bq, :] = X[b, i*bq:(i+1)*bq, :] @ W_h^T (+ bias_h)
with W_h the D rows of the projection weight that belong to head h; blocks whose flag is set
(their attention output will be reused from the cache, so their queries are never read) are
left exactly as they were.  Arithmetic is IEEE double on the exactly widened bf16 inputs; the
library matmul is the only primitive.
"""
import numpy as np


def _widen(bits):
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def _narrow(x):
    """fp64 -> fp32 -> bf16, round to nearest even; returns uint16 patterns (statistics copy only)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    return ((u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)).astype(np.uint16)


def gemm_q(X, W, bias, cache_flags, block_q, H, D, Q_init_bits=None):
    """X: uint16 bf16 bits [B, L, C]; W: [H*D, C] (one row per output feature, as a Linear layer
    stores it); bias: [H*D] or None; cache_flags: uint8 [B, H, L/block_q] or None.

    Returns (Q_f64, Q_bits) of shape [B, H, L, D].  Skipped blocks keep Q_init_bits (zeros if
    not given) in Q_bits and its widened value in Q_f64.
    """
    X = np.ascontiguousarray(X, dtype=np.uint16)
    W = np.ascontiguousarray(W, dtype=np.uint16)
    B, L, C = X.shape
    if W.shape != (H * D, C):
        raise ValueError("W must be [H*D, C]")
    if L % block_q:
        raise ValueError("L must be a multiple of block_q")
    Tq = L // block_q
    if cache_flags is not None and np.asarray(cache_flags).shape != (B, H, Tq):
        raise ValueError("cache_flags must be [B, H, Tq]")
    Q_bits = np.zeros((B, H, L, D), dtype=np.uint16) if Q_init_bits is None else np.array(Q_init_bits, dtype=np.uint16, copy=True)
    Q_f64 = _widen(Q_bits)
    Xf, Wf = _widen(X), _widen(W)
    bf = None if bias is None else _widen(bias)
    for b in range(B):
        for h in range(H):
            full = Xf[b] @ Wf[h * D:(h + 1) * D].T          # [L, D]
            if bf is not None:
                full = full + bf[h * D:(h + 1) * D][None, :]
            for i in range(Tq):
                if cache_flags is not None and cache_flags[b, h, i]:
                    continue
                rows = slice(i * block_q, (i + 1) * block_q)
                Q_f64[b, h, rows] = full[rows]
                Q_bits[b, h, rows] = _narrow(full[rows])
    return Q_f64, Q_bits


def computed_flops(cache_flags, B, H, L, C, D, block_q):
    """2*bq*D*C per computed (b,h,i) tile: the work the projection actually does."""
    Tq = L // block_q
    n = B * H * Tq if cache_flags is None else int((np.asarray(cache_flags) == 0).sum())
    return 2.0 * block_q * D * C * n
