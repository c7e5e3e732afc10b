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


def rms_norm(y, weight, eps):
    """Token-wise RMS normalisation over the last axis: y / sqrt(mean(y^2) + eps) * weight."""
    ms = (y * y).mean(axis=-1, keepdims=True)
    out = y / np.sqrt(ms + eps)
    return out if weight is None else out * weight


def rope(y, cos, sin):
    """Rotary position encoding on adjacent channel pairs: (y[2m], y[2m+1]) of token l is rotated by the
    angle whose cosine and sine are cos[l, m], sin[l, m].  y: [L, D]; cos, sin: [L, D/2]."""
    even, odd = y[..., 0::2], y[..., 1::2]
    out = np.empty_like(y)
    out[..., 0::2] = even * cos - odd * sin
    out[..., 1::2] = even * sin + odd * cos
    return out


def gemm_q(X, W, bias, cache_flags, block_q, H, D, Q_init_bits=None, norm_weight=None, eps=None, rope_cos=None,
           rope_sin=None):
    """X: uint16 bf16 bits [B, L, C]; W: [H*D, C] (one row per output feature, as a Linear layer
    stores it); bias: [H*D] or None; cache_flags: uint8 [B, H, L/block_q] or None.

    With eps given, the projection of every (token, head) is RMS-normalised over its D channels
    (norm_weight: uint16 bf16 bits [D] or None for ones) and, with rope_cos / rope_sin (float [L, D/2])
    given, rotated -- Equation 2's OP_RoPE(OP_RMSNorm(X W)), both token-wise -- before the one
    rounding to bf16.

    Returns (Q_f64, Q_bits) of shape [B, H, L, D].  Skipped blocks keep Q_init_bits (zeros if
    not given) in Q_bits and its widened value in Q_f64.
    """
    X = np.ascontiguousarray(X, dtype=np.uint16)
    W = np.ascontiguousarray(W, dtype=np.uint16)
    B, L, C = X.shape
    if W.shape != (H * D, C):
        raise ValueError("W must be [H*D, C]")
    Tq = -(-L // block_q)      # Definition 1 counts ceil(L / b) blocks: the last token block may be short
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
            if eps is not None:
                full = rms_norm(full, None if norm_weight is None else _widen(norm_weight), float(eps))
            if rope_cos is not None:
                full = rope(full, np.asarray(rope_cos, dtype=np.float64), np.asarray(rope_sin, dtype=np.float64))
            for i in range(Tq):
                if cache_flags is not None and cache_flags[b, h, i]:
                    continue
                rows = slice(i * block_q, (i + 1) * block_q)
                Q_f64[b, h, rows] = full[rows]
                Q_bits[b, h, rows] = _narrow(full[rows])
    return Q_f64, Q_bits


def computed_flops(cache_flags, B, H, L, C, D, block_q):
    """2*bq*D*C per computed (b,h,i) tile: the work the projection actually does."""
    Tq = -(-L // block_q)
    n = B * H * Tq if cache_flags is None else int((np.asarray(cache_flags) == 0).sum())
    return 2.0 * block_q * D * C * n
