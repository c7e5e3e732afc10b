"""Test-side helpers: independent brute-force attention (numpy/scipy) and bf16 views.

The brute force takes a different route from the oracle on purpose: it expands the block
mask to one boolean per (query, key) element, adds -inf to masked scores and calls
library softmax and matmul on whole matrices.
"""
import numpy as np
from scipy.special import softmax


def bits_to_f64(bits):
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def brute_force_attention(Q, K, V, M_s, cache_flags, block_q, block_k):
    """Q,K,V: uint16 bf16 bits [B,H,L,D]; M_s: {0,1} [B,H,Tq,Tkv] or None.

    Returns fp64 [B,H,L,D] with NaN in rows of cached blocks (they are not attention
    outputs) and 0 in computed rows whose mask row is empty.
    """
    Qf, Kf, Vf = bits_to_f64(Q), bits_to_f64(K), bits_to_f64(V)
    B, H, L, D = Qf.shape
    Tq = -(-L // block_q)
    out = np.empty((B, H, L, D), dtype=np.float64)
    for b in range(B):
        for h in range(H):
            S = Qf[b, h] @ Kf[b, h].T / np.sqrt(D)
            if M_s is not None:
                elem = np.kron(np.asarray(M_s[b, h], dtype=bool), np.ones((block_q, block_k), dtype=bool))[:L, :L]
                S = np.where(elem, S, -np.inf)
            empty = ~np.isfinite(S).any(axis=1)
            S[empty] = 0.0
            P = softmax(S, axis=1)
            O = P @ Vf[b, h]
            O[empty] = 0.0
            if cache_flags is not None:
                for i in range(Tq):
                    if cache_flags[b, h, i]:
                        O[i * block_q:(i + 1) * block_q] = np.nan
            out[b, h] = O
    return out


def computed_row_mask(cache_flags, B, H, L, block_q):
    """bool [B,H,L]: True for rows that belong to computed (non-cached) blocks."""
    if cache_flags is None:
        return np.ones((B, H, L), dtype=bool)
    return np.repeat(np.asarray(cache_flags) == 0, block_q, axis=2)[:, :, :L]
