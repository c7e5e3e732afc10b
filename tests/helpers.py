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


# --- comparison of generated sparse symbols with the fp64 oracle -------------------------------------------------
EPS_FLAG = 1e-4     # caching decisions: distance from flipping, relative to the metric's total
EPS_SKIP = 2e-5     # skipping decisions: absolute (rows of the compressed map sum to one)


def decidable_symbols(ref, eps_flag=EPS_FLAG, eps_skip=EPS_SKIP):
    """Which of the oracle's yes/no decisions an fp32 evaluation has to reproduce: those whose deciding sum is
    further from its threshold than rounding can move it (eps) and than a swap with a near-equal neighbour in the
    ascending order could move it (twice the entry's own share).  Returns (flags [B,H,T], pairs [B,H,T,T]) booleans."""
    robust_f = ref["flag_margin"] > eps_flag + np.where(ref["flag_tie"], 2 * ref["flag_window"], 0.0)
    robust_s = np.abs(ref["skip_margin"]) > eps_skip + np.where(ref["skip_tie"], 2 * ref["own_value"], 0.0)
    return robust_f, robust_s


def compare_symbols(ref, flags, bits, label, max_ambiguous=0.02, require_identical=False):
    """flags [B,H,T] and bits [B,H,T,T] (unpacked mask) against the oracle's symbols.  Every decidable decision must
    agree and the undecidable ones must be rare; with require_identical every decision must agree."""
    assert set(np.unique(flags)) <= {0, 1} and set(np.unique(bits)) <= {0, 1}
    robust_f, robust_s = decidable_symbols(ref)
    diff_f, diff_s = flags != ref["cache_flags"], bits != ref["M_s"]
    print(f"[symbols] {label}: cached {ref['cache_flags'].mean():.3f} kept {ref['M_s'].mean():.3f} "
          f"undecidable flags {(~robust_f).mean():.4f} pairs {(~robust_s).mean():.5f} "
          f"raw mismatches flags {diff_f.sum()} pairs {diff_s.sum()}", flush=True)
    assert not (diff_f & robust_f).any(), f"{label}: {(diff_f & robust_f).sum()} cache flags differ from the oracle beyond rounding"
    assert not (diff_s & robust_s).any(), f"{label}: {(diff_s & robust_s).sum()} mask bits differ from the oracle beyond rounding"
    assert (~robust_f).mean() <= max_ambiguous and (~robust_s).mean() <= max_ambiguous, f"{label}: too many undecidable entries"
    if require_identical:
        worst_f = ref["flag_margin"][diff_f].max() if diff_f.any() else 0.0
        worst_s = np.abs(ref["skip_margin"][diff_s]).max() if diff_s.any() else 0.0
        assert not diff_f.any() and not diff_s.any(), (
            f"{label}: {diff_f.sum()} flags / {diff_s.sum()} mask bits differ from the oracle "
            f"(largest margins {worst_f:.2e} / {worst_s:.2e}: all inside the rounding window, but this input is "
            "expected to be reproduced exactly)")
