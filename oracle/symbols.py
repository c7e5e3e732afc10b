"""CPU oracle of the sparse-symbol generation of an Update step (Section 3.3 "Logical Masks Generation",
Equation 1, and the tau_q / tau_kv / S_q descriptions of the settings table in the appendix).

TEST INFRASTRUCTURE ONLY.  The steps follow the paper's order; every place where its text leaves a choice
is stated next to the step.  Per (batch, head), with block size b
(= b_q = b_k, granularity n = 1), T = L / b blocks, the first n_t = N_text / b blocks being text:

 1. token gathering: q~_i, k~_j = mean of the b query / key rows of block i / j;
 2. compressed map: S~ = q~ k~^T / sqrt(d) (scale as in Section 3.1), P~ = row softmax of S~;
 3. vision-to-text contribution of vision block v:  C_v = sum over text rows j < n_t of P~[j, n_t + v];
 4. text-to-vision guidance: beta = softmax along the vision axis of (P~[n_t:, :n_t])^T, G_v = sum_j beta[j, v];
 5. Equation 1: with CumSum_up(X)_v the sum of all X_u that come at or before X_v in ascending order (ties by
    index), vision block v is cached iff CumSum_up(C)_v <= tau_c * sum(C) and CumSum_up(G)_v <= tau_c * sum(G);
    text blocks are never cached (Observation 1);
 6. degrade rule (S_q): if the fraction of blocks of the head that still need computation is below S_q, every
    block of the head is cached;
 7. block-sparse skipping (tau_kv): in every row i of P~ the blocks are taken in ascending order of P~[i, j]
    and block j is skipped iff CumSum_up(P~[i, :])_j <= tau_kv (rows of P~ sum to one) -- the same rule as
    Equation 1, the only formal statement of "until the cumulative importance exceeds the threshold".

Besides the symbols the oracle returns, for every yes/no decision, how far the deciding quantity is from its
threshold (and whether a near-tie in the ordering could move it), so that a test can tell a real
disagreement from a decision that floating point cannot make reliably.  All arithmetic is IEEE double.
"""
import numpy as np

from .gemm_q import _widen


def _softmax(x, axis=-1):
    m = x.max(axis=axis, keepdims=True)
    e = np.exp(x - m)
    return e / e.sum(axis=axis, keepdims=True)


def _cumsum_up(x):
    """Inclusive cumulative sum in ascending order of x (ties by index), returned in x's own order,
    plus the relative gap of every element to its nearest neighbour in that order."""
    order = np.argsort(x, kind="stable")
    cs_sorted = np.cumsum(x[order])
    cs = np.empty_like(cs_sorted)
    cs[order] = cs_sorted
    xs = x[order]
    gap_sorted = np.full(x.shape, np.inf)
    if x.size > 1:
        d = np.diff(xs)
        gap_sorted[:-1] = d
        gap_sorted[1:] = np.minimum(gap_sorted[1:], d)
    rel = gap_sorted / np.maximum(np.abs(xs), 1e-300)
    gap = np.empty_like(rel)
    gap[order] = rel
    return cs, gap


def compressed_map(Q, K, block):
    """Steps 1-2.  Q, K: uint16 bf16 bits [B,H,L,D].  Returns P~ as fp64 [B,H,T,T]."""
    Qf, Kf = _widen(Q), _widen(K)
    B, H, L, D = Qf.shape
    T = -(-L // block)          # a short last block counts as a block; its mean is over the tokens that exist
    qt = np.stack([Qf[:, :, t * block:(t + 1) * block].mean(axis=2) for t in range(T)], axis=2)
    kt = np.stack([Kf[:, :, t * block:(t + 1) * block].mean(axis=2) for t in range(T)], axis=2)
    S = np.einsum("bhid,bhjd->bhij", qt, kt) / np.sqrt(D)
    return _softmax(S, axis=-1)


def caching_metrics(P, n_t):
    """Steps 3-4 for one head.  P: [T,T].  Returns (C, G), each of length T - n_t."""
    C = P[:n_t, n_t:].sum(axis=0)
    beta = _softmax(P[n_t:, :n_t].T, axis=-1)
    G = beta.sum(axis=0)
    return C, G


def update_symbols(Q, K, block, text_tokens, tau_c, tau_kv, s_q=0.0, tie_rel=1e-5):
    """Steps 1-7 on whole tensors.

    Returns a dict with
      cache_flags  uint8 [B,H,T]      1 = block is cached (the ABI's polarity: M_c = 1 - cache_flags)
      M_s          uint8 [B,H,T,T]    1 = compute the pair
      flag_margin  fp64  [B,H,T]      signed distance of the caching decision from flipping, relative to the metric's
                                      sum (min over the two conditions when cached, max when not); +inf for text
                                      blocks and for heads decided by the degrade rule
      flag_tie     bool  [B,H,T]      a near-tie in the ascending order could move this block's cumulative sums
      flag_window  fp64  [B,H,T]      ... by at most this much (the block's own share of the metric's total)
      skip_margin  fp64  [B,H,T,T]    tau_kv - CumSum_up (positive = skipped)
      skip_tie     bool  [B,H,T,T]
      own_value    fp64  [B,H,T,T]    P~ itself (how far a near-tie can move a cumulative sum)
    """
    B, H, L, D = np.asarray(Q).shape
    if text_tokens % block or not (0 < text_tokens < L):
        raise ValueError("the text length must be a multiple of the block size, with vision tokens left over")
    T, n_t = -(-L // block), text_tokens // block
    P = compressed_map(Q, K, block)
    flags = np.zeros((B, H, T), dtype=np.uint8)
    flag_margin = np.full((B, H, T), np.inf)
    flag_tie = np.zeros((B, H, T), dtype=bool)
    flag_window = np.zeros((B, H, T))
    M_s = np.ones((B, H, T, T), dtype=np.uint8)
    skip_margin = np.zeros((B, H, T, T))
    skip_tie = np.zeros((B, H, T, T), dtype=bool)
    for b in range(B):
        for h in range(H):
            C, G = caching_metrics(P[b, h], n_t)
            csC, gapC = _cumsum_up(C)
            csG, gapG = _cumsum_up(G)
            # the totals are the last entries of the ascending sums, so that tau_c = 1 selects every block
            # whatever the rounding order
            dC = (tau_c * csC.max() - csC) / csC.max()
            dG = (tau_c * csG.max() - csG) / csG.max()
            cached = (dC >= 0) & (dG >= 0)
            flags[b, h, n_t:] = cached
            flag_margin[b, h, n_t:] = np.where(cached, np.minimum(dC, dG), np.maximum(np.where(dC < 0, -dC, 0), np.where(dG < 0, -dG, 0)))
            flag_tie[b, h, n_t:] = (gapC < tie_rel) | (gapG < tie_rel)
            flag_window[b, h, n_t:] = np.maximum(C / csC.max(), G / csG.max())
            if (T - int(cached.sum())) / T < s_q:
                flags[b, h, :] = 1
                flag_margin[b, h, :] = np.inf
                flag_tie[b, h, :] = False
            for i in range(T):
                cs, gap = _cumsum_up(P[b, h, i])
                skip_margin[b, h, i] = tau_kv - cs
                skip_tie[b, h, i] = gap < tie_rel
                M_s[b, h, i] = (cs > tau_kv).astype(np.uint8)
    return dict(cache_flags=flags, M_s=M_s, flag_margin=flag_margin, flag_tie=flag_tie, flag_window=flag_window,
                skip_margin=skip_margin, skip_tie=skip_tie, own_value=P)
