"""CPU oracle of the sparse-symbol generation of an Update step (Section 3.3 "Logical Masks Generation",
Equation 1, and the tau_q / tau_kv / S_q descriptions of the settings table in the appendix).

TEST INFRASTRUCTURE ONLY.  The steps follow the paper's order; every place where its text leaves a choice
is stated next to the step.  Per (batch, head), with query and key block sizes b_q, b_k and symbol
granularity n (one symbol covers n consecutive blocks), N_text leading text tokens:

 1. token gathering: q~_i = mean of the n*b_q query rows of pooled block i, k~_j = mean of the n*b_k key rows
    of pooled block j (a short last block is averaged over the tokens that exist); T_q = ceil(L / (n b_q)) and
    T_k = ceil(L / (n b_k)) pooled blocks, of which the first n_tq = ceil(N_text / (n b_q)) and
    n_tk = ceil(N_text / (n b_k)) count as text (the ceiling of Section 3.3: a pooled block that holds any
    text token is a text block);
 2. compressed map: S~ = q~ k~^T / sqrt(d) (scale as in Section 3.1), P~ = row softmax of S~, [T_q, T_k];
 3. vision-to-text contribution: alpha = P~[:n_tq, n_tk:], C_u = sum over text rows of alpha[:, u], one value per
    vision KEY block u;
 4. text-to-vision guidance: beta = softmax along the vision axis of (P~[n_tq:, :n_tk])^T, G_v = sum_j beta[j, v],
    one value per vision QUERY block v;
 5. Equation 1 decides per vision query block (an output block is what gets cached), so C is carried over to
    the query axis: C_v = sum_u C_u * |tokens of v and u in common| / |tokens of u| (each key block's
    contribution spread evenly over its tokens; the identity when n b_q = n b_k).  With CumSum_up(X)_v the sum of
    all X_u that come at or before X_v in ascending order (ties by index), block v is cached iff
    CumSum_up(C)_v <= tau_c * sum(C) and CumSum_up(G)_v <= tau_c * sum(G); text blocks are never cached
    (Observation 1);
 6. degrade rule (S_q): if the fraction of blocks of the head that still need computation is below S_q, every
    block of the head is cached;
 7. block-sparse skipping (tau_kv): in every row i of P~ the blocks are taken in ascending order of P~[i, j]
    and block j is skipped iff CumSum_up(P~[i, :])_j <= tau_kv (rows of P~ sum to one) -- the rule of
    Equation 1 applied to a row of the map: blocks are marked in ascending order of importance for as long as
    their accumulated importance stays within the threshold.

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


def _pool(X, size):
    """Mean over consecutive groups of `size` tokens (axis 2); the last group may be short."""
    L = X.shape[2]
    T = -(-L // size)
    return np.stack([X[:, :, t * size:(t + 1) * size].mean(axis=2) for t in range(T)], axis=2)


def compressed_map(Q, K, block, block_k=None, granularity=1):
    """Steps 1-2.  Q, K: uint16 bf16 bits [B,H,L,D].  Returns P~ as fp64 [B,H,T_q,T_k]."""
    Qf, Kf = _widen(Q), _widen(K)
    D = Qf.shape[-1]
    block_k = block if block_k is None else block_k
    qt, kt = _pool(Qf, granularity * block), _pool(Kf, granularity * block_k)
    S = np.einsum("bhid,bhjd->bhij", qt, kt) / np.sqrt(D)
    return _softmax(S, axis=-1)


def caching_metrics(P, n_t, n_tk=None):
    """Steps 3-4 for one head.  P: [T_q, T_k]; n_t text rows, n_tk text columns (default: the same number).
    Returns (C over the vision key blocks, G over the vision query blocks)."""
    n_tk = n_t if n_tk is None else n_tk
    C = P[:n_t, n_tk:].sum(axis=0)
    beta = _softmax(P[n_t:, :n_tk].T, axis=-1)
    G = beta.sum(axis=0)
    return C, G


def contribution_on_query_axis(C_key, L, pool_q, pool_k, n_tq, n_tk):
    """Step 5, first half: the contribution of the vision key blocks carried over to the vision query blocks by
    token overlap, C_v = sum_u C_u * |v and u| / |u|."""
    Tq = -(-L // pool_q)
    out = np.zeros(Tq - n_tq)
    for u, c in enumerate(C_key):
        k0, k1 = (n_tk + u) * pool_k, min((n_tk + u + 1) * pool_k, L)
        for v in range(Tq - n_tq):
            q0, q1 = (n_tq + v) * pool_q, min((n_tq + v + 1) * pool_q, L)
            common = min(k1, q1) - max(k0, q0)
            if common > 0:
                out[v] += c * common / (k1 - k0)
    return out


def cached_set(C, G, tau_c, tie_rel=1e-5):
    """Equation 1 on the two metrics of the vision blocks of one head.  Returns a dict with
      cached  bool   the block is selected for caching
      margin  fp64   how far the decision is from flipping, in units of the metric's total: for a selected block the
                     smaller of its two slacks (tau_c - CumSum_up / total), for the others the larger of the two
                     overshoots (both conditions must hold, so that is what has to be undone)
      tie     bool   the block's value of C or of G is within tie_rel (relative) of its neighbour in the ascending
                     order: the order, and with it the block's cumulative sums, is then not reliable
      window  fp64   the block's own share of the totals (the larger of the two): what swapping it with an
                     equal neighbour moves a cumulative sum by
    """
    C, G = np.asarray(C, dtype=np.float64), np.asarray(G, dtype=np.float64)
    csC, gapC = _cumsum_up(C)
    csG, gapG = _cumsum_up(G)
    # the totals are the last entries of the ascending sums, so that tau_c = 1 selects every block
    # whatever the rounding order
    totC, totG = csC.max(), csG.max()
    dC = (tau_c * totC - csC) / totC
    dG = (tau_c * totG - csG) / totG
    cached = (dC >= 0) & (dG >= 0)
    margin = np.where(cached, np.minimum(dC, dG), np.maximum(np.where(dC < 0, -dC, 0.0), np.where(dG < 0, -dG, 0.0)))
    return dict(cached=cached, margin=margin, tie=(gapC < tie_rel) | (gapG < tie_rel),
                window=np.maximum(C / totC, G / totG))


def skipped_set(p, tau_kv, tie_rel=1e-5):
    """Step 7 on one row of the compressed map.  Returns a dict with
      keep    uint8  1 = the pair is computed (its ascending cumulative sum exceeds tau_kv)
      margin  fp64   tau_kv - CumSum_up (positive = skipped): the distance of the decision from its threshold
      tie     bool   the entry is within tie_rel (relative) of its neighbour in the ascending order
    """
    p = np.asarray(p, dtype=np.float64)
    cs, gap = _cumsum_up(p)
    return dict(keep=(cs > tau_kv).astype(np.uint8), margin=tau_kv - cs, tie=gap < tie_rel)


def update_symbols(Q, K, block, text_tokens, tau_c, tau_kv, s_q=0.0, tie_rel=1e-5, block_k=None, granularity=1):
    """Steps 1-7 on whole tensors.  `block` is b_q; `block_k` defaults to it; `granularity` is n.

    Returns a dict with (T_q, T_k pooled blocks, see the module text)
      cache_flags  uint8 [B,H,T_q]      1 = block is cached (the ABI's polarity: M_c = 1 - cache_flags)
      M_s          uint8 [B,H,T_q,T_k]  1 = compute the pair
      flag_margin  fp64  [B,H,T_q]      `margin` of cached_set; +inf for text blocks and for heads decided by the
                                        degrade rule
      flag_tie     bool  [B,H,T_q]      `tie` of cached_set
      flag_window  fp64  [B,H,T_q]      `window` of cached_set
      skip_margin  fp64  [B,H,T_q,T_k]  `margin` of skipped_set
      skip_tie     bool  [B,H,T_q,T_k]  `tie` of skipped_set
      own_value    fp64  [B,H,T_q,T_k]  P~ itself (how far a near-tie can move a cumulative sum)
    """
    B, H, L, D = np.asarray(Q).shape
    block_k = block if block_k is None else block_k
    pool_q, pool_k = granularity * block, granularity * block_k
    Tq, Tk = -(-L // pool_q), -(-L // pool_k)
    n_tq, n_tk = -(-text_tokens // pool_q), -(-text_tokens // pool_k)
    if not (0 < text_tokens < L) or n_tq >= Tq or n_tk >= Tk:
        raise ValueError("text and vision blocks must both exist on the query and on the key axis")
    P = compressed_map(Q, K, block, block_k, granularity)
    flags = np.zeros((B, H, Tq), dtype=np.uint8)
    flag_margin = np.full((B, H, Tq), np.inf)
    flag_tie = np.zeros((B, H, Tq), dtype=bool)
    flag_window = np.zeros((B, H, Tq))
    M_s = np.ones((B, H, Tq, Tk), dtype=np.uint8)
    skip_margin = np.zeros((B, H, Tq, Tk))
    skip_tie = np.zeros((B, H, Tq, Tk), dtype=bool)
    for b in range(B):
        for h in range(H):
            C_key, G = caching_metrics(P[b, h], n_tq, n_tk)
            C = C_key if pool_q == pool_k else contribution_on_query_axis(C_key, L, pool_q, pool_k, n_tq, n_tk)
            sel = cached_set(C, G, tau_c, tie_rel)
            flags[b, h, n_tq:] = sel["cached"]
            flag_margin[b, h, n_tq:] = sel["margin"]
            flag_tie[b, h, n_tq:] = sel["tie"]
            flag_window[b, h, n_tq:] = sel["window"]
            if (Tq - int(sel["cached"].sum())) / Tq < s_q:
                flags[b, h, :] = 1
                flag_margin[b, h, :] = np.inf
                flag_tie[b, h, :] = False
            for i in range(Tq):
                row = skipped_set(P[b, h, i], tau_kv, tie_rel)
                skip_margin[b, h, i] = row["margin"]
                skip_tie[b, h, i] = row["tie"]
                M_s[b, h, i] = row["keep"]
    return dict(cache_flags=flags, M_s=M_s, flag_margin=flag_margin, flag_tie=flag_tie, flag_window=flag_window,
                skip_margin=skip_margin, skip_tie=skip_tie, own_value=P)
