"""Pins of the symbol-generation oracle (Section 3.3, Equation 1, settings table of the appendix)."""
import numpy as np
import pytest

import oracle
from paper_2509_25401_amd import synth
from helpers import bits_to_f64


def test_brute_force_loops_on_a_tiny_case():
    B, H, L, D, blk, text = 1, 2, 12, 4, 2, 4          # T = 6 blocks, 2 of them text
    Q, K = synth.structured_qk(1, B, H, L, D, blk)
    tau_c, tau_kv = 0.45, 0.3
    out = oracle.update_symbols(Q, K, blk, text, tau_c, tau_kv)
    Qf, Kf = bits_to_f64(Q), bits_to_f64(K)
    T, nt = L // blk, text // blk
    for h in range(H):
        qt = [[sum(Qf[0, h, i * blk + r, d] for r in range(blk)) / blk for d in range(D)] for i in range(T)]
        kt = [[sum(Kf[0, h, i * blk + r, d] for r in range(blk)) / blk for d in range(D)] for i in range(T)]
        P = []
        for i in range(T):
            s = [sum(qt[i][d] * kt[j][d] for d in range(D)) / np.sqrt(D) for j in range(T)]
            m = max(s)
            e = [np.exp(x - m) for x in s]
            P.append([x / sum(e) for x in e])
        C = [sum(P[j][nt + v] for j in range(nt)) for v in range(T - nt)]
        beta = []
        for j in range(nt):
            col = [P[nt + v][j] for v in range(T - nt)]
            m = max(col)
            e = [np.exp(x - m) for x in col]
            beta.append([x / sum(e) for x in e])
        G = [sum(beta[j][v] for j in range(nt)) for v in range(T - nt)]

        def cum_up(x):
            order = sorted(range(len(x)), key=lambda t: (x[t], t))
            cs, run = [0.0] * len(x), 0.0
            for t in order:
                run += x[t]
                cs[t] = run
            return cs
        cC, cG = cum_up(C), cum_up(G)
        for v in range(T - nt):
            want = int(cC[v] <= tau_c * sum(C) and cG[v] <= tau_c * sum(G))
            assert out["cache_flags"][0, h, nt + v] == want
        assert (out["cache_flags"][0, h, :nt] == 0).all()
        for i in range(T):
            cs = cum_up(P[i])
            for j in range(T):
                assert out["M_s"][0, h, i, j] == int(cs[j] > tau_kv)
        assert np.abs(out["own_value"][0, h] - np.array(P)).max() < 1e-14


def test_uniform_map_closed_form():
    """Q = 0: P~ = 1/T everywhere, all metrics tie, ties go by index: the first floor(tau * count) entries are taken."""
    B, H, L, D, blk, text = 1, 1, 160, 8, 8, 32       # T = 20, n_t = 4, 16 vision blocks
    Q = np.zeros((B, H, L, D), dtype=np.uint16)
    _, K = synth.structured_qk(2, B, H, L, D, blk)
    out = oracle.update_symbols(Q, K, blk, text, 0.33, 0.27)
    flags = out["cache_flags"][0, 0]
    assert flags[:4].sum() == 0 and flags[4:].tolist() == [1] * 5 + [0] * 11      # floor(0.33 * 16) = 5
    for i in range(20):
        assert out["M_s"][0, 0, i].tolist() == [0] * 5 + [1] * 15                   # floor(0.27 * 20) = 5 skipped


def test_thresholds_zero_and_one_and_monotonicity():
    B, H, L, D, blk, text = 1, 2, 256, 16, 16, 32
    Q, K = synth.structured_qk(3, B, H, L, D, blk)
    nt = text // blk
    lo = oracle.update_symbols(Q, K, blk, text, 0.0, 0.0)
    assert lo["cache_flags"].sum() == 0 and (lo["M_s"] == 1).all()
    hi = oracle.update_symbols(Q, K, blk, text, 1.0, 0.5)
    assert (hi["cache_flags"][..., nt:] == 1).all() and (hi["cache_flags"][..., :nt] == 0).all()
    prev_f, prev_m = lo["cache_flags"], lo["M_s"]
    for tau in (0.2, 0.4, 0.6, 0.8):
        cur = oracle.update_symbols(Q, K, blk, text, tau, tau)
        assert (cur["cache_flags"] >= prev_f).all()          # cached set grows with tau_c
        assert (cur["M_s"] <= prev_m).all()                  # kept set shrinks with tau_kv
        kept_mass = (cur["own_value"] * cur["M_s"]).sum(axis=-1)
        assert (kept_mass >= 1 - tau - 1e-12).all()          # skipped importance never exceeds tau_kv
        assert (cur["M_s"].sum(axis=-1) >= 1).all()          # the largest entry of a row is always kept
        prev_f, prev_m = cur["cache_flags"], cur["M_s"]


def test_metrics_follow_their_definitions_on_a_hand_made_map():
    P = np.array([[0.7, 0.1, 0.1, 0.1],      # text row
                  [0.2, 0.5, 0.2, 0.1],
                  [0.6, 0.2, 0.1, 0.1],
                  [0.1, 0.1, 0.1, 0.7]])
    C, G = oracle.caching_metrics(P, 1)
    assert np.allclose(C, [0.1, 0.1, 0.1])                                    # text row's weights on the three vision blocks
    e = np.exp(np.array([0.2, 0.6, 0.1]))
    assert np.allclose(G, e / e.sum())                                        # softmax over vision blocks of their weight on text
    assert np.argmax(G) == 1                                                  # the block that listens to text most is guided most


def test_degrade_rule_and_block_permutation():
    B, H, L, D, blk, text = 1, 1, 256, 16, 16, 32
    Q, K = synth.structured_qk(4, B, H, L, D, blk)
    T, nt = L // blk, text // blk
    base = oracle.update_symbols(Q, K, blk, text, 0.7, 0.2)
    need = (T - base["cache_flags"].sum()) / T
    assert 0 < need < 1
    off = oracle.update_symbols(Q, K, blk, text, 0.7, 0.2, s_q=need - 1e-6)
    on = oracle.update_symbols(Q, K, blk, text, 0.7, 0.2, s_q=need + 1e-6)
    assert (off["cache_flags"] == base["cache_flags"]).all() and (on["cache_flags"] == 1).all()
    # permuting vision blocks (queries and keys together) permutes the symbols
    perm = np.concatenate([np.arange(nt), nt + np.random.default_rng(5).permutation(T - nt)])
    def blocks(x):
        return np.ascontiguousarray(x.reshape(B, H, T, blk, D)[:, :, perm].reshape(x.shape))
    p = oracle.update_symbols(blocks(Q), blocks(K), blk, text, 0.7, 0.2)
    robust = ~base["flag_tie"][0, 0] & (base["flag_margin"][0, 0] > 1e-9)
    assert (p["cache_flags"][0, 0][robust[perm]] == base["cache_flags"][0, 0][perm][robust[perm]]).all()
    assert (p["M_s"][0, 0] == base["M_s"][0, 0][perm][:, perm]).mean() > 0.999


def test_short_last_block_is_pooled_over_the_tokens_that_exist():
    B, H, L, D, blk, text = 1, 1, 14, 4, 4, 4           # 4 blocks, the last one holds 2 tokens
    Q, K = synth.structured_qk(6, B, H, 16, D, blk)
    Q, K = np.ascontiguousarray(Q[:, :, :L]), np.ascontiguousarray(K[:, :, :L])
    P = oracle.compressed_map(Q, K, blk)
    assert P.shape == (1, 1, 4, 4)
    Qf, Kf = bits_to_f64(Q)[0, 0], bits_to_f64(K)[0, 0]
    qt = [Qf[0:4].mean(0), Qf[4:8].mean(0), Qf[8:12].mean(0), (Qf[12] + Qf[13]) / 2]
    kt = [Kf[0:4].mean(0), Kf[4:8].mean(0), Kf[8:12].mean(0), (Kf[12] + Kf[13]) / 2]
    S = np.array([[qi @ kj / 2.0 for kj in kt] for qi in qt])          # sqrt(D) = 2
    E = np.exp(S - S.max(axis=1, keepdims=True))
    assert np.abs(P[0, 0] - E / E.sum(axis=1, keepdims=True)).max() < 1e-14
    out = oracle.update_symbols(Q, K, blk, text, 0.5, 0.2)
    assert out["cache_flags"].shape == (1, 1, 4) and out["M_s"].shape == (1, 1, 4, 4)


# --- the diagnostics that decide which decisions a GPU run is compared on -------------------------------------
def test_cached_set_margins_windows_and_ties_on_hand_made_metrics():
    """C ascending, G descending, both summing to one: the ascending sums and every margin can be read off."""
    C, G = [0.1, 0.2, 0.3, 0.4], [0.4, 0.3, 0.2, 0.1]
    # CumSum_up(C) = [0.1, 0.3, 0.6, 1.0]; CumSum_up(G) = [1.0, 0.6, 0.3, 0.1]
    lo = oracle.cached_set(C, G, 0.35)
    assert lo["cached"].tolist() == [False] * 4                      # no block satisfies both conditions
    assert np.allclose(lo["margin"], [0.65, 0.25, 0.25, 0.65])       # the larger overshoot has to be undone
    hi = oracle.cached_set(C, G, 0.65)
    assert hi["cached"].tolist() == [False, True, True, False]
    assert np.allclose(hi["margin"], [0.35, 0.05, 0.05, 0.35])       # cached: the smaller slack; others: the overshoot
    assert np.allclose(hi["window"], [0.4, 0.3, 0.3, 0.4])           # the block's own share, exactly (not a bound)
    assert not hi["tie"].any()
    # totals other than one: margins and windows are relative to the totals
    sc = oracle.cached_set(3.0 * np.array(C), 5.0 * np.array(G), 0.65)
    assert np.allclose(sc["margin"], hi["margin"]) and np.allclose(sc["window"], hi["window"])
    # a near-tie marks exactly the two neighbours in the order, in whichever metric it occurs
    t = oracle.cached_set([0.1, 0.2, 0.2 * (1 + 1e-7), 0.5], [0.4, 0.3, 0.2, 0.1], 0.5, tie_rel=1e-5)
    assert t["tie"].tolist() == [False, True, True, False]
    t = oracle.cached_set([0.1, 0.2, 0.3, 0.4], [0.3, 0.3 * (1 - 1e-7), 0.2, 0.2], 0.5, tie_rel=1e-5)
    assert t["tie"].tolist() == [True, True, True, True]             # 0.2 == 0.2 exactly, 0.3 ~ 0.3
    assert not oracle.cached_set([0.1, 0.2, 0.2 * (1 + 1e-3), 0.5], [0.4, 0.3, 0.2, 0.1], 0.5, tie_rel=1e-5)["tie"].any()


def test_skipped_set_margins_and_ties_on_a_hand_made_row():
    p = np.array([1, 6, 3, 2, 4]) / 16.0                              # ascending sums: 1, 16, 6, 3, 10 sixteenths (exact)
    r = oracle.skipped_set(p, 6 / 16.0)
    assert r["keep"].tolist() == [0, 1, 0, 0, 1]                      # a sum equal to tau_kv is still skipped
    assert (r["margin"] == np.array([5, -10, 0, 3, -4]) / 16.0).all()
    assert not r["tie"].any()
    r = oracle.skipped_set([0.1, 0.1 * (1 + 1e-8), 0.3, 0.5], 0.25, tie_rel=1e-5)
    assert r["tie"].tolist() == [True, True, False, False]


def _planted(ref):
    flags, bits = ref["cache_flags"].copy(), ref["M_s"].copy()
    return flags, bits


def test_comparator_accepts_only_undecidable_differences():
    """The rule that tells a real disagreement from a rounding-level one, exercised on planted mistakes (CPU only):
    flipping a decision the oracle is sure of must fail, flipping one inside the window must pass -- and only as long
    as such entries stay rare."""
    from helpers import compare_symbols, decidable_symbols
    B, H, L, D, blk, text = 1, 2, 1280, 16, 16, 64                   # 80 blocks, 4 text
    Q, K = synth.structured_qk(9, B, H, L, D, blk)
    # thresholds placed ON a cumulative sum (tau_kv = the sum at the median entry of row 0, to within 1e-9): the
    # decision there is undecidable by construction
    P = oracle.compressed_map(Q, K, blk)
    row = np.sort(P[0, 0, 5])
    tau_kv = float(np.cumsum(row)[40] + 1e-9)
    ref = oracle.update_symbols(Q, K, blk, text, 0.5, tau_kv)
    robust_f, robust_s = decidable_symbols(ref)
    assert robust_f.mean() > 0.9 and robust_s.mean() > 0.99 and not robust_s.all()
    flags, bits = _planted(ref)
    compare_symbols(ref, flags, bits, "identical", require_identical=True)
    # a decision inside the window may differ ...
    i, j = np.argwhere(~robust_s[0, 0])[0]
    bits[0, 0, i, j] ^= 1
    compare_symbols(ref, flags, bits, "one undecidable pair flipped")
    with pytest.raises(AssertionError, match="expected to be reproduced exactly"):
        compare_symbols(ref, flags, bits, "one undecidable pair flipped", require_identical=True)
    # ... a decision outside it may not, whichever way it is flipped
    for want in (0, 1):
        flags, bits = _planted(ref)
        i, j = np.argwhere(robust_s[0, 1] & (ref["M_s"][0, 1] == want))[0]
        bits[0, 1, i, j] ^= 1
        with pytest.raises(AssertionError, match="mask bits differ"):
            compare_symbols(ref, flags, bits, "robust pair flipped")
        flags, bits = _planted(ref)
        v = np.argwhere(robust_f[0, 0] & (ref["cache_flags"][0, 0] == want) & (np.arange(L // blk) >= 4))[0, 0]
        flags[0, 0, v] ^= 1
        with pytest.raises(AssertionError, match="cache flags differ"):
            compare_symbols(ref, flags, bits, "robust flag flipped")
    # and the excuse only holds while undecidable entries are rare
    wide = dict(ref, flag_margin=np.zeros_like(ref["flag_margin"]))
    with pytest.raises(AssertionError, match="too many undecidable"):
        compare_symbols(wide, ref["cache_flags"], ref["M_s"], "everything undecidable")


def test_a_widened_window_would_excuse_a_real_mistake_and_is_caught_by_the_pins():
    """Why flag_window is pinned to the block's own share: with a window a million times wider every tied block
    becomes undecidable and a planted mistake on a tied block goes through."""
    from helpers import decidable_symbols
    C = np.array([0.02, 0.03, 0.03 * (1 + 1e-8), 0.42, 0.5])          # blocks 1 and 2 tie; both far from tau_c = 0.7
    G = np.array([0.5, 0.03, 0.02, 0.05, 0.4])
    sel = oracle.cached_set(C, G, 0.7)
    ref = dict(flag_margin=sel["margin"][None, None], flag_tie=sel["tie"][None, None], flag_window=sel["window"][None, None],
               skip_margin=np.ones((1, 1, 5, 5)), skip_tie=np.zeros((1, 1, 5, 5), bool), own_value=np.zeros((1, 1, 5, 5)))
    robust_f, _ = decidable_symbols(ref)
    assert sel["tie"].tolist() == [False, True, True, False, False]
    assert robust_f[0, 0].tolist() == [True, True, True, True, True]  # tied blocks: margins 0.65 / 0.62 against 2 * own share = 0.06
    ref["flag_window"] = ref["flag_window"] * 1e6
    assert decidable_symbols(ref)[0][0, 0].tolist() == [True, False, False, True, True]


# --- granularity n and b_q != b_k ---------------------------------------------------------------------------------
def test_granularity_pools_n_blocks_and_counts_text_blocks_with_a_ceiling():
    B, H, L, D, bq = 1, 1, 50, 4, 4                                   # n = 3: pooled blocks of 12 tokens, the last holds 2
    Q, K = synth.structured_qk(12, B, H, 52, D, 4)
    Q, K = np.ascontiguousarray(Q[:, :, :L]), np.ascontiguousarray(K[:, :, :L])
    P = oracle.compressed_map(Q, K, bq, granularity=3)
    assert P.shape == (1, 1, 5, 5)
    Qf, Kf = bits_to_f64(Q)[0, 0], bits_to_f64(K)[0, 0]
    qt = [Qf[12 * t:12 * t + 12].mean(0) for t in range(5)]
    kt = [Kf[12 * t:12 * t + 12].mean(0) for t in range(5)]
    S = np.array([[qi @ kj / 2.0 for kj in kt] for qi in qt])
    E = np.exp(S - S.max(axis=1, keepdims=True))
    assert np.abs(P[0, 0] - E / E.sum(axis=1, keepdims=True)).max() < 1e-14
    # 13 text tokens: ceil(13 / 12) = 2 text blocks (a pooled block with any text token is text), never cached
    out = oracle.update_symbols(Q, K, bq, 13, 1.0, 0.2, granularity=3)
    assert out["cache_flags"].shape == (1, 1, 5) and out["M_s"].shape == (1, 1, 5, 5)
    assert out["cache_flags"][0, 0].tolist() == [0, 0, 1, 1, 1]
    # the symbols at granularity n are the symbols of the same tensors at block size n * b
    big = oracle.update_symbols(Q, K, 3 * bq, 13, 0.6, 0.2)
    fine = oracle.update_symbols(Q, K, bq, 13, 0.6, 0.2, granularity=3)
    assert (big["cache_flags"] == fine["cache_flags"]).all() and (big["M_s"] == fine["M_s"]).all()


def test_unequal_blocks_carry_the_contribution_over_by_token_overlap():
    # b_k = 2 b_q: one vision key block covers two vision query blocks, each gets half of its contribution
    C_key = np.array([0.3, 0.1])
    got = oracle.contribution_on_query_axis(C_key, L=48, pool_q=8, pool_k=16, n_tq=2, n_tk=1)   # text: 16 tokens
    assert np.allclose(got, [0.15, 0.15, 0.05, 0.05])
    # b_q = 2 b_k: a vision query block collects its two key blocks
    got = oracle.contribution_on_query_axis(np.array([0.1, 0.2, 0.3, 0.4]), L=48, pool_q=16, pool_k=8, n_tq=1, n_tk=2)
    assert np.allclose(got, [0.3, 0.7])
    # boundaries that do not line up, short last blocks: text = 10 tokens, pool_q = 8 (2 text blocks: tokens 0..15),
    # pool_k = 6 (2 text blocks: tokens 0..11); vision key blocks [12,18) [18,24) [24,26); vision query blocks [16,24) [24,26)
    got = oracle.contribution_on_query_axis(np.array([0.6, 0.3, 0.1]), L=26, pool_q=8, pool_k=6, n_tq=2, n_tk=2)
    assert np.allclose(got, [0.6 * 2 / 6 + 0.3, 0.1])
    # the map itself: rows pooled by b_q, columns by b_k
    B, H, L, D = 1, 1, 48, 4
    Q, K = synth.structured_qk(13, B, H, L, D, 8)
    out = oracle.update_symbols(Q, K, 8, 16, 0.5, 0.3, block_k=16)
    assert out["cache_flags"].shape == (1, 1, 6) and out["M_s"].shape == (1, 1, 6, 3)
    P = oracle.compressed_map(Q, K, 8, 16)
    C_key, G = oracle.caching_metrics(P[0, 0], 2, 1)
    C = oracle.contribution_on_query_axis(C_key, L, 8, 16, 2, 1)
    assert (out["cache_flags"][0, 0, 2:] == oracle.cached_set(C, G, 0.5)["cached"]).all()
    assert (out["cache_flags"][0, 0, :2] == 0).all()
    for i in range(6):
        assert (out["M_s"][0, 0, i] == oracle.skipped_set(P[0, 0, i], 0.3)["keep"]).all()
