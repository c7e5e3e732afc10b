"""GPU tests of the reusable plan (sparse_attn_plan_*): the stored pre-pass must drive the same kernel to the same
bits as the one-shot call, run after run, and symbols at granularity n must decode as Section 3.4 defines."""
import numpy as np
import pytest
import torch

import oracle
import paper_2509_25401_amd as pkg
from paper_2509_25401_amd import synth
from gpu_utils import DeviceCase, dev, up_bf16, up_u8, down_bits, oracle_full, check_against_oracle

pytestmark = pytest.mark.gpu


def fresh_O(w, fill=0x4242):
    return torch.from_numpy(np.full(w.Q.shape, fill, dtype=np.uint16).view(np.int16)).view(torch.bfloat16).to(dev())


@pytest.mark.parametrize("D,bq,bk", [(128, 128, 128), (64, 64, 128), (128, 128, 64)])
def test_plan_reproduces_the_one_shot_call_bit_for_bit(D, bq, bk):
    w = synth.random_case(synth.BASE_SEED + 90 + D + bq, 2, 3, 1024, D, bq, bk, keep=0.4, cached_frac=0.3)
    case = DeviceCase(w)
    want = case.run()
    flags, mask = case.flags.clone(), case.mask.clone()
    plan = pkg.SparseAttnPlan(flags, mask, w.B, w.H, w.L, bq, bk)
    torch.cuda.synchronize()
    flags.fill_(1)                        # the plan holds its own decoded copy: the symbol arrays may change
    mask.zero_()
    for rep in range(3):                  # the queue counters are reset for every run
        O = fresh_O(w)
        plan.run(case.Q, case.K, case.V, case.Oc, O)
        torch.cuda.synchronize()
        assert (down_bits(O) == want).all(), f"run {rep} differs from the one-shot call"
    ref, ref_bits = oracle_full(w)
    check_against_oracle(w, want, ref, ref_bits, f"plan D{D} {bq}x{bk}")
    plan.destroy()


@pytest.mark.parametrize("D,bq,bk,n_terms", [(128, 128, 128, 2), (64, 64, 64, 3)])
def test_plan_with_forecast_reproduces_the_one_shot_forecast(D, bq, bk, n_terms):
    """Stored plan + Taylor forecast in the cache branch: the same bits as sparse_attn_fwd_forecast (whose parity
    with the oracle is checked where that entry point is tested), run after run."""
    w = synth.random_case(synth.BASE_SEED + 95 + n_terms, 1, 4, 1152, D, bq, bk, keep=0.5, cached_frac=0.4)
    rng = np.random.default_rng(synth.BASE_SEED + 96 + n_terms)
    terms = [up_bf16(w.O_cache)] + [up_bf16(synth.normal_bf16(rng, w.Q.shape)) for _ in range(n_terms - 1)]
    coef = pkg.sparse_taylor_coefficients(n_terms - 1, 3.0)
    case = DeviceCase(w)
    want = fresh_O(w)
    pkg.sparse_attn_fwd_forecast(case.Q, case.K, case.V, case.flags, case.mask, terms, coef, want, bq, bk)
    plan = pkg.SparseAttnPlan(case.flags, case.mask, w.B, w.H, w.L, bq, bk)
    torch.cuda.synchronize()
    rows = np.repeat(w.cache_flags != 0, bq, axis=2)
    assert rows.any() and (~rows).any()
    for rep in range(2):
        O = fresh_O(w)
        plan.run_forecast(case.Q, case.K, case.V, terms, coef, O)
        torch.cuda.synchronize()
        assert (down_bits(O) == down_bits(want)).all(), f"run {rep} differs from the one-shot forecast"
    # and it is not the plain copy: the forecast moved the cached blocks away from term 0
    assert (down_bits(want)[rows] != w.O_cache[rows]).any()
    plan.destroy()


@pytest.mark.parametrize("n,L", [(2, 1024), (3, 896), (4, 2048)])
def test_granularity_decodes_like_the_expanded_symbols(n, L):
    B, H, D, blk = 1, 2, 128, 128
    T = L // blk
    sT = -(-T // n)
    rng = np.random.default_rng(synth.BASE_SEED + 95 + n)
    w = synth.random_case(synth.BASE_SEED + 96 + n, B, H, L, D, blk, blk, keep=1.0, cached_frac=0.0, with_cache_tensor=True)
    coarse_flags = (rng.random((B, H, sT)) < 0.3).astype(np.uint8)
    coarse_M = (rng.random((B, H, sT, sT)) < 0.5).astype(np.uint8)
    coarse_M[..., 0] = 1                                           # every row keeps something
    f, m = oracle.expand_granularity(coarse_flags, coarse_M, n, T, T)
    ref, ref_bits = oracle.sparse_attention(w.Q, w.K, w.V, f, oracle.pack_symbols(m), w.O_cache, blk, blk)
    Q, K, V, Oc = up_bf16(w.Q), up_bf16(w.K), up_bf16(w.V), up_bf16(w.O_cache)
    plan = pkg.SparseAttnPlan(up_u8(coarse_flags), up_u8(pkg.sparse_attn_pack_mask(coarse_M)), B, H, L, blk, blk, granularity=n)
    O = fresh_O(w)
    plan.run(Q, K, V, Oc, O)
    torch.cuda.synchronize()
    got = down_bits(O)
    w.cache_flags, w.M_s = f, m
    check_against_oracle(w, got, ref, ref_bits, f"granularity {n}")
    # the same tiles through the one-shot call with symbols expanded to granularity 1: identical bits
    O1 = fresh_O(w)
    pkg.sparse_attn_fwd(Q, K, V, up_u8(f), up_u8(pkg.sparse_attn_pack_mask(m)), Oc, O1, blk, blk)
    torch.cuda.synchronize()
    assert (down_bits(O1) == got).all()
    plan.destroy()


def test_plan_without_symbols_is_dense_attention_and_skips_the_prepass_time():
    w = synth.random_case(synth.BASE_SEED + 99, 1, 4, 4608, 128, 128, 128, keep=1.0)
    case = DeviceCase(w)
    plan = pkg.SparseAttnPlan(None, None, w.B, w.H, w.L, 128, 128)
    O = fresh_O(w)
    plan.run(case.Q, case.K, case.V, None, O)
    torch.cuda.synchronize()
    O1 = fresh_O(w)
    pkg.sparse_attn_fwd(case.Q, case.K, case.V, None, None, None, O1, 128, 128)
    torch.cuda.synchronize()
    assert (down_bits(O) == down_bits(O1)).all()
    # timing, for the log only: stored plan vs pre-pass on every call
    def timed(fn, reps=20):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps
    t_plan = timed(lambda: plan.run(case.Q, case.K, case.V, None, O))
    t_shot = timed(lambda: pkg.sparse_attn_fwd(case.Q, case.K, case.V, None, None, None, O1, 128, 128))
    print(f"[plan] 4608 tokens x 4 heads dense: stored plan {t_plan * 1e3:.1f} us/call, one-shot {t_shot * 1e3:.1f} us/call", flush=True)
    plan.destroy()


def test_caller_supplied_workspace_and_scratch_release():
    """sparse_attn_fwd_workspace writes the bits of the one-shot call using only the caller's buffer (a buffer one
    byte short is refused); releasing the library's scratch of the stream leaves the next one-shot call working."""
    w = synth.random_case(synth.BASE_SEED + 97, 2, 3, 1100, 128, 128, 64, keep=0.5, cached_frac=0.3)
    case = DeviceCase(w)
    want = case.run()
    need = pkg.sparse_attn_workspace_bytes(w.B, w.H, w.L, w.block_q, w.block_k)
    ws = torch.full((need + 512,), 0xAB, dtype=torch.uint8, device=dev())
    base = (-ws.data_ptr()) % 256
    O = fresh_O(w)
    pkg.sparse_attn_fwd_workspace(case.Q, case.K, case.V, case.flags, case.mask, case.Oc, O, w.block_q, w.block_k,
                                  ws[base:base + need])
    torch.cuda.synchronize()
    assert (down_bits(O) == want).all()
    assert (ws[base + need:] == 0xAB).all() and (ws[:base] == 0xAB).all(), "wrote outside the workspace"
    with pytest.raises(pkg.SparseAttnError):
        pkg.sparse_attn_fwd_workspace(case.Q, case.K, case.V, case.flags, case.mask, case.Oc, O, w.block_q, w.block_k,
                                      ws[base:base + need - 1])
    pkg.sparse_attn_release_scratch()
    pkg.sparse_attn_release_scratch()          # nothing left to free: still fine
    assert (case.run() == want).all()
