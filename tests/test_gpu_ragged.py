"""GPU parity for sequence lengths that are not a multiple of the blocks (Definition 1: ceil(L / b) blocks, the
last query block and the last key block are short)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2509_25401_amd as pkg
from paper_2509_25401_amd import synth
from gpu_utils import DeviceCase, dev, up_bf16, up_u8, down_bits, oracle_full, check_against_oracle

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("D,bq,bk,L", [
    (128, 128, 128, 1000),     # last block: 104 rows; its second 64-key sub-tile holds 40 keys
    (128, 128, 128, 1060),     # last block: 36 rows; its second sub-tile does not exist
    (128, 128, 64, 513),       # one row / one key in the last block
    (128, 64, 128, 1100),
    (64, 64, 128, 777),
    (64, 128, 64, 650),
    (64, 64, 64, 200),
    (128, 128, 128, 90),       # a single short block
])
def test_short_last_blocks_match_oracle(D, bq, bk, L):
    print(f"[case] ragged D={D} {bq}x{bk} L={L}", flush=True)
    w = synth.random_case(synth.BASE_SEED + 200 + L, 2, 3, L, D, bq, bk, keep=0.5, cached_frac=0.3)
    w.M_s[..., -1] = 1                                   # the short key block is visited by every row
    case = DeviceCase(w)
    got = case.run()
    ref, ref_bits = oracle_full(w)
    check_against_oracle(w, got, ref, ref_bits, f"ragged D{D} {bq}x{bk} L{L}")
    # dense (no symbols at all) on the same tensors
    got = case.run(mask=None, flags=None, O_cache=None)
    ref, ref_bits = oracle.sparse_attention(w.Q, w.K, w.V, None, None, None, bq, bk)
    w.cache_flags = None
    check_against_oracle(w, got, ref, ref_bits, f"ragged dense D{D} {bq}x{bk} L{L}")


@pytest.mark.parametrize("D,blk,L", [(64, 64, 1), (64, 64, 7), (64, 64, 65), (128, 128, 1), (128, 128, 31), (128, 128, 129)])
def test_one_head_of_a_handful_of_tokens(D, blk, L):
    """One or two work items in all: seven of the eight work queues are empty from the start, the single token of
    L = 1 attends to itself (O = V)."""
    print(f"[case] tiny D={D} {blk}x{blk} L={L}", flush=True)
    w = synth.random_case(synth.BASE_SEED + 300 + L, 1, 1, L, D, blk, blk, keep=1.0, cached_frac=0.0)
    got = DeviceCase(w).run()
    ref, ref_bits = oracle_full(w)
    check_against_oracle(w, got, ref, ref_bits, f"tiny D{D} L{L}")
    if L == 1:
        assert (got == w.V).all()


def test_nothing_past_the_end_is_read_or_written():
    """One head whose tensors sit at the start of larger buffers: NaN behind Q, K, V and the cache, a marker
    behind O.  A read past the end would put NaN into the result (0 * NaN), a write would change the marker."""
    D, bq, bk, L, pad = 128, 128, 128, 300, 256
    w = synth.random_case(synth.BASE_SEED + 260, 1, 1, L, D, bq, bk, keep=1.0, cached_frac=0.0, with_cache_tensor=True)
    w.cache_flags = np.array([[[0, 0, 1]]], dtype=np.uint8)            # the short block is a cached one too, in a second run
    nan_bits = np.uint16(0x7FC0)

    def padded(bits, fill):
        buf = np.full((L + pad, D), fill, dtype=np.uint16)
        buf[:L] = bits[0, 0]
        t = up_bf16(buf)
        return t, t[:L].view(1, 1, L, D)

    (bQ, Q), (bK, K), (bV, V), (bC, Oc) = (padded(x, nan_bits) for x in (w.Q, w.K, w.V, w.O_cache))
    bO, O = padded(np.zeros_like(w.Q), np.uint16(0x4242))
    for flags in (None, w.cache_flags):
        bO[:L].zero_()
        pkg.sparse_attn_fwd(Q, K, V, up_u8(flags), None, Oc, O, bq, bk)
        torch.cuda.synchronize()
        whole = down_bits(bO)
        assert (whole[L:] == 0x4242).all(), "rows past the end of O were written"
        got = whole[:L][None, None]
        assert np.isfinite(synth.bf16_bits_to_f32(got)).all(), "something past the end of an input was read"
        ref, ref_bits = oracle.sparse_attention(w.Q, w.K, w.V, flags, None, w.O_cache, bq, bk)
        w2 = synth.random_case(1, 1, 1, L, D, bq, bk)                 # only for its shape fields
        w2.cache_flags = flags
        check_against_oracle(w2, got, ref, ref_bits, f"padded buffers, flags {'set' if flags is not None else 'none'}")


def test_plan_and_forecast_on_a_short_sequence():
    D, bq, bk, L = 128, 128, 128, 700
    w = synth.random_case(synth.BASE_SEED + 270, 1, 2, L, D, bq, bk, keep=0.6, cached_frac=0.4)
    case = DeviceCase(w)
    want = case.run()
    plan = pkg.SparseAttnPlan(case.flags, case.mask, w.B, w.H, L, bq, bk)
    O = torch.zeros_like(case.Q)
    plan.run(case.Q, case.K, case.V, case.Oc, O)
    torch.cuda.synchronize()
    assert (down_bits(O) == want).all()
    plan.destroy()
    rng = np.random.default_rng(5)
    terms = [w.O_cache, synth.normal_bf16(rng, w.Q.shape)]
    coef = pkg.sparse_taylor_coefficients(1, 2.0)
    O.zero_()
    pkg.sparse_attn_fwd_forecast(case.Q, case.K, case.V, case.flags, case.mask, [up_bf16(t) for t in terms], coef, O, bq, bk)
    torch.cuda.synchronize()
    ref, ref_bits = oracle.attention_with_forecast(w.Q, w.K, w.V, w.cache_flags, oracle.pack_symbols(w.M_s), terms, coef, bq, bk)
    rows = np.repeat(w.cache_flags != 0, bq, axis=2)[:, :, :L]
    got = down_bits(O)
    assert (got[rows] == ref_bits[rows]).mean() > 0.999
    err = np.abs(synth.bf16_bits_to_f32(got[~rows]).astype(np.float64) - ref[~rows])
    assert err.max() <= 1e-2 and err.mean() <= 1e-3
