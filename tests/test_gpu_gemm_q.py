"""GPU parity of the sparse query projection (GEMM-Q) against its CPU oracle.

Bar: skipped blocks bit-identical to what was in Q before the call; computed elements within one
bf16 rounding of the fp64 result: |got - ref| <= 2^-8 |ref| + 1e-3 (fp32 accumulation of C <= 3072
products of O(1) terms contributes < 1e-4)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2509_25401_amd as pkg
from paper_2509_25401_amd import synth
from gpu_utils import up_bf16, up_u8, down_bits

pytestmark = pytest.mark.gpu


def _case(seed, B, L, C, H, D, bq, cached, bias=True):
    r = np.random.default_rng(seed)
    X = synth.normal_bf16(r, (B, L, C))
    W = synth.f32_to_bf16_bits((r.standard_normal((H * D, C)) / np.sqrt(C)).astype(np.float32))
    b = synth.normal_bf16(r, (H * D,)) if bias else None
    flags = (r.random((B, H, L // bq)) < cached).astype(np.uint8) if cached > 0 else None
    return X, W, b, flags


def _run(X, W, b, flags, B, L, C, H, D, bq, fill=0x4242):
    Q = torch.from_numpy(np.full((B, H, L, D), fill, dtype=np.uint16).view(np.int16)).view(torch.bfloat16).to("cuda:0")
    pkg.sparse_gemm_q(up_bf16(X), up_bf16(W), None if b is None else up_bf16(b), up_u8(flags), Q, bq)
    torch.cuda.synchronize()
    return down_bits(Q)


def _check(got_bits, ref, ref_bits, flags, bq, label):
    skipped = np.zeros(got_bits.shape[:3], dtype=bool) if flags is None else np.repeat(flags != 0, bq, axis=2)
    if skipped.any():
        assert (got_bits[skipped] == 0x4242).all(), f"{label}: skipped blocks were written"
    got = synth.bf16_bits_to_f32(got_bits).astype(np.float64)[~skipped]
    want = ref[~skipped]
    err = np.abs(got - want)
    tol = np.abs(want) * 2.0 ** -8 + 1e-3
    exact = (got_bits[~skipped] == ref_bits[~skipped]).mean()
    print(f"[parity] {label}: max-abs {err.max():.3e}, bit-identical to the rounded oracle: {exact * 100:.2f}%", flush=True)
    assert (err <= tol).all(), f"{label}: max violation {(err - tol).max()}"
    assert exact > 0.98


@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("bq", [64, 128])
def test_small_cases_all_variants(D, bq):
    print(f"[case] gemm_q small D={D} bq={bq}", flush=True)
    B, L, C, H = 2, 384, 320, 3       # C = 5 stages of 64: odd number of stages
    X, W, b, flags = _case(10 + D + bq, B, L, C, H, D, bq, cached=0.3)
    got = _run(X, W, b, flags, B, L, C, H, D, bq)
    ref, ref_bits = oracle.gemm_q(X, W, b, flags, bq, H, D)
    _check(got, ref, ref_bits, flags, bq, f"gemm_q D={D} bq={bq}")


def test_single_stage_and_no_bias_no_flags():
    print("[case] gemm_q C=64", flush=True)
    B, L, C, H, D, bq = 1, 256, 64, 2, 128, 128
    X, W, _, _ = _case(20, B, L, C, H, D, bq, cached=0, bias=False)
    got = _run(X, W, None, None, B, L, C, H, D, bq)
    ref, ref_bits = oracle.gemm_q(X, W, None, None, bq, H, D)
    _check(got, ref, ref_bits, None, bq, "gemm_q C=64")


def test_one_hot_tokens_select_weight_entries_exactly():
    print("[case] gemm_q one-hot", flush=True)
    B, L, C, H, D, bq = 1, 256, 128, 2, 64, 64
    r = np.random.default_rng(21)
    W = synth.normal_bf16(r, (H * D, C))
    Xf = np.zeros((B, L, C), dtype=np.float32)
    Xf[0, np.arange(L), (np.arange(L) * 7) % C] = 1.0
    got = _run(synth.f32_to_bf16_bits(Xf), W, None, None, B, L, C, H, D, bq)
    expect = W.reshape(H, D, C).transpose(0, 2, 1)[None, :, (np.arange(L) * 7) % C, :]
    assert (got == expect).all()


def test_all_blocks_flagged_writes_nothing():
    B, L, C, H, D, bq = 1, 256, 128, 2, 128, 128
    X, W, b, _ = _case(22, B, L, C, H, D, bq, cached=0)
    got = _run(X, W, b, np.ones((B, H, L // bq), dtype=np.uint8), B, L, C, H, D, bq)
    assert (got == 0x4242).all()


def test_image_dit_shape_with_flags_feeds_attention():
    """FLUX-like projection (4608 tokens, 3072 channels, 24 heads of 128) with config 3's flags; the
    projected queries of the computed blocks then go through the attention kernel and its oracle."""
    print("[case] gemm_q image-DiT shape", flush=True)
    w = synth.config_image_cache_skip()
    B, L, C, H, D, bq = 1, w.L, 3072, w.H, w.D, w.block_q
    X, W, b, _ = _case(23, B, L, C, H, D, bq, cached=0)
    got = _run(X, W, b, w.cache_flags, B, L, C, H, D, bq)
    ref, ref_bits = oracle.gemm_q(X, W, b, w.cache_flags, bq, H, D)
    _check(got, ref, ref_bits, w.cache_flags, bq, "gemm_q image-DiT")


# ---- fused token-wise RMSNorm + RoPE epilogue (Equation 2) ----

def _rope_tables(L, D, base=10000.0):
    pos = np.arange(L, dtype=np.float64)[:, None]
    freq = base ** (-np.arange(D // 2, dtype=np.float64) / (D // 2))[None, :]
    ang = pos * freq
    return np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)


def _run_fused(X, W, b, g, eps, cos, sin, flags, B, L, C, H, D, bq, fill=0x4242):
    Q = torch.from_numpy(np.full((B, H, L, D), fill, dtype=np.uint16).view(np.int16)).view(torch.bfloat16).to("cuda:0")
    dcos = None if cos is None else torch.from_numpy(cos).to("cuda:0")
    dsin = None if sin is None else torch.from_numpy(sin).to("cuda:0")
    pkg.sparse_gemm_q_norm_rope(up_bf16(X), up_bf16(W), None if b is None else up_bf16(b), None if g is None else up_bf16(g),
                                eps, dcos, dsin, up_u8(flags), Q, bq)
    torch.cuda.synchronize()
    return down_bits(Q)


@pytest.mark.parametrize("D,bq", [(128, 128), (64, 128), (128, 64), (64, 64)])
def test_fused_norm_rope_small_cases(D, bq):
    print(f"[case] gemm_q norm+rope D={D} bq={bq}", flush=True)
    B, L, C, H = 2, 384, 320, 3
    X, W, b, flags = _case(40 + D + bq, B, L, C, H, D, bq, cached=0.3)
    g = synth.f32_to_bf16_bits((1.0 + 0.2 * np.random.default_rng(41).standard_normal(D)).astype(np.float32))
    cos, sin = _rope_tables(L, D)
    got = _run_fused(X, W, b, g, 1e-6, cos, sin, flags, B, L, C, H, D, bq)
    ref, ref_bits = oracle.gemm_q(X, W, b, flags, bq, H, D, norm_weight=g, eps=float(np.float32(1e-6)), rope_cos=cos, rope_sin=sin)
    _check(got, ref, ref_bits, flags, bq, f"gemm_q norm+rope D={D} bq={bq}")


def test_fused_variants_without_gain_or_rotation():
    B, L, C, H, D, bq = 1, 256, 128, 2, 128, 128
    X, W, b, flags = _case(50, B, L, C, H, D, bq, cached=0.0, bias=False)
    cos, sin = _rope_tables(L, D)
    # normalisation only
    got = _run_fused(X, W, None, None, 0.0, None, None, None, B, L, C, H, D, bq)
    ref, ref_bits = oracle.gemm_q(X, W, None, None, bq, H, D, eps=0.0)
    _check(got, ref, ref_bits, None, bq, "gemm_q norm only")
    ms = (synth.bf16_bits_to_f32(got).astype(np.float64) ** 2).mean(axis=-1)
    assert np.abs(ms - 1.0).max() < 2e-2                        # unit mean square up to bf16 rounding
    # rotation without gain
    got = _run_fused(X, W, None, None, 1e-5, cos, sin, None, B, L, C, H, D, bq)
    ref, ref_bits = oracle.gemm_q(X, W, None, None, bq, H, D, eps=float(np.float32(1e-5)), rope_cos=cos, rope_sin=sin)
    _check(got, ref, ref_bits, None, bq, "gemm_q norm + rope, no gain")


def test_fused_norm_rope_full_width_sampled():
    """Channel count of the video workload (3072 -> 24 heads x 128), 1024 tokens."""
    print("[case] gemm_q norm+rope C=3072", flush=True)
    B, L, C, H, D, bq = 1, 1024, 3072, 24, 128, 128
    X, W, b, flags = _case(51, B, L, C, H, D, bq, cached=0.5)
    g = synth.f32_to_bf16_bits((1.0 + 0.2 * np.random.default_rng(52).standard_normal(D)).astype(np.float32))
    cos, sin = _rope_tables(L, D)
    got = _run_fused(X, W, b, g, 1e-6, cos, sin, flags, B, L, C, H, D, bq)
    ref, ref_bits = oracle.gemm_q(X, W, b, flags, bq, H, D, norm_weight=g, eps=float(np.float32(1e-6)), rope_cos=cos, rope_sin=sin)
    _check(got, ref, ref_bits, flags, bq, "gemm_q norm+rope C=3072")


@pytest.mark.parametrize("D,bq,L", [(128, 128, 1000), (64, 64, 200), (128, 64, 513), (64, 128, 90)])
def test_short_last_token_block(D, bq, L):
    """ceil(L / block_q) token blocks; nothing past row L - 1 of X may be read, nothing past it of Q written."""
    print(f"[case] gemm_q ragged D={D} bq={bq} L={L}", flush=True)
    B, C, H = 1, 192, 3
    X, W, b, _ = _case(60 + L, B, L, C, H, D, bq, cached=0.0)
    Tq = -(-L // bq)
    flags = (np.random.default_rng(61 + L).random((B, H, Tq)) < 0.3).astype(np.uint8)
    flags[0, 0, -1] = 0                                   # the short block is computed for head 0 ...
    flags[0, 1, -1] = 1                                   # ... and skipped for head 1
    # X sits at the start of a larger buffer with NaN behind it, Q likewise with a marker behind it
    pad = 256
    xbuf = np.full((L + pad, C), 0x7FC0, dtype=np.uint16)
    xbuf[:L] = X[0]
    dX = up_bf16(xbuf)[:L].view(1, L, C)
    qbuf = torch.from_numpy(np.full((H * L + pad, D), 0x4242, dtype=np.uint16).view(np.int16)).view(torch.bfloat16).to("cuda:0")
    Q = qbuf[:H * L].view(1, H, L, D)
    cos, sin = _rope_tables(L, D)
    g = synth.f32_to_bf16_bits((1.0 + 0.2 * np.random.default_rng(62).standard_normal(D)).astype(np.float32))
    for fused in (False, True):
        qbuf.copy_(torch.from_numpy(np.full((H * L + pad, D), 0x4242, dtype=np.uint16).view(np.int16)).view(torch.bfloat16))
        if fused:
            pkg.sparse_gemm_q_norm_rope(dX, up_bf16(W), up_bf16(b), up_bf16(g), 1e-6, torch.from_numpy(cos).to("cuda:0"),
                                        torch.from_numpy(sin).to("cuda:0"), up_u8(flags), Q, bq)
            ref, ref_bits = oracle.gemm_q(X, W, b, flags, bq, H, D, norm_weight=g, eps=float(np.float32(1e-6)), rope_cos=cos, rope_sin=sin)
        else:
            pkg.sparse_gemm_q(dX, up_bf16(W), up_bf16(b), up_u8(flags), Q, bq)
            ref, ref_bits = oracle.gemm_q(X, W, b, flags, bq, H, D)
        torch.cuda.synchronize()
        whole = down_bits(qbuf)
        assert (whole[H * L:] == 0x4242).all(), "rows past the end of Q were written"
        got = whole[:H * L].reshape(1, H, L, D)
        skipped = np.repeat(flags != 0, bq, axis=2)[:, :, :L]
        assert (got[skipped] == 0x4242).all()
        vals = synth.bf16_bits_to_f32(got).astype(np.float64)[~skipped]
        assert np.isfinite(vals).all(), "something past the end of X was read"
        err = np.abs(vals - ref[~skipped])
        assert (err <= np.abs(ref[~skipped]) * 2.0 ** -8 + 1e-3).all()
        assert (got[~skipped] == ref_bits[~skipped]).mean() > 0.98
