"""Seeded synthetic workloads shaped like the paper's DiT attention calls.

This module only draws random inputs and logical block masks.  It holds none of the
method's arithmetic: no attention, no symbol packing, no scheduling.  Both the GPU path
and the test oracle are fed from here; each packs the logical masks with its own packer.

The paper benchmarks its kernel with randomly generated sparse symbols at the token
counts of FLUX.1-dev (4.5K) and HunyuanVideo (33K) (Section 4.3 and the attention
appendix); the model activations, COCO-2017 / VBench prompts and weights are not
available here, so N(0,1) tensors of those shapes stand in for them.  Text tokens come
first in the sequence (the compressed map is sliced as [:n_t, n_t:] in Section 3.3), text
query blocks are never cached and text key blocks are always kept (Observation 1).
"""
from dataclasses import dataclass, field
from typing import Optional

import numpy as np

BASE_SEED = 250925400


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest even); returns the 16-bit patterns as uint16."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal_bf16(rng: np.random.Generator, shape, chunk: int = 1 << 24) -> np.ndarray:
    """N(0,1) samples rounded to bf16, generated in chunks to bound peak memory."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint16)
    for s in range(0, n, chunk):
        e = min(n, s + chunk)
        out[s:e] = f32_to_bf16_bits(rng.standard_normal(e - s, dtype=np.float32))
    return out.reshape(shape)


@dataclass
class Workload:
    name: str
    B: int
    H: int
    L: int
    D: int
    block_q: int
    block_k: int
    Q: np.ndarray            # uint16 [B,H,L,D] bf16 bit patterns
    K: np.ndarray
    V: np.ndarray
    M_s: Optional[np.ndarray]          # uint8 {0,1} [B,H,Tq,Tkv]; 1 = compute the pair; None = all kept
    cache_flags: Optional[np.ndarray]  # uint8 {0,1} [B,H,Tq]; 1 = reuse cached block; None = none
    O_cache: Optional[np.ndarray]      # uint16 [B,H,L,D] or None
    notes: dict = field(default_factory=dict)

    @property
    def Tq(self):
        return -(-self.L // self.block_q)

    @property
    def Tkv(self):
        return -(-self.L // self.block_k)

    def kept_pairs(self) -> int:
        """Number of (q-block, kv-block) pairs that are computed (plain counting on the logical mask)."""
        rows = np.ones((self.B, self.H, self.Tq), dtype=bool) if self.cache_flags is None else (self.cache_flags == 0)
        if self.M_s is None:
            return int(rows.sum()) * self.Tkv
        return int((self.M_s.astype(bool) & rows[..., None]).sum())

    def total_pairs(self) -> int:
        return self.B * self.H * self.Tq * self.Tkv


def _rngs(index: int, n: int):
    return [np.random.default_rng(s) for s in np.random.SeedSequence(BASE_SEED + index).spawn(n)]


def _fill_to_keep(rng, forced: np.ndarray, keep: float) -> np.ndarray:
    """forced: bool [..., Tkv].  Adds Bernoulli entries so that every row keeps `keep` in expectation."""
    Tkv = forced.shape[-1]
    f = forced.sum(axis=-1, keepdims=True).astype(np.float64)
    p = np.clip((keep * Tkv - f) / np.maximum(Tkv - f, 1.0), 0.0, 1.0)
    extra = rng.random(forced.shape) < p
    return (forced | extra)


def _qkv(rngs, B, H, L, D, with_cache):
    Q = normal_bf16(rngs[0], (B, H, L, D))
    K = normal_bf16(rngs[1], (B, H, L, D))
    V = normal_bf16(rngs[2], (B, H, L, D))
    Oc = normal_bf16(rngs[3], (B, H, L, D)) if with_cache else None
    return Q, K, V, Oc


def random_case(seed, B, H, L, D, block_q, block_k, keep=0.5, cached_frac=0.0, name=None,
                force_diagonal=True, with_cache_tensor=None) -> Workload:
    """Generic small case: i.i.d. Bernoulli(keep) mask (+ diagonal), random cached rows."""
    r = [np.random.default_rng(s) for s in np.random.SeedSequence(seed).spawn(6)]
    Tq, Tkv = -(-L // block_q), -(-L // block_k)      # a short last block counts as a block
    with_cache = cached_frac > 0 if with_cache_tensor is None else with_cache_tensor
    Q, K, V, Oc = _qkv(r, B, H, L, D, with_cache)
    M = r[4].random((B, H, Tq, Tkv)) < keep
    if force_diagonal:
        for i in range(Tq):
            M[:, :, i, min(Tkv - 1, (i * block_q) // block_k)] = True
    flags = None
    if cached_frac > 0:
        flags = (r[5].random((B, H, Tq)) < cached_frac).astype(np.uint8)
    return Workload(name or f"random-{seed}", B, H, L, D, block_q, block_k, Q, K, V,
                    M.astype(np.uint8), flags, Oc)


def config_tiny() -> Workload:
    """Config 1: B=1 H=2 L=512 D=64, 64x64 blocks, Bernoulli(0.5) mask with the diagonal kept, no caching."""
    B, H, L, D, bq, bk = 1, 2, 512, 64, 64, 64
    r = _rngs(1, 6)
    Q, K, V, _ = _qkv(r, B, H, L, D, False)
    T = L // bq
    M = r[4].random((B, H, T, T)) < 0.5
    M |= np.eye(T, dtype=bool)[None, None]
    return Workload("tiny", B, H, L, D, bq, bk, Q, K, V, M.astype(np.uint8), None, None)


def _image_shapes():
    return 1, 24, 4608, 128, 128, 128, 4  # B,H,L,D,bq,bk, text blocks


def config_image_skip(keep: float = 0.5) -> Workload:
    """Config 2: image-DiT shape, skipping only; text key columns + diagonal + Bernoulli fill to `keep` overall."""
    B, H, L, D, bq, bk, nt = _image_shapes()
    r = _rngs(2, 6)
    Q, K, V, _ = _qkv(r, B, H, L, D, False)
    T = L // bq
    forced = np.zeros((B, H, T, T), dtype=bool)
    forced[..., :nt] = True
    forced |= np.eye(T, dtype=bool)[None, None]
    nf = forced[0, 0].sum()
    p = (keep * T * T - nf) / (T * T - nf)
    M = forced | (r[4].random(forced.shape) < p)
    return Workload("image-skip", B, H, L, D, bq, bk, Q, K, V, M.astype(np.uint8), None, None,
                    {"text_blocks": nt, "target_keep": keep})


def config_image_cache_skip(keep: float = 0.3, cached: int = 18) -> Workload:
    """Config 3: image-DiT shape; per head `cached` of the 32 vision q-blocks flagged; other rows keep ~30%."""
    B, H, L, D, bq, bk, nt = _image_shapes()
    r = _rngs(3, 6)
    Q, K, V, Oc = _qkv(r, B, H, L, D, True)
    T = L // bq
    forced = np.zeros((B, H, T, T), dtype=bool)
    forced[..., :nt] = True
    forced |= np.eye(T, dtype=bool)[None, None]
    M = _fill_to_keep(r[4], forced, keep)
    flags = np.zeros((B, H, T), dtype=np.uint8)
    for b in range(B):
        for h in range(H):
            flags[b, h, nt + r[5].permutation(T - nt)[:cached]] = 1
    # symbol rows of cached blocks are never read: fill them with noise
    noise = r[5].random(M.shape) < 0.5
    M = np.where(flags[..., None] != 0, noise, M)
    return Workload("image-cache-skip", B, H, L, D, bq, bk, Q, K, V, M.astype(np.uint8), flags, Oc,
                    {"text_blocks": nt, "target_keep": keep, "cached_per_head": cached})


VIDEO_SHAPE = dict(B=1, H=24, L=33024, D=128, block_q=128, block_k=128, text_blocks=2, T_lat=8, Yp=32)


def _video_window(T, nt, T_lat, Yp):
    """Local 3-D window between video blocks: |dt| <= 1 and |dyp| <= 2 (block v = t*Yp + yp covers two latent rows)."""
    w = np.zeros((T, T), dtype=bool)
    v = np.arange(T - nt)
    t, y = v // Yp, v % Yp
    near = (np.abs(t[:, None] - t[None, :]) <= 1) & (np.abs(y[:, None] - y[None, :]) <= 2)
    w[nt:, nt:] = near
    return w


def config_video_multi(keep: float = 0.25, cached_frac: float = 0.25, H: Optional[int] = None,
                       seed_index: int = 4) -> Workload:
    """Config 4: video-DiT shape, 25% of the video q-blocks cached, 25% keep from window + text + random fill."""
    s = VIDEO_SHAPE
    B, L, D, bq, bk, nt = s["B"], s["L"], s["D"], s["block_q"], s["block_k"], s["text_blocks"]
    H = s["H"] if H is None else H
    r = _rngs(seed_index, 6)
    Q, K, V, Oc = _qkv(r, B, H, L, D, True)
    T = L // bq
    forced = np.zeros((B, H, T, T), dtype=bool)
    forced[..., :nt] = True
    forced[:, :, :nt, :] |= np.eye(T, dtype=bool)[None, None, :nt]
    forced |= _video_window(T, nt, s["T_lat"], s["Yp"])[None, None]
    M = _fill_to_keep(r[4], forced, keep)
    ncache = int(round(cached_frac * (T - nt)))
    flags = np.zeros((B, H, T), dtype=np.uint8)
    for b in range(B):
        for h in range(H):
            flags[b, h, nt + r[5].permutation(T - nt)[:ncache]] = 1
    noise = r[5].random(M.shape) < 0.5
    M = np.where(flags[..., None] != 0, noise, M)
    return Workload("video-multi", B, H, L, D, bq, bk, Q, K, V, M.astype(np.uint8), flags, Oc,
                    {"text_blocks": nt, "target_keep": keep, "cached_per_head": ncache})


def video_sweep_mask(rng, B, H, T, nt, keep: float, skewed: bool = False):
    """Config 5 masks: band |i-j| <= 1 + text columns + Bernoulli fill; `skewed`: 10% of rows keep 90%."""
    if keep >= 1.0:
        return np.ones((B, H, T, T), dtype=np.uint8)
    i = np.arange(T)
    forced = np.zeros((B, H, T, T), dtype=bool)
    forced |= (np.abs(i[:, None] - i[None, :]) <= 1)[None, None]
    forced[..., :nt] = True
    if not skewed:
        return _fill_to_keep(rng, forced, keep).astype(np.uint8)
    rest = (keep - 0.09) / 0.9
    if rest <= 0:
        raise ValueError("skewed variant infeasible at this keep ratio")
    heavy = np.zeros((B, H, T), dtype=bool)
    nheavy = int(round(0.1 * T))
    for b in range(B):
        for h in range(H):
            heavy[b, h, rng.permutation(T)[:nheavy]] = True
    row_keep = np.where(heavy, 0.9, rest)[..., None]
    Tkv = T
    f = forced.sum(axis=-1, keepdims=True).astype(np.float64)
    p = np.clip((row_keep * Tkv - f) / np.maximum(Tkv - f, 1.0), 0.0, 1.0)
    return (forced | (rng.random(forced.shape) < p)).astype(np.uint8)


def config_video_sweep(keep: float, skewed: bool = False, H: Optional[int] = None,
                       tensors: Optional[tuple] = None) -> Workload:
    """Config 5: video shape, no caching, band + text + random mask at the given keep ratio.

    `tensors` = (Q, K, V) reuses already drawn inputs so a sweep draws them once.
    """
    s = VIDEO_SHAPE
    B, L, D, bq, bk, nt = s["B"], s["L"], s["D"], s["block_q"], s["block_k"], s["text_blocks"]
    H = s["H"] if H is None else H
    r = _rngs(5, 6)
    if tensors is None:
        Q, K, V, _ = _qkv(r, B, H, L, D, False)
    else:
        Q, K, V = tensors
    T = L // bq
    mrng = np.random.default_rng(np.random.SeedSequence([BASE_SEED + 5, int(round(keep * 10000)), int(skewed)]))
    M = video_sweep_mask(mrng, B, H, T, nt, keep, skewed)
    name = f"video-sweep-{keep:g}" + ("-skewed" if skewed else "")
    return Workload(name, B, H, L, D, bq, bk, Q, K, V, M, None, None,
                    {"text_blocks": nt, "target_keep": keep, "skewed": skewed})


PAPER_POINTS = ("bss80", "fc80", "combined90")


def paper_operating_point(name: str, H: Optional[int] = None):
    """Symbols of the three operating points the paper quotes for its kernel (Section 4.3 and the attention
    sweep of the appendix, random symbols): 'bss80' = 80 % block-sparse skipping (20 % keep, nothing cached),
    'fc80' = 80 % of the vision query blocks cached (nothing skipped), 'combined90' = half of the vision query
    blocks cached and the rest at 20 % keep.  Returns (M_s or None, cache_flags or None) at the video shape."""
    s = VIDEO_SHAPE
    B, T, nt = s["B"], s["L"] // s["block_q"], s["text_blocks"]
    H = s["H"] if H is None else H
    rng = np.random.default_rng(np.random.SeedSequence([BASE_SEED + 6, PAPER_POINTS.index(name)]))

    def vision_flags(frac):
        f = np.zeros((B, H, T), dtype=np.uint8)
        n = int(round(frac * (T - nt)))
        for b in range(B):
            for h in range(H):
                f[b, h, nt + rng.permutation(T - nt)[:n]] = 1
        return f
    M = None if name == "fc80" else video_sweep_mask(rng, B, H, T, nt, 0.2, False)
    flags = None if name == "bss80" else vision_flags(0.8 if name == "fc80" else 0.5)
    return M, flags


def structured_qk(seed, B, H, L, D, block, signal=1.2):
    """Q, K with block-level structure, for the symbol generation of an Update step: every block of `block`
    tokens shares a random direction of strength `signal` on top of N(0,1) noise, so that the mean-pooled
    attention map has logits of O(1) spread (pure noise pools to an almost uniform map)."""
    r = [np.random.default_rng(s) for s in np.random.SeedSequence(seed).spawn(4)]
    T = L // block
    out = []
    for k in range(2):
        mu = (signal * r[k].standard_normal((B, H, T, 1, D), dtype=np.float32))
        x = r[2 + k].standard_normal((B, H, T, block, D), dtype=np.float32) + mu
        out.append(f32_to_bf16_bits(x.reshape(B, H, L, D)))
    return out[0], out[1]
