"""Shared plumbing of the GPU parity tests: upload a workload, call the C-ABI, compare."""
import numpy as np
import torch

import oracle
import paper_2509_25401_amd as pkg
from paper_2509_25401_amd import synth

MAX_ABS_TOL = 1e-2    # computed outputs, N(0,1) inputs
MEAN_ABS_TOL = 1e-3


def dev():
    return torch.device("cuda:0")


def up_bf16(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).to(dev())


def down_bits(t):
    return t.cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def up_u8(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint8)).to(dev())


class DeviceCase:
    """A workload resident on the GPU, symbols packed by the product's own packer."""

    def __init__(self, w, o_fill=0x4242):
        self.w = w
        self.Q, self.K, self.V = up_bf16(w.Q), up_bf16(w.K), up_bf16(w.V)
        self.Oc = None if w.O_cache is None else up_bf16(w.O_cache)
        self.flags = up_u8(w.cache_flags)
        self.mask_host = None if w.M_s is None else pkg.sparse_attn_pack_mask(w.M_s)
        self.mask = up_u8(self.mask_host)
        self.o_fill = o_fill

    def run(self, O_cache="own", mask="own", flags="own", timed=False):
        w = self.w
        O = torch.from_numpy(np.full(w.Q.shape, self.o_fill, dtype=np.uint16).view(np.int16)).view(torch.bfloat16).to(dev())
        oc = self.Oc if isinstance(O_cache, str) else O_cache
        if isinstance(O_cache, str) and O_cache == "alias":
            oc = O
        mk = self.mask if isinstance(mask, str) else mask
        fl = self.flags if isinstance(flags, str) else flags
        fn = pkg.sparse_attn_fwd_timed if timed else pkg.sparse_attn_fwd
        res = fn(self.Q, self.K, self.V, fl, mk, oc, O, w.block_q, w.block_k)
        torch.cuda.synchronize()
        return (down_bits(O), res) if timed else down_bits(O)


def oracle_full(w):
    mask = None if w.M_s is None else oracle.pack_symbols(w.M_s)
    return oracle.sparse_attention(w.Q, w.K, w.V, w.cache_flags, mask, w.O_cache, w.block_q, w.block_k)


def cached_rows(w):
    if w.cache_flags is None:
        return np.zeros((w.B, w.H, w.L), dtype=bool)
    return np.repeat(np.asarray(w.cache_flags) != 0, w.block_q, axis=2)[:, :, :w.L]


def check_against_oracle(w, got_bits, ref_f64, ref_bits, label=""):
    """The parity bar: cached blocks bit exact; computed outputs max-abs <= 1e-2, mean-abs <= 1e-3."""
    c = cached_rows(w)
    if c.any():
        assert (got_bits[c] == ref_bits[c]).all(), f"{label}: cached blocks are not bit exact"
    comp = ~c
    got = synth.bf16_bits_to_f32(got_bits).astype(np.float64)
    assert np.isfinite(got[comp]).all(), f"{label}: non-finite output"
    err = np.abs(got[comp] - ref_f64[comp])
    rel = np.sqrt((err ** 2).sum() / max((ref_f64[comp] ** 2).sum(), 1e-300))
    print(f"[parity] {label or w.name}: max-abs {err.max():.3e} mean-abs {err.mean():.3e} rel-fro {rel:.3e}", flush=True)
    assert err.max() <= MAX_ABS_TOL, f"{label}: max abs error {err.max()}"
    assert err.mean() <= MEAN_ABS_TOL, f"{label}: mean abs error {err.mean()}"
    assert rel <= 2e-2, f"{label}: relative error {rel}"
    return err.max(), err.mean(), rel
