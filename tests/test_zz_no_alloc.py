"""GPU test of sparse_attn_fwd_noalloc, the entry point for callers that cannot allocate: through the C ABI it
must write the same bits as sparse_attn_fwd_stream, on two calls in a row that share the library's fixed scratch
array, the second with a smaller input (the array then still holds the longer work list of the first call)."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2509_25401_amd as pkg
from paper_2509_25401_amd import synth
from gpu_utils import DeviceCase, dev, down_bits, oracle_full, check_against_oracle

pytestmark = pytest.mark.gpu


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _call(entry, case, O):
    """Calls `entry` (a ctypes function with sparse_attn_fwd_stream's signature) on raw pointers."""
    w = case.w
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    rc = entry(_ptr(case.Q), _ptr(case.K), _ptr(case.V), _ptr(case.flags), _ptr(case.mask), _ptr(case.Oc), _ptr(O),
               w.B, w.H, w.L, w.D, w.block_q, w.block_k, stream)
    assert rc == 0, pkg.sparse_attn_last_error()
    torch.cuda.synchronize()
    return down_bits(O)


def _fresh(w, fill):
    return torch.from_numpy(np.full(w.Q.shape, fill, dtype=np.uint16).view(np.int16)).view(torch.bfloat16).to(dev())


def test_no_alloc_entry_point_matches_the_allocating_one_twice_in_a_row():
    lib = pkg.load_library()
    big = synth.random_case(synth.BASE_SEED + 701, 2, 3, 1664, 128, 128, 128, keep=0.4, cached_frac=0.3)
    small = synth.random_case(synth.BASE_SEED + 702, 1, 2, 600, 64, 64, 128, keep=0.6, cached_frac=0.25)
    for label, w in (("first call", big), ("second, smaller call", small)):
        case = DeviceCase(w)
        want = _call(lib.sparse_attn_fwd_stream, case, _fresh(w, 0x4242))
        got = _call(lib.sparse_attn_fwd_noalloc, case, _fresh(w, 0x4242))
        assert (got == want).all(), f"{label}: output differs from sparse_attn_fwd_stream"
        ref, ref_bits = oracle_full(w)
        check_against_oracle(w, got, ref, ref_bits, f"no-alloc, {label}")
