"""Host-side checks of the C-ABI library: exported symbols, argument validation (which runs
before any HIP call, so no GPU is needed) and the pure-host helpers against the oracle."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import paper_2509_25401_amd as pkg
from paper_2509_25401_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    names = []
    inc = os.path.join(ROOT, "include")
    for fn in sorted(os.listdir(inc)):
        if not fn.endswith(".h"):
            continue
        text = open(os.path.join(inc, fn)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names += re.findall(r"\b(sparse_(?:attn|gemm|symbols|op|taylor)_\w+)\s*\(", text)
    return sorted(set(names))


def test_library_exports_every_declared_symbol():
    lib = pkg.load_library()
    names = _declared_functions()
    assert "sparse_attn_fwd" in names and "sparse_attn_fwd_stream" in names and "sparse_gemm_q" in names and "sparse_gemm_o" in names and "sparse_symbols_update" in names and "sparse_op_reuse" in names and "sparse_taylor_coefficients" in names and "sparse_taylor_update" in names and len(names) >= 19
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in include/ but not exported"
    assert pkg.sparse_attn_version() >= 100


def test_bench_probe_is_a_library_of_its_own():
    """The MFMA-only probe bench.py reports is built beside it and is neither exported by the product library nor
    declared in include/; its argument check needs no GPU."""
    path = os.path.join(ROOT, "bench_mfma_probe.so")
    if not os.path.exists(path):
        pytest.skip("bench_mfma_probe.so not built (python -c 'import __graft_entry__ as g; g.build()')")
    probe = ctypes.CDLL(path)
    probe.bench_mfma_probe.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
    probe.bench_mfma_probe.restype = ctypes.c_int
    assert probe.bench_mfma_probe(0, 0, None, None) == -1          # launches out of range, no result pointer
    assert probe.bench_mfma_probe(1, 65, None, None) == -1
    assert not hasattr(pkg.load_library(), "bench_mfma_probe")
    assert not any("probe" in n for n in _declared_functions())


FAKE = ctypes.c_void_p(0x10000)   # never dereferenced: every call below fails validation first


def _fwd(B=1, H=1, L=128, D=128, bq=128, bk=128, Q=FAKE, K=FAKE, V=FAKE, O=ctypes.c_void_p(0x90000000)):
    return pkg.load_library().sparse_attn_fwd(Q, K, V, None, None, None, O, B, H, L, D, bq, bk)


@pytest.mark.parametrize("kw,code", [
    (dict(B=0), -1), (dict(H=-1), -1), (dict(L=0), -1), (dict(D=0), -1),
    (dict(D=96), -2), (dict(D=256), -2),
    (dict(bq=32), -2), (dict(bk=256), -2), (dict(bq=0), -1),
    (dict(Q=None), -1), (dict(K=None), -1), (dict(V=None), -1), (dict(O=None), -1),
    (dict(O=FAKE), -1),                # O aliases Q
    (dict(O=ctypes.c_void_p(0x10000 + 64)), -1),   # O overlaps Q
    (dict(Q=ctypes.c_void_p(0x10008)), -1),        # misaligned
    (dict(L=64 * 20000, bq=64, bk=64), -2),        # Tq beyond the supported maximum
])
def test_argument_validation_precedes_any_device_work(kw, code):
    assert _fwd(**kw) == code
    assert pkg.sparse_attn_last_error() != ""


def test_no_alloc_entry_point_rejects_shapes_beyond_its_scratch():
    """The size check precedes every HIP call: B*H*Tq = 64*64*256 rows of 8 + 2 words need 40 MiB, the fixed array
    holds 2 MiB."""
    lib = pkg.load_library()
    assert pkg.sparse_attn_workspace_bytes(64, 64, 32768, 128, 128) > (2 << 20)
    far = [ctypes.c_void_p(0x10000 + k * (1 << 40)) for k in range(4)]
    rc = lib.sparse_attn_fwd_noalloc(far[0], far[1], far[2], None, None, None, far[3], 64, 64, 32768, 128, 128, 128, None)
    assert rc == -2 and "scratch" in pkg.sparse_attn_last_error()
    # validation of the ordinary arguments is shared with the other entry points
    assert lib.sparse_attn_fwd_noalloc(None, far[1], far[2], None, None, None, far[3], 1, 1, 128, 128, 128, 128, None) == -1


def test_caller_supplied_workspace_is_validated_before_any_device_work():
    lib = pkg.load_library()
    far = [ctypes.c_void_p(0x10000 + k * (1 << 40)) for k in range(4)]
    need = pkg.sparse_attn_workspace_bytes(1, 2, 1024, 128, 128)
    def call(ws, size):
        return lib.sparse_attn_fwd_workspace(far[0], far[1], far[2], None, None, None, far[3], 1, 2, 1024, 128, 128, 128,
                                             ws, size, None)
    assert call(None, need) == -1 and "workspace" in pkg.sparse_attn_last_error()
    assert call(ctypes.c_void_p(0x50000040), need) == -1 and "aligned" in pkg.sparse_attn_last_error()
    assert call(ctypes.c_void_p(0x50000000), need - 1) == -1 and str(need) in pkg.sparse_attn_last_error()


def test_workspace_bytes():
    assert pkg.sparse_attn_workspace_bytes(1, 24, 33024, 128, 128) >= 24 * 258 * (4 + 4 + 9 * 4)
    assert pkg.sparse_attn_workspace_bytes(1, 24, 33024, 128, 128) < 1 << 20
    assert pkg.sparse_attn_workspace_bytes(1, 1, 100, 128, 128) == pkg.sparse_attn_workspace_bytes(1, 1, 128, 128, 128) > 0
    assert pkg.sparse_attn_workspace_bytes(1, 1, 128, 32, 128) == 0


def test_pack_mask_matches_printed_example_and_oracle_packer():
    assert pkg.sparse_attn_pack_mask(np.array([1, 1, 1, 0])).tolist() == [224]   # Section 3.3 worked example
    rng = np.random.default_rng(3)
    for Tkv in (1, 7, 8, 9, 36, 258):
        M = (rng.random((2, 3, 5, Tkv)) < 0.5).astype(np.uint8)
        assert (pkg.sparse_attn_pack_mask(M) == oracle.pack_symbols(M)).all()


def test_count_kept_matches_oracle_accounting():
    w = synth.random_case(40, 2, 3, 1152, 8, 128, 64, keep=0.35, cached_frac=0.4)
    mask = pkg.sparse_attn_pack_mask(w.M_s)
    dirty = mask.copy()
    dirty[..., -1] |= 0x3F      # Tkv = 18: the last byte has 6 padding bits
    for m in (mask, dirty):
        assert pkg.sparse_attn_count_kept(w.cache_flags, m, w.B, w.H, w.L, 128, 64) == \
            oracle.count_pairs(w.cache_flags, mask, w.B, w.H, w.L, 128, 64) == (w.kept_pairs(), w.total_pairs())
    assert pkg.sparse_attn_count_kept(None, None, w.B, w.H, w.L, 128, 64) == (w.total_pairs(), w.total_pairs())
    # a short last block counts as a block (Definition 1): 100 tokens = 1 query block x 2 key blocks
    assert pkg.sparse_attn_count_kept(None, None, 1, 1, 100, 128, 64) == oracle.count_pairs(None, None, 1, 1, 100, 128, 64) == (2, 2)
    with pytest.raises(pkg.SparseAttnError):
        pkg.sparse_attn_count_kept(None, None, 1, 1, 100, 32, 64)


def test_workload_recipes_hit_their_keep_ratios():
    w2 = synth.config_image_skip()
    assert abs(w2.kept_pairs() / w2.total_pairs() - 0.5) < 0.01
    assert (w2.M_s[..., :4] == 1).all() and all(w2.M_s[0, 0, i, i] for i in range(w2.Tq))
    w3 = synth.config_image_cache_skip()
    assert (w3.cache_flags.sum(axis=-1) == 18).all() and (w3.cache_flags[..., :4] == 0).all()
    rows = w3.M_s[w3.cache_flags == 0]
    assert abs(rows.mean() - 0.3) < 0.01


def _gemm_q(B=1, L=128, C=64, H=1, D=128, bq=128, X=FAKE, W=ctypes.c_void_p(0x20000000), Q=ctypes.c_void_p(0x90000000)):
    return pkg.load_library().sparse_gemm_q(X, W, None, None, Q, B, L, C, H, D, bq)


@pytest.mark.parametrize("kw,code", [
    (dict(B=0), -1), (dict(L=0), -1), (dict(C=0), -1), (dict(H=0), -1), (dict(D=0), -1), (dict(bq=0), -1),
    (dict(C=96), -2),                    # channels must come in stages of 64
    (dict(D=96), -2), (dict(bq=32), -2),
    (dict(X=None), -1), (dict(W=None), -1), (dict(Q=None), -1),
    (dict(Q=FAKE), -1),                  # Q aliases X
    (dict(X=ctypes.c_void_p(0x10004)), -1),
])
def test_gemm_q_argument_validation_precedes_any_device_work(kw, code):
    assert _gemm_q(**kw) == code
    assert pkg.sparse_attn_last_error() != ""


def _gemm_o(B=1, H=2, L=128, D=128, C_out=128, bq=128, sel=0, O=FAKE, W=ctypes.c_void_p(0x20000000),
            addend=None, Out=ctypes.c_void_p(0x90000000)):
    return pkg.load_library().sparse_gemm_o(O, W, None, None, sel, addend, Out, B, H, L, D, C_out, bq)


@pytest.mark.parametrize("kw,code", [
    (dict(B=0), -1), (dict(H=0), -1), (dict(L=0), -1), (dict(D=0), -1), (dict(C_out=0), -1), (dict(bq=0), -1),
    (dict(sel=2), -1),
    (dict(C_out=192), -2), (dict(D=96), -2), (dict(bq=32), -2), (dict(H=65), -2),
    (dict(O=None), -1), (dict(W=None), -1), (dict(Out=None), -1),
    (dict(Out=FAKE), -1),                                   # Out aliases O
    (dict(addend=ctypes.c_void_p(0x90000000 + 64)), -1),    # addend overlaps Out without being Out
    (dict(O=ctypes.c_void_p(0x10004)), -1),
])
def test_gemm_o_argument_validation_precedes_any_device_work(kw, code):
    assert _gemm_o(**kw) == code
    assert pkg.sparse_attn_last_error() != ""


def _symbols(B=1, H=1, L=512, D=128, blk=128, text=128, tau_c=0.5, tau_kv=0.1, s_q=0.0, Q=FAKE,
             K=ctypes.c_void_p(0x20000000), flags=ctypes.c_void_p(0x30000000), mask=ctypes.c_void_p(0x40000000)):
    return pkg.load_library().sparse_symbols_update(Q, K, flags, mask, B, H, L, D, blk, text, tau_c, tau_kv, s_q)


@pytest.mark.parametrize("kw,code", [
    (dict(B=0), -1), (dict(H=0), -1), (dict(L=0), -1), (dict(D=0), -1), (dict(blk=0), -1),
    (dict(text=400), -1),                                   # ceil(400 / 128) = 4 text blocks of 4: no vision block left
    (dict(text=0), -1), (dict(text=512), -1),               # no text tokens / no vision tokens
    (dict(D=96), -2), (dict(blk=32), -2),
    (dict(L=128 * 2049, text=128), -2),                      # more blocks than the kernels are sized for
    (dict(tau_c=-0.1), -1), (dict(tau_c=1.5), -1), (dict(tau_kv=float("nan")), -1), (dict(s_q=2.0), -1),
    (dict(Q=None), -1), (dict(K=None), -1), (dict(flags=None), -1), (dict(mask=None), -1),
    (dict(Q=ctypes.c_void_p(0x10004)), -1),
])
def test_symbols_argument_validation_precedes_any_device_work(kw, code):
    assert _symbols(**kw) == code
    assert pkg.sparse_attn_last_error() != ""


@pytest.mark.parametrize("kw,code", [
    (dict(n=0), -1), (dict(n=65), -1), (dict(bk=32), -2), (dict(bq=256), -2),
    (dict(n=4, L=1024, text=600), -1),                      # pooled blocks of 512 tokens: both query blocks hold text
    (dict(n=2, bk=64, L=512, text=300), -1),                # 256-token query blocks: ceil(300 / 256) = 2 of 2 are text
    (dict(n=16, L=128 * 16 * 2049, text=128), -2),          # more pooled blocks than the kernels are sized for
])
def test_granular_symbols_argument_validation(kw, code):
    a = dict(B=1, H=1, L=512, D=128, bq=128, bk=128, n=1, text=128)
    a.update(kw)
    rc = pkg.load_library().sparse_symbols_update_granular(
        FAKE, ctypes.c_void_p(0x20000000), ctypes.c_void_p(0x30000000), ctypes.c_void_p(0x40000000), a["B"], a["H"],
        a["L"], a["D"], a["bq"], a["bk"], a["n"], a["text"], 0.5, 0.1, 0.0, None)
    assert rc == code and pkg.sparse_attn_last_error() != ""


def _ptr_array(vals):
    arr = (ctypes.c_void_p * len(vals))(*vals)
    return arr


def _op_reuse(n_terms=2, terms=(0x10000, 0x20000000), coef=(1.0, 0.5), out=ctypes.c_void_p(0x90000000), n=1024,
              null_terms=False, null_coef=False):
    t = None if null_terms else _ptr_array(list(terms))
    c = None if null_coef else (ctypes.c_float * len(coef))(*coef)
    return pkg.load_library().sparse_op_reuse(t, c, n_terms, out, n, None)


@pytest.mark.parametrize("kw,code", [
    (dict(n_terms=0), -2), (dict(n_terms=5), -2),
    (dict(null_terms=True), -1), (dict(null_coef=True), -1), (dict(out=None), -1),
    (dict(n=0), -1), (dict(n=1001), -1),
    (dict(terms=(0x10000, None)), -1), (dict(terms=(0x10004, 0x20000000)), -1),
    (dict(out=ctypes.c_void_p(0x90000008)), -1),
    (dict(terms=(0x10000, 0x90000000 + 64)), -1),          # overlaps out without being out
    (dict(coef=(1.0, float("inf"))), -1), (dict(coef=(float("nan"), 1.0)), -1),
])
def test_op_reuse_argument_validation_precedes_any_device_work(kw, code):
    assert _op_reuse(**kw) == code
    assert pkg.sparse_attn_last_error() != ""


def _forecast(n_terms=2, terms=(0x30000000, 0x40000000), coef=(1.0, 2.0), O=ctypes.c_void_p(0x90000000), null_terms=False,
              B=1, H=1, L=128, D=128, bq=128, bk=128):
    t = None if null_terms else _ptr_array(list(terms))
    c = (ctypes.c_float * len(coef))(*coef)
    return pkg.load_library().sparse_attn_fwd_forecast(FAKE, ctypes.c_void_p(0x20000000), ctypes.c_void_p(0x28000000), None, None,
                                                       t, c, n_terms, O, B, H, L, D, bq, bk, None)


@pytest.mark.parametrize("kw,code", [
    (dict(n_terms=0), -2), (dict(n_terms=5), -2), (dict(null_terms=True), -1),
    (dict(terms=(0x30000000, None)), -1), (dict(terms=(0x30000004, 0x40000000)), -1),
    (dict(terms=(0x30000000, 0x90000000)), -1),            # a term overlaps O
    (dict(coef=(1.0, float("nan"))), -1),
    (dict(L=0), -1), (dict(D=96), -2),
])
def test_forecast_argument_validation_precedes_any_device_work(kw, code):
    assert _forecast(**kw) == code
    assert pkg.sparse_attn_last_error() != ""


def test_taylor_coefficients_match_the_oracle():
    import oracle
    for order, k in ((0, 3.0), (1, 2.0), (2, 2.5), (3, 4.0)):
        assert pkg.sparse_taylor_coefficients(order, k) == [float(np.float32(c)) for c in oracle.taylor_coefficients(order, k)]


def _gemm_q_nr(eps=1e-6, cos=ctypes.c_void_p(0x50000000), sin=ctypes.c_void_p(0x58000000), norm=ctypes.c_void_p(0x60000000),
               B=1, L=128, C=64, H=1, D=128, bq=128):
    return pkg.load_library().sparse_gemm_q_norm_rope(FAKE, ctypes.c_void_p(0x20000000), None, norm, eps, cos, sin, None,
                                                      ctypes.c_void_p(0x90000000), B, L, C, H, D, bq, None)


@pytest.mark.parametrize("kw,code", [
    (dict(eps=-1.0), -1), (dict(eps=float("nan")), -1), (dict(eps=float("inf")), -1),
    (dict(sin=None), -1), (dict(cos=None), -1),                 # only one of the two tables
    (dict(cos=ctypes.c_void_p(0x50000004)), -1),
    (dict(norm=ctypes.c_void_p(0x60000001)), -1),
    (dict(L=0), -1), (dict(C=96), -2), (dict(D=96), -2),
])
def test_gemm_q_norm_rope_argument_validation_precedes_any_device_work(kw, code):
    assert _gemm_q_nr(**kw) == code
    assert pkg.sparse_attn_last_error() != ""


def test_plan_create_validation_precedes_any_device_work():
    lib = pkg.load_library()
    h = ctypes.c_void_p(0x1234)
    for kw, code in ((dict(L=0), -1), (dict(bq=32), -2), (dict(g=0), -1), (dict(g=65), -1), (dict(B=0), -1)):
        a = dict(B=1, H=1, L=256, bq=128, bk=128, g=1)
        a.update(kw)
        assert lib.sparse_attn_plan_create(None, None, a["B"], a["H"], a["L"], a["bq"], a["bk"], a["g"], None, ctypes.byref(h)) == code
        assert h.value is None and pkg.sparse_attn_last_error() != ""
        h = ctypes.c_void_p(0x1234)
    assert lib.sparse_attn_plan_create(None, None, 1, 1, 256, 128, 128, 1, None, None) == -1
    assert lib.sparse_attn_plan_run(None, FAKE, FAKE, FAKE, None, FAKE, 128, None) == -1
    assert lib.sparse_attn_plan_run_forecast(None, FAKE, FAKE, FAKE, None, None, 1, FAKE, 128, None) == -1
    assert lib.sparse_attn_plan_destroy(None) == 0


def _taylor_update(n_terms=2, n_valid=1, interval=5.0, fresh=FAKE, terms=(0x20000000, 0x30000000), n=1024, null_terms=False):
    t = None if null_terms else _ptr_array(list(terms))
    return pkg.load_library().sparse_taylor_update(fresh, t, n_terms, n_valid, interval, n, None)


@pytest.mark.parametrize("kw,code", [
    (dict(n_terms=0), -2), (dict(n_terms=5), -2), (dict(n_valid=-1), -1), (dict(n_valid=3), -1),
    (dict(interval=0.0), -1), (dict(interval=float("nan")), -1), (dict(interval=float("inf")), -1),
    (dict(fresh=None), -1), (dict(null_terms=True), -1), (dict(n=0), -1), (dict(n=1001), -1),
    (dict(terms=(0x20000000, None)), -1), (dict(terms=(0x20000004, 0x30000000)), -1),
    (dict(terms=(0x20000000, 0x20000100)), -1),            # two terms overlap
    (dict(terms=(0x10000 + 64, 0x30000000)), -1),          # a term overlaps fresh
])
def test_taylor_update_argument_validation_precedes_any_device_work(kw, code):
    assert _taylor_update(**kw) == code
    assert pkg.sparse_attn_last_error() != ""


def _cpu_case(B=1, H=2, L=256, D=64, bq=64, bk=128):
    import torch
    Tq, Tkv = -(-L // bq), -(-L // bk)
    t = lambda: torch.zeros((B, H, L, D), dtype=torch.bfloat16)
    return dict(Q=t(), K=t(), V=t(), O=t(), O_cache=t(), flags=torch.zeros((B, H, Tq), dtype=torch.uint8),
                mask=torch.zeros((B, H, Tq, (Tkv + 7) // 8), dtype=torch.uint8), bq=bq, bk=bk)


@pytest.mark.parametrize("field,make,needle", [
    ("Q", lambda t: t.float(), "dtype"),
    ("V", lambda t: t.to(__import__("torch").float16), "dtype"),
    ("K", lambda t: t[:, :, :128], "shape"),
    ("O", lambda t: t[:, :1], "shape"),
    ("O_cache", lambda t: t[..., :32], "shape"),
    ("flags", lambda t: t.to(__import__("torch").int32), "dtype"),
    ("flags", lambda t: t.bool(), "dtype"),
    ("flags", lambda t: t[..., :3], "shape"),                  # Tq = 4
    ("mask", lambda t: t.to(__import__("torch").int64), "dtype"),
    ("mask", lambda t: __import__("torch").zeros((1, 2, 4, 2), dtype=__import__("torch").uint8), "shape"),   # packed for block_k = 64
    ("mask", lambda t: t[:, :, :2], "shape"),
])
def test_binding_rejects_tensors_the_kernels_would_read_past(field, make, needle):
    """Wrong dtype or shape is caught in the binding, before any pointer reaches the library (CPU tensors suffice:
    the checks come first, and a tensor that passes them but is not in device memory is rejected after them)."""
    c = _cpu_case()
    c[field] = make(c[field])
    with pytest.raises(ValueError, match=needle):
        pkg.sparse_attn_fwd(c["Q"], c["K"], c["V"], c["flags"], c["mask"], c["O_cache"], c["O"], c["bq"], c["bk"])
    with pytest.raises(ValueError, match=needle):
        pkg.sparse_attn_fwd_noalloc(c["Q"], c["K"], c["V"], c["flags"], c["mask"], c["O_cache"], c["O"], c["bq"], c["bk"])
    ok = _cpu_case()
    with pytest.raises(ValueError, match="device memory"):
        pkg.sparse_attn_fwd(ok["Q"], ok["K"], ok["V"], ok["flags"], ok["mask"], ok["O_cache"], ok["O"], ok["bq"], ok["bk"])


def test_plan_binding_checks_symbol_shapes_with_granularity():
    import torch
    B, H, L, bq, bk, n = 1, 2, 1280, 128, 64, 3          # Tq = 10, Tkv = 20 -> 4 x 7 symbols, 1 mask byte per row
    good_f = torch.zeros((B, H, 4), dtype=torch.uint8)
    good_m = torch.zeros((B, H, 4, 1), dtype=torch.uint8)
    for f, m, needle in ((good_f[..., :3], good_m, "shape"), (good_f, torch.zeros((B, H, 4, 3), dtype=torch.uint8), "shape"),
                         (good_f.int(), good_m, "dtype"), (good_f, good_m.bool(), "dtype")):
        with pytest.raises(ValueError, match=needle):
            pkg.SparseAttnPlan(f, m, B, H, L, bq, bk, granularity=n)
    with pytest.raises(ValueError, match="device memory"):
        pkg.SparseAttnPlan(good_f, good_m, B, H, L, bq, bk, granularity=n)
