"""Pins of the OP_reuse (Taylor forecast) oracle: textbook facts about Taylor polynomials."""
import math

import numpy as np

import oracle
from paper_2509_25401_amd import synth
from helpers import bits_to_f64


def exact_bf16(x):
    """float64 array -> bf16 bits, asserting that the values are exactly representable."""
    bits = synth.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))
    assert (bits_to_f64(bits) == np.asarray(x, dtype=np.float64)).all()
    return bits


def test_coefficients_are_the_exponential_series():
    for k in (0.5, 1.0, 3.0):
        c = oracle.taylor_coefficients(30, k)
        assert c[0] == 1.0 and c[1] == k and abs(c[2] - k * k / 2) < 1e-15
        assert abs(sum(c) - math.exp(k)) < 1e-9 * math.exp(k)      # e^k = sum k^d / d!
    assert oracle.taylor_coefficients(0, 7.0) == [1.0]
    assert oracle.taylor_coefficients(3, 0.0) == [1.0, 0.0, 0.0, 0.0]   # at the expansion point only the value counts


def test_order_zero_is_the_identity_bit_for_bit():
    x = synth.normal_bf16(np.random.default_rng(1), (3, 5, 7))
    f, bits = oracle.op_reuse([x], [1.0])
    assert (bits == x).all() and (f == bits_to_f64(x)).all()


def test_polynomial_features_are_forecast_exactly():
    """A feature that moves along p(t) = a + b t + c t^2 with its exact derivatives at t0 is reproduced at t0 + k."""
    a = np.array([[1.0, -2.0, 0.5, 8.0]])
    b = np.array([[0.25, 3.0, -1.0, 0.0]])
    c = np.array([[0.5, -0.125, 2.0, 1.0]])
    t0, k = 2.0, 3.0
    value = a + b * t0 + c * t0 ** 2
    d1 = b + 2 * c * t0
    d2 = 2 * c
    terms = [exact_bf16(value), exact_bf16(d1), exact_bf16(d2)]
    f, bits = oracle.op_reuse(terms, oracle.taylor_coefficients(2, k))
    want = a + b * (t0 + k) + c * (t0 + k) ** 2
    assert (f == want).all()                       # small dyadic numbers: exact in double
    assert (bits == exact_bf16(want)).all()
    # truncating the series at order 1 misses exactly the quadratic remainder c k^2
    f1, _ = oracle.op_reuse(terms[:2], oracle.taylor_coefficients(1, k))
    assert (want - f1 == c * k ** 2).all()


def test_linearity_and_single_rounding():
    rng = np.random.default_rng(2)
    t = [synth.normal_bf16(rng, (64, 33)) for _ in range(3)]
    coef = [1.0, 2.0, 2.0]
    f, bits = oracle.op_reuse(t, coef)
    assert np.allclose(f, sum(cf * bits_to_f64(x) for cf, x in zip(coef, t)), rtol=0, atol=1e-15)
    # rounded once, to the nearest bf16: never further than half a unit in the last place of the result
    back = bits_to_f64(bits)
    ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(f), 1e-30))) - 7)
    assert (np.abs(back - f) <= 0.5 * ulp + 1e-30).all()
    # element-wise: permuting elements permutes results (no cross-talk)
    perm = rng.permutation(64)
    _, bits_p = oracle.op_reuse([x[perm] for x in t], coef)
    assert (bits_p == bits[perm]).all()


def test_attention_with_forecast_composes_the_two_branches():
    w = synth.random_case(11, 1, 2, 256, 64, 64, 64, keep=0.6, cached_frac=0.5)
    rng = np.random.default_rng(3)
    terms = [w.O_cache, synth.normal_bf16(rng, w.Q.shape)]
    coef = oracle.taylor_coefficients(1, 2.0)
    mask = oracle.pack_symbols(w.M_s)
    O, bits = oracle.attention_with_forecast(w.Q, w.K, w.V, w.cache_flags, mask, terms, coef, 64, 64)
    ref, ref_bits = oracle.sparse_attention(w.Q, w.K, w.V, w.cache_flags, mask, w.O_cache, 64, 64)
    rows = np.repeat(w.cache_flags != 0, 64, axis=2)
    assert rows.any() and (~rows).any()
    assert (bits[~rows] == ref_bits[~rows]).all()                                   # computed blocks untouched
    want = bits_to_f64(terms[0]) + 2.0 * bits_to_f64(terms[1])
    assert (O[rows] == want[rows]).all()
    # order 0 falls back to the plain copy of Algorithm 1
    O0, bits0 = oracle.attention_with_forecast(w.Q, w.K, w.V, w.cache_flags, mask, [w.O_cache], [1.0], 64, 64)
    assert (bits0 == ref_bits).all()


def test_finite_difference_refresh_on_polynomial_trajectories():
    """Features sampled every N steps.  Linear motion: one refresh pair gives the exact slope and the forecast is
    exact.  f(t) = t^2: backward differences give slope 3N and curvature 2 after the samples at 0, N, 2N, so the
    second-order forecast k steps on is 4N^2 + 3Nk + k^2 (the true value is (2N + k)^2: the slope lags by N)."""
    N, k = 4.0, 3.0
    a = np.array([[1.0, -2.0, 0.5]])
    b = np.array([[0.25, 3.0, -1.0]])
    terms = [np.zeros((1, 3), dtype=np.uint16) for _ in range(3)]
    n_valid = 0
    for t in (0.0, N, 2 * N):
        terms = oracle.taylor_update(exact_bf16(a + b * t), terms, n_valid, N)
        n_valid = min(n_valid + 1, 3)
    assert (bits_to_f64(terms[1]) == b).all() and (bits_to_f64(terms[2]) == 0).all()
    f, _ = oracle.op_reuse(terms, oracle.taylor_coefficients(2, k))
    assert (f == a + b * (2 * N + k)).all()
    # quadratic
    terms = [np.zeros((1, 1), dtype=np.uint16) for _ in range(3)]
    n_valid = 0
    for t in (0.0, N, 2 * N):
        terms = oracle.taylor_update(exact_bf16(np.array([[t * t]])), terms, n_valid, N)
        n_valid = min(n_valid + 1, 3)
    assert bits_to_f64(terms[0])[0, 0] == 4 * N * N and bits_to_f64(terms[1])[0, 0] == 3 * N and bits_to_f64(terms[2])[0, 0] == 2.0
    f, _ = oracle.op_reuse(terms, oracle.taylor_coefficients(2, k))
    assert f[0, 0] == 4 * N * N + 3 * N * k + k * k


def test_refresh_uses_only_as_many_orders_as_there_were_refreshes():
    rng = np.random.default_rng(9)
    x0, x1 = synth.normal_bf16(rng, (5, 8)), synth.normal_bf16(rng, (5, 8))
    junk = [synth.normal_bf16(rng, (5, 8)) for _ in range(3)]
    first = oracle.taylor_update(x0, junk, 0, 5.0)
    assert (first[0] == x0).all() and (first[1] == 0).all() and (first[2] == 0).all()
    second = oracle.taylor_update(x1, first, 1, 5.0)
    assert (second[0] == x1).all() and (second[2] == 0).all()
    want = (bits_to_f64(x1) - bits_to_f64(x0)) / 5.0
    back = bits_to_f64(second[1])
    assert np.abs(back - want).max() <= np.abs(want).max() * 2.0 ** -8
