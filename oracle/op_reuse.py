"""CPU oracle of OP_reuse as a Taylor-series forecast (Section 3.3: cached blocks are forecast by a Taylor
expansion around the step at which the feature and its derivatives were stored; Section 3.4: the cache-then-reuse path is an element-wise
operation of sums and products; Section 3.5: the same operation applied to the cached bias B_c).

TEST INFRASTRUCTURE ONLY.  The operation is the Taylor polynomial written out:
    OP_reuse(terms; k) = sum over d = 0..order of  k^d / d!  *  terms[d]
with terms[0] the stored feature, terms[d] its stored d-th derivative per step, and k the number of steps since
the features were stored.  order 0 is the identity (direct reuse).  How the derivatives are estimated at Update
steps is not stated in the paper; `taylor_update` restates what the cited forecasting method does (backward finite
differences), and `op_reuse` itself takes the terms as inputs whatever their origin.
Arithmetic is IEEE double on exactly widened bf16 inputs, the result is rounded once to bf16.
"""
import math

import numpy as np

from .gemm_q import _widen, _narrow


def taylor_coefficients(order, k):
    """[k^d / d! for d = 0..order]: the weights of the Taylor polynomial k steps away from the expansion point."""
    return [float(k) ** d / math.factorial(d) for d in range(order + 1)]


def taylor_update(fresh, terms, n_valid, interval):
    """Refresh of the stored terms at an Update step by backward finite differences over the Update interval --
    how the forecasting method the paper cites estimates the derivatives (the paper itself does not say):
        new[0] = fresh,   new[d] = (new[d-1] - old[d-1]) / interval   for 1 <= d <= n_valid,   new[d] = 0 beyond,
    where n_valid is the number of stored terms that were valid before this refresh (0 at the very first one: a
    d-th difference needs d earlier refreshes).  Every term is stored in bf16; the differences are taken between
    stored (rounded) values in double and rounded once.  fresh, terms[d]: uint16 bf16 bits of one shape.
    Returns the list of new term bits."""
    if not (0 <= n_valid <= len(terms)) or interval <= 0:
        raise ValueError("0 <= n_valid <= number of terms, interval > 0")
    new = [np.array(fresh, dtype=np.uint16, copy=True)]
    for d in range(1, len(terms)):
        if d <= n_valid:
            new.append(_narrow((_widen(new[d - 1]) - _widen(terms[d - 1])) / float(interval)))
        else:
            new.append(np.zeros_like(new[0]))
    return new


def op_reuse(terms, coef):
    """terms: list of uint16 bf16-bit arrays of one shape; coef: one weight per term.  Returns (fp64, bf16 bits)."""
    if len(terms) != len(coef) or not terms:
        raise ValueError("one coefficient per term")
    acc = np.zeros(np.asarray(terms[0]).shape, dtype=np.float64)
    for t, c in zip(terms, coef):
        acc += float(c) * _widen(t)
    return acc, _narrow(acc)


def attention_with_forecast(Q, K, V, cache_flags, kv_mask, terms, coef, block_q, block_k):
    """Algorithm 1 with OP_reuse = the forecast above: computed blocks as in `sparse_attention`, cached blocks
    (cache_flags != 0) = op_reuse of the same rows of the stored terms.  Returns (O_f64, O_bits)."""
    from .reference import sparse_attention
    O, O_bits = sparse_attention(Q, K, V, cache_flags, kv_mask, None, block_q, block_k)
    if cache_flags is not None:
        f, fb = op_reuse(terms, coef)
        rows = np.repeat(np.asarray(cache_flags) != 0, block_q, axis=2)[:, :, :O.shape[2]]
        O[rows] = f[rows]
        O_bits[rows] = fb[rows]
    return O, O_bits
