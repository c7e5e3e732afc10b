"""CPU oracle of OP_reuse as a Taylor-series forecast (Section 3.3: cached blocks are forecast "via Taylor series
expansion using stored features and their derivatives"; Section 3.4: the cache-then-reuse path is an element-wise
operation of sums and products; Section 3.5: the same operation applied to the cached bias B_c).

TEST INFRASTRUCTURE ONLY.  The operation is the Taylor polynomial written out:
    OP_reuse(terms; k) = sum over d = 0..order of  k^d / d!  *  terms[d]
with terms[0] the stored feature, terms[d] its stored d-th derivative per step, and k the number of steps since
the features were stored.  order 0 is the identity (direct reuse).  How the derivatives are estimated at Update
steps is the caller's business (the paper does not say); the oracle and the kernels take them as inputs.
Arithmetic is IEEE double on exactly widened bf16 inputs, the result is rounded once to bf16.
"""
import math

import numpy as np

from .gemm_q import _widen, _narrow


def taylor_coefficients(order, k):
    """[k^d / d! for d = 0..order]: the weights of the Taylor polynomial k steps away from the expansion point."""
    return [float(k) ** d / math.factorial(d) for d in range(order + 1)]


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
