"""CPU oracle of the sparse output projection (GEMM-O, Section 3.5, Observation 3 / Equations 3-4).

TEST INFRASTRUCTURE ONLY.  Equation 3 splits the output projection of a token block i over the heads
whose attention output is computed at this step (set H_i) and the heads whose output is reused from
the cache:  Out_i = sum_{h not in H_i} O_i^h W^h  +  sum_{h in H_i} O_i^h W^h.  With OP_reuse the
identity (Equation 4) the first sum does not change between Update steps and is kept as the cached
bias B_c.  One function covers both stages of the paper's GEMM-O:
    stage 1 (Update step):   B_c[i] = sum over heads WITH the cache flag set   (select = 1, no addend)
    stage 2 (every step):    Out[i] = addend[i] + bias + sum over heads with the flag CLEAR (select = 0)
Arithmetic is IEEE double on exactly widened bf16 inputs; the library matmul is the only primitive.
"""
import numpy as np

from .gemm_q import _widen, _narrow


def gemm_o(O, W, bias, cache_flags, select, addend, block_q):
    """O: uint16 bf16 bits [B, H, L, D] (attention output); W: [C_out, H*D] (one row per output feature);
    bias: [C_out] or None; cache_flags: uint8 [B, H, L/block_q] or None (None = no head is cached);
    select: 0 -> sum over heads whose flag is clear, 1 -> sum over heads whose flag is set;
    addend: uint16 bf16 bits [B, L, C_out] or None (the cached bias B_c in stage 2).
    Returns (Out_f64, Out_bits) of shape [B, L, C_out].
    """
    O = np.ascontiguousarray(O, dtype=np.uint16)
    W = np.ascontiguousarray(W, dtype=np.uint16)
    B, H, L, D = O.shape
    C_out = W.shape[0]
    if W.shape != (C_out, H * D):
        raise ValueError("W must be [C_out, H*D]")
    Tq = -(-L // block_q)      # Definition 1 counts ceil(L / b) blocks: the last token block may be short
    Of, Wf = _widen(O), _widen(W)
    out = np.zeros((B, L, C_out), dtype=np.float64)
    for b in range(B):
        for i in range(Tq):
            rows = slice(i * block_q, (i + 1) * block_q)
            for h in range(H):
                flag = 0 if cache_flags is None else int(cache_flags[b, h, i] != 0)
                if flag != select:
                    continue
                out[b, rows] += Of[b, h, rows] @ Wf[:, h * D:(h + 1) * D].T
    if addend is not None:
        out += _widen(addend)
    if bias is not None:
        out += _widen(bias)[None, None, :]
    return out, _narrow(out)


def gemm_o_reuse(O, W, bias, cache_flags, terms, coef, block_q):
    """Stage 2 at a Dispatch step as Section 3.5 words it, "output initialised by OP_reuse(B_c)" and then the heads
    that were really computed accumulated onto it:  Out = OP_reuse(terms of B_c) + bias + sum over heads with the flag
    clear.  OP_reuse is the Taylor sum of op_reuse.op_reuse (whose result is a stored bf16 tensor, rounded once, as
    the cached bias itself is); it then plays the part of the addend of gemm_o."""
    from .op_reuse import op_reuse
    _, forecast_bits = op_reuse(terms, coef)
    return gemm_o(O, W, bias, cache_flags, 0, forecast_bits, block_q)


def reduced_heads(cache_flags, select, B, H, Tq):
    """Number of (b, i, h) reduction segments a call with this selection visits."""
    if cache_flags is None:
        return B * H * Tq if select == 0 else 0
    f = np.asarray(cache_flags) != 0
    return int(f.sum()) if select == 1 else int((~f).sum())


def speedup_model(N, s):
    """Theoretical GEMM-O speed-up over N steps at cached fraction s (appendix "GEMM-O Speedup Metrics"):
    one Update step does the whole projection, the other N-1 steps only the (1-s) computed part."""
    return N / (1.0 + (N - 1) * (1.0 - s))
