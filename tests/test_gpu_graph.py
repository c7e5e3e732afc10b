"""The Dispatch-step chain (GEMM-Q -> attention through a stored plan -> OP_reuse of the cached bias -> GEMM-O)
captured into a HIP graph and replayed: every replay must reproduce the eager result bit for bit.  None of these
entry points allocates or clears memory with a memset once the plan exists, so they can be captured."""
import numpy as np
import pytest
import torch

import paper_2509_25401_amd as pkg
from paper_2509_25401_amd import synth
from gpu_utils import dev, up_bf16, up_u8, down_bits

pytestmark = pytest.mark.gpu


def test_dispatch_chain_replays_bit_identically_from_a_graph():
    rng = np.random.default_rng(synth.BASE_SEED + 400)
    B, H, L, D, C, blk = 1, 4, 1024, 128, 256, 128
    T = L // blk
    X = up_bf16(synth.normal_bf16(rng, (B, L, C)))
    Wq = up_bf16(synth.f32_to_bf16_bits((rng.standard_normal((H * D, C)) / np.sqrt(C)).astype(np.float32)))
    Wo = up_bf16(synth.f32_to_bf16_bits((rng.standard_normal((C, H * D)) / np.sqrt(H * D)).astype(np.float32)))
    K, V, Oc = (up_bf16(synth.normal_bf16(rng, (B, H, L, D))) for _ in range(3))
    Bc = [up_bf16(synth.normal_bf16(rng, (B, L, C))) for _ in range(2)]
    flags_h = (rng.random((B, H, T)) < 0.4).astype(np.uint8)
    M = (rng.random((B, H, T, T)) < 0.6).astype(np.uint8)
    M[..., 0] = 1
    flags, mask = up_u8(flags_h), up_u8(pkg.sparse_attn_pack_mask(M))
    plan = pkg.SparseAttnPlan(flags, mask, B, H, L, blk, blk)
    Q = torch.zeros((B, H, L, D), dtype=torch.bfloat16, device=dev())
    O = torch.zeros_like(Q)
    Out = torch.zeros((B, L, C), dtype=torch.bfloat16, device=dev())
    coef = pkg.sparse_taylor_coefficients(1, 2.0)

    def chain():
        pkg.sparse_gemm_q(X, Wq, None, flags, Q, blk)
        plan.run(Q, K, V, Oc, O)
        pkg.sparse_op_reuse(Bc, coef, Out)
        pkg.sparse_gemm_o(O, Wo, None, flags, 0, Out, Out, blk)

    chain()
    torch.cuda.synchronize()
    want = (down_bits(Q), down_bits(O), down_bits(Out))

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        chain()                                   # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            chain()
    torch.cuda.synchronize()
    for rep in range(3):
        Q.zero_(); O.zero_(); Out.zero_()         # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = (down_bits(Q), down_bits(O), down_bits(Out))
        for name, g, w in zip(("Q", "O", "Out"), got, want):
            assert (g == w).all(), f"replay {rep}: {name} differs from the eager run"
    plan.destroy()
