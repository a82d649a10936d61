"""The forward pass inside a HIP graph: captured once (after a warm-up call has created the context's workspaces),
replayed several times with the program's own eager work and synchronisations in between, every replay checked
against the eager result.  Covers the small-problem path (image-query and text-query rows in one launch) and the
path of one launch after the other."""
import pytest
import torch

from paper_2412_16112_amd import clear_attn as ca
from paper_2412_16112_amd.inputs import make_qkv_shape

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("n_text,gh,gw,r,H", [
    (96, 32, 40, 8, 2),     # few workgroups: image-query and text-query rows in one launch
    (64, 544, 544, 8, 24),  # more than 64 workgroups per CU: one launch after the other
])
def test_forward_replays_from_a_graph(n_text, gh, gw, r, H):
    d = 128
    ctx = ca.ClearAttn(n_text, gh, gw, d, r, ca.CLEAR_BF16)
    Q, K, V = make_qkv_shape(1, H, n_text, gh, gw, d, "bf16", seed=800 + gh, device=DEV)
    O = torch.empty_like(Q)
    try:
        ctx.forward(Q, K, V, O)  # warm-up: allocates the workspace, sets kernel attributes
        torch.cuda.synchronize()
        eager = O.clone()
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream(device=DEV)
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                ctx.forward(Q, K, V, O, stream=side.cuda_stream)
        torch.cuda.synchronize()
        for rep in range(4):
            O.fill_(float("nan"))
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(O, eager), rep
            # eager work of the program between replays, on the same context
            Q2, K2, V2 = make_qkv_shape(1, H, n_text, gh, gw, d, "bf16", seed=900 + rep, device=DEV)
            other = ctx.forward(Q2, K2, V2)
            torch.cuda.synchronize()
            assert torch.isfinite(other.float()).all()
        # new inputs in the captured buffers, replay again
        Q3, K3, V3 = make_qkv_shape(1, H, n_text, gh, gw, d, "bf16", seed=950, device=DEV)
        expect = ctx.forward(Q3, K3, V3)
        Q.copy_(Q3); K.copy_(K3); V.copy_(V3)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(O, expect)
        del graph
    finally:
        torch.cuda.synchronize()
        ctx.destroy()
