"""Backward pass through the C ABI against the fp64 oracle (oracle/clear_oracle.c, backward functions)."""
import numpy as np
import pytest
import torch

from oracle import clear_oracle as orc
from paper_2412_16112_amd import clear_attn as ca
from paper_2412_16112_amd.inputs import make_qkv_shape
from tests.parity_util import TOL, error_metrics

pytestmark = pytest.mark.gpu

# Gradients are sums of products of bf16-rounded factors (P and dS are rounded to bf16 before the matrix
# instruction, like P in the forward pass) accumulated in fp32 and rounded to bf16 once: the same error
# model as the forward output, on values of a different size.  The bar is the forward bar made relative:
# max-abs error <= 2e-2 of the largest reference magnitude, relative RMS <= 1e-2.
def check_grad(name, got, ref):
    max_abs, rel_rms = error_metrics(got, ref)
    scale = float(np.abs(ref).max())
    assert np.isfinite(got).all(), name
    assert max_abs <= TOL["bf16"][0] * max(scale, 1e-30) and rel_rms <= TOL["bf16"][1], (name, max_abs, scale, rel_rms)


def run_case(n_text, gridH, gridW, r, H, seed, q_scale=1.0, B=1):
    d = 128
    Q, K, V = make_qkv_shape(B, H, n_text, gridH, gridW, d, "bf16", seed=seed, device="cuda:0", q_scale=q_scale)
    g = torch.Generator(device="cuda:0").manual_seed(seed + 1000)
    dO = torch.randn(Q.shape, generator=g, device="cuda:0", dtype=torch.float32).to(torch.bfloat16)
    ctx = ca.ClearAttn(n_text, gridH, gridW, d, r, ca.CLEAR_BF16)
    try:
        O, lse = ctx.forward_lse(Q, K, V)
        dQ, dK, dV = ctx.backward(Q, K, V, O, dO, lse)
        torch.cuda.synchronize()
    finally:
        ctx.destroy()
    return Q, K, V, dO, O, lse, dQ, dK, dV


CASES = [
    # n_text, gridH, gridW, r, H
    (37, 20, 24, 5, 2),      # ragged text tile, ragged grid tiles
    (0, 17, 33, 4, 1),       # no text
    (64, 16, 16, 1, 1),      # r = 1: an image token sees the text and itself
    (16, 12, 12, 40, 1),     # r beyond the diagonal: full attention
    (200, 48, 40, 16, 1),    # several tile rows and columns, r = 16
]


@pytest.mark.parametrize("n_text,gridH,gridW,r,H", CASES)
def test_backward_all_rows(n_text, gridH, gridW, r, H):
    Q, K, V, dO, O, lse, dQ, dK, dV = run_case(n_text, gridH, gridW, r, H, seed=300 + r)
    for h in range(H):
        q, k, v, g = (t[0, h].float().cpu().numpy() for t in (Q, K, V, dO))
        rQ, rK, rV = orc.backward(q, k, v, g, n_text, gridH, gridW, r)
        check_grad("dQ", dQ[0, h].float().cpu().numpy(), rQ)
        check_grad("dK", dK[0, h].float().cpu().numpy(), rK)
        check_grad("dV", dV[0, h].float().cpu().numpy(), rV)


def test_backward_batch_of_two():
    n_text, gridH, gridW, r, H = 40, 20, 28, 4, 3
    Q, K, V, dO, O, lse, dQ, dK, dV = run_case(n_text, gridH, gridW, r, H, seed=71, B=2)
    for b, h in ((0, 0), (1, 2)):
        q, k, v, g = (t[b, h].float().cpu().numpy() for t in (Q, K, V, dO))
        rQ, rK, rV = orc.backward(q, k, v, g, n_text, gridH, gridW, r)
        check_grad("dQ", dQ[b, h].float().cpu().numpy(), rQ)
        check_grad("dK", dK[b, h].float().cpu().numpy(), rK)
        check_grad("dV", dV[b, h].float().cpu().numpy(), rV)


def test_forward_lse_is_the_log_of_the_softmax_denominator():
    n_text, gridH, gridW, r = 37, 20, 24, 5
    Q, K, V, dO, O, lse, *_ = run_case(n_text, gridH, gridW, r, 1, seed=77, q_scale=2.0)
    q, k, v = (t[0, 0].float().cpu().numpy() for t in (Q, K, V))
    N = q.shape[0]
    _, m, l, _ = orc.attention_rows(q, k, v, np.arange(N), n_text, gridH, gridW, r, return_stats=True)
    np.testing.assert_allclose(lse[0, 0].cpu().numpy(), m + np.log(l), rtol=0, atol=2e-3)


def test_backward_flux_1024_sampled():
    """64 x 64 grid + 512 text tokens, r = 16 (the 1024^2 shape), one head: sampled rows and columns."""
    n_text, gridH, gridW, r = 512, 64, 64, 16
    Q, K, V, dO, O, lse, dQ, dK, dV = run_case(n_text, gridH, gridW, r, 1, seed=9)
    q, k, v, g = (t[0, 0].float().cpu().numpy() for t in (Q, K, V, dO))
    rng = np.random.default_rng(3)
    N = q.shape[0]
    rows = np.unique(np.concatenate([[0, 1, 255, 256, 511, 512, 513, 512 + 63, 512 + 64, 512 + 15 * 64 + 15, 512 + 16 * 64 + 16, N - 1],
                                     rng.integers(0, N, size=200)]))
    check_grad("dQ", dQ[0, 0].float().cpu().numpy()[rows], orc.backward_dq_rows(q, k, v, g, rows, n_text, gridH, gridW, r))
    cols = np.unique(np.concatenate([[0, 511, 512, 512 + 63, N - 1], rng.integers(0, n_text, size=6), rng.integers(n_text, N, size=60)]))
    rK, rV = orc.backward_dkv_cols(q, k, v, g, cols, n_text, gridH, gridW, r)
    check_grad("dK", dK[0, 0].float().cpu().numpy()[cols], rK)
    check_grad("dV", dV[0, 0].float().cpu().numpy()[cols], rV)


@pytest.mark.slow
def test_backward_flux_2048_sampled():
    """128 x 128 grid + 512 text tokens, r = 16 (the 2048^2 shape), one head: sampled query rows, image-key
    columns at corners, borders and tile boundaries, and two text-key columns (every query row feeds those)."""
    n_text, gridH, gridW, r = 512, 128, 128, 16
    Q, K, V, dO, O, lse, dQ, dK, dV = run_case(n_text, gridH, gridW, r, 1, seed=19, q_scale=1.5)
    q, k, v, g = (t[0, 0].float().cpu().numpy() for t in (Q, K, V, dO))
    rng = np.random.default_rng(5)
    N = q.shape[0]
    img = lambda y, x: n_text + y * gridW + x
    rows = np.unique(np.concatenate([[0, 255, 256, 511, img(0, 0), img(0, 127), img(127, 0), img(127, 127), img(15, 15), img(16, 16), img(63, 64)],
                                     rng.integers(0, N, size=300)]))
    check_grad("dQ", dQ[0, 0].float().cpu().numpy()[rows], orc.backward_dq_rows(q, k, v, g, rows, n_text, gridH, gridW, r))
    cols = np.unique(np.concatenate([[3, 500, img(0, 0), img(0, 127), img(127, 127), img(15, 16), img(16, 15), img(64, 63), img(112, 8)],
                                     rng.integers(n_text, N, size=40)]))
    rK, rV = orc.backward_dkv_cols(q, k, v, g, cols, n_text, gridH, gridW, r)
    check_grad("dK", dK[0, 0].float().cpu().numpy()[cols], rK)
    check_grad("dV", dV[0, 0].float().cpu().numpy()[cols], rV)


def test_backward_wide_grid_sampled():
    """A grid more than 16 row tiles wide (400 columns): the row tiles are dealt to the workgroups in 2 x 16 blocks."""
    n_text, gridH, gridW, r, H = 48, 40, 400, 8, 2
    Q, K, V, dO, O, lse, dQ, dK, dV = run_case(n_text, gridH, gridW, r, H, seed=39)
    rng = np.random.default_rng(11)
    N = Q.shape[2]
    img = lambda y, x: n_text + y * gridW + x
    for h in range(H):
        q, k, v, g = (t[0, h].float().cpu().numpy() for t in (Q, K, V, dO))
        rows = np.unique(np.concatenate([[0, 47, img(0, 0), img(0, 399), img(39, 0), img(39, 399), img(15, 255), img(16, 256), img(31, 271), img(32, 272)],
                                         rng.integers(0, N, size=150)]))
        check_grad("dQ", dQ[0, h].float().cpu().numpy()[rows], orc.backward_dq_rows(q, k, v, g, rows, n_text, gridH, gridW, r))
        cols = np.unique(np.concatenate([[7, img(0, 0), img(39, 399), img(16, 255), img(15, 256), img(33, 383), img(2, 384)], rng.integers(n_text, N, size=40)]))
        rK, rV = orc.backward_dkv_cols(q, k, v, g, cols, n_text, gridH, gridW, r)
        check_grad("dK", dK[0, h].float().cpu().numpy()[cols], rK)
        check_grad("dV", dV[0, h].float().cpu().numpy()[cols], rV)


@pytest.mark.slow
def test_backward_many_workgroups_sampled():
    """96 heads on a 224 x 224 grid: more than 64 image workgroups per CU, where the backward pass sends its four
    kernels out one after the other and the forward pass its two (smaller problems share one launch).  Sampled rows
    and columns of the first and the last head."""
    n_text, gridH, gridW, r, H = 64, 224, 224, 8, 96
    Q, K, V, dO, O, lse, dQ, dK, dV = run_case(n_text, gridH, gridW, r, H, seed=29)
    rng = np.random.default_rng(7)
    N = Q.shape[2]
    img = lambda y, x: n_text + y * gridW + x
    for h in (0, H - 1):
        q, k, v, g = (t[0, h].float().cpu().numpy() for t in (Q, K, V, dO))
        rows = np.unique(np.concatenate([[0, 63, img(0, 0), img(0, 223), img(223, 0), img(223, 223), img(15, 16), img(111, 112)],
                                         rng.integers(0, N, size=120)]))
        ref_o = orc.attention_rows(q, k, v, rows, n_text, gridH, gridW, r)
        max_abs, rel_rms = error_metrics(O[0, h].float().cpu().numpy()[rows], ref_o)
        assert max_abs <= TOL["bf16"][0] and rel_rms <= TOL["bf16"][1], (h, max_abs, rel_rms)
        check_grad("dQ", dQ[0, h].float().cpu().numpy()[rows], orc.backward_dq_rows(q, k, v, g, rows, n_text, gridH, gridW, r))
        cols = np.unique(np.concatenate([[5, img(0, 0), img(223, 223), img(7, 8), img(112, 111)], rng.integers(n_text, N, size=30)]))
        rK, rV = orc.backward_dkv_cols(q, k, v, g, cols, n_text, gridH, gridW, r)
        check_grad("dK", dK[0, h].float().cpu().numpy()[cols], rK)
        check_grad("dV", dV[0, h].float().cpu().numpy()[cols], rV)


@pytest.mark.slow
def test_backward_many_workgroups_without_text():
    """The same launch shape with no text token: delta, which the dQ kernel of the image rows forms on its way for the
    dK / dV kernel launched after it, then comes from that one kernel alone."""
    n_text, gridH, gridW, r, H = 0, 224, 224, 8, 96
    Q, K, V, dO, O, lse, dQ, dK, dV = run_case(n_text, gridH, gridW, r, H, seed=31)
    rng = np.random.default_rng(8)
    N = Q.shape[2]
    for h in (0, H // 2, H - 1):
        q, k, v, g = (t[0, h].float().cpu().numpy() for t in (Q, K, V, dO))
        rows = np.unique(np.concatenate([[0, 223, N - 224, N - 1], rng.integers(0, N, size=60)]))
        check_grad("dQ", dQ[0, h].float().cpu().numpy()[rows], orc.backward_dq_rows(q, k, v, g, rows, n_text, gridH, gridW, r))
        cols = np.unique(np.concatenate([[0, N - 1], rng.integers(0, N, size=30)]))
        rK, rV = orc.backward_dkv_cols(q, k, v, g, cols, n_text, gridH, gridW, r)
        check_grad("dK", dK[0, h].float().cpu().numpy()[cols], rK)
        check_grad("dV", dV[0, h].float().cpu().numpy()[cols], rV)


@pytest.mark.slow
def test_backward_many_workgroups_strided_mask():
    """The strided mask (r * r residue classes, each a dense problem of its own) at a size where the four kernels go out
    one after the other: 128 heads x 16 classes x 9 row tiles."""
    n_text, gridH, gridW, r, H, layer, d = 40, 160, 160, 4, 128, 6, 128
    Q, K, V = make_qkv_shape(1, H, n_text, gridH, gridW, d, "bf16", seed=33, device="cuda:0")
    gen = torch.Generator(device="cuda:0").manual_seed(34)
    dO = torch.randn(Q.shape, generator=gen, device="cuda:0", dtype=torch.float32).to(torch.bfloat16)
    ctx = ca.ClearAttn(n_text, gridH, gridW, d, r, ca.CLEAR_BF16, orc.MASK_STRIDED, layer)  # (the two sides number the mask kinds alike)
    try:
        O, lse = ctx.forward_lse(Q, K, V)
        dQ, dK, dV = ctx.backward(Q, K, V, O, dO, lse)
        torch.cuda.synchronize()
    finally:
        ctx.destroy()
    rng = np.random.default_rng(9)
    N = Q.shape[2]
    with orc.mask_kind(orc.MASK_STRIDED, layer):
        for h in (0, H - 1):
            q, k, v, g = (t[0, h].float().cpu().numpy() for t in (Q, K, V, dO))
            rows = np.unique(np.concatenate([[0, n_text - 1, n_text, N - 1], rng.integers(0, N, size=60)]))
            check_grad("dQ", dQ[0, h].float().cpu().numpy()[rows], orc.backward_dq_rows(q, k, v, g, rows, n_text, gridH, gridW, r))
            cols = np.unique(np.concatenate([[3, n_text, N - 1], rng.integers(0, N, size=30)]))
            rK, rV = orc.backward_dkv_cols(q, k, v, g, cols, n_text, gridH, gridW, r)
            check_grad("dK", dK[0, h].float().cpu().numpy()[cols], rK)
            check_grad("dV", dV[0, h].float().cpu().numpy()[cols], rV)


def test_backward_rejects_bad_arguments():
    n_text, gridH, gridW, r, d = 8, 16, 16, 4, 128
    Q, K, V = make_qkv_shape(1, 1, n_text, gridH, gridW, d, "bf16", seed=1, device="cuda:0")
    ctx = ca.ClearAttn(n_text, gridH, gridW, d, r, ca.CLEAR_BF16)
    try:
        O, lse = ctx.forward_lse(Q, K, V)
        L = ca.lib()
        import ctypes
        vp = ctypes.c_void_p
        args = [ctx._ctx, Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), O.data_ptr(), lse.data_ptr()]
        # dQ aliasing an input
        rc = L.clear_attn_backward(*args, Q.data_ptr(), torch.empty_like(Q).data_ptr(), torch.empty_like(Q).data_ptr(), 1, 1, n_text, gridH, gridW, d, r, vp(0))
        assert rc == ca.CLEAR_ERR_INVALID_ARG
        a, b, c = torch.empty_like(Q), torch.empty_like(Q), torch.empty_like(Q)
        rc = L.clear_attn_backward(*args, a.data_ptr(), b.data_ptr(), c.data_ptr(), 1, 1, n_text, gridH, gridW + 1, d, r, vp(0))
        assert rc == ca.CLEAR_ERR_MISMATCH
        rc = L.clear_attn_backward(*args[:6], None, a.data_ptr(), b.data_ptr(), c.data_ptr(), 1, 1, n_text, gridH, gridW, d, r, vp(0))
        assert rc == ca.CLEAR_ERR_INVALID_ARG
    finally:
        ctx.destroy()
    # fp32 contexts have no backward pass
    ctx = ca.ClearAttn(8, 16, 16, 64, 4, ca.CLEAR_F32)
    try:
        with pytest.raises(ca.ClearAttnError) as e:
            ca._check(ca.lib().clear_attn_reserve_backward(ctx._ctx, 1), ctx._ctx)
        assert e.value.status == ca.CLEAR_ERR_UNSUPPORTED
    finally:
        ctx.destroy()


def test_autograd_function_matches_the_oracle():
    from paper_2412_16112_amd.autograd import clear_attention, clear_context_cache
    n_text, gridH, gridW, r, d = 20, 18, 21, 6, 128
    Q, K, V = make_qkv_shape(1, 2, n_text, gridH, gridW, d, "bf16", seed=55, device="cuda:0")
    Q.requires_grad_(True), K.requires_grad_(True), V.requires_grad_(True)
    g = torch.Generator(device="cuda:0").manual_seed(56)
    W = torch.randn(Q.shape, generator=g, device="cuda:0", dtype=torch.float32).to(torch.bfloat16)
    try:
        O = clear_attention(Q, K, V, n_text, gridH, gridW, r)
        (O.float() * W.float()).sum().backward()
        torch.cuda.synchronize()
        with torch.no_grad():
            O2 = clear_attention(Q.detach(), K.detach(), V.detach(), n_text, gridH, gridW, r)
        assert torch.equal(O, O2)  # the forward with and without the statistics output gives the same bits
    finally:
        clear_context_cache()
    for h in range(2):
        q, k, v, w = (t[0, h].detach().float().cpu().numpy() for t in (Q, K, V, W))
        rQ, rK, rV = orc.backward(q, k, v, w, n_text, gridH, gridW, r)
        check_grad("dQ", Q.grad[0, h].float().cpu().numpy(), rQ)
        check_grad("dK", K.grad[0, h].float().cpu().numpy(), rK)
        check_grad("dV", V.grad[0, h].float().cpu().numpy(), rV)
