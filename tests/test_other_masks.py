"""The other local masks (square window, Swin windows) through the same scheduler: oracle pins (CPU) and
parity of the HIP path (GPU)."""
import numpy as np
import pytest
import torch

from oracle import clear_oracle as orc
from paper_2412_16112_amd import clear_attn as ca
from paper_2412_16112_amd.inputs import make_qkv_shape
from tests.parity_util import TOL, error_metrics

KINDS = [(orc.MASK_SQUARE, 0), (orc.MASK_SWIN, 0), (orc.MASK_SWIN, 3)]


def _mask_by_definition(kind, shift, n_text, gridH, gridW, r):
    """The mask written out from its definition with numpy broadcasting (independent of the C oracle)."""
    N = n_text + gridH * gridW
    M = np.ones((N, N), dtype=bool)
    y, x = np.divmod(np.arange(gridH * gridW), gridW)
    if kind == orc.MASK_SQUARE:
        img = (np.abs(y[:, None] - y[None, :]) < r) & (np.abs(x[:, None] - x[None, :]) < r)
    else:
        wy, wx = (y + shift) // r, (x + shift) // r
        img = (wy[:, None] == wy[None, :]) & (wx[:, None] == wx[None, :])
    M[n_text:, n_text:] = img
    return M


@pytest.mark.parametrize("kind,shift", KINDS)
def test_oracle_masks_match_their_definitions_and_the_closed_form_counts(kind, shift):
    for n_text, gridH, gridW, r in [(3, 7, 9, 4), (0, 10, 6, 4), (5, 4, 4, 8), (2, 9, 13, 5)]:
        if kind == orc.MASK_SWIN and shift >= r:
            continue
        with orc.mask_kind(kind, shift):
            M = orc.mask_dense(n_text, gridH, gridW, r).astype(bool)
            total = orc.mask_count(n_text, gridH, gridW, r)
        ref = _mask_by_definition(kind, shift, n_text, gridH, gridW, r)
        assert (M == ref).all()
        assert (M == M.T).all()
        assert total == int(ref.sum()) == ca.clear_attn_mask_count_masked(n_text, gridH, gridW, r, kind, shift)
    # outside the context manager the disc is back
    assert orc.mask_count(0, 5, 5, 2) == ca.clear_attn_mask_count(0, 5, 5, 2)


def test_swin_without_shift_on_aligned_grid_is_block_diagonal_attention():
    # 8 x 8 grid, windows of 4: four independent windows of 16 tokens, each a full attention of its own
    gridH = gridW = 8
    r, d = 4, 8
    rng = np.random.default_rng(1)
    Q, K, V = (rng.standard_normal((gridH * gridW, d)) for _ in range(3))
    with orc.mask_kind(orc.MASK_SWIN, 0):
        O = orc.attention_rows(Q, K, V, np.arange(gridH * gridW), 0, gridH, gridW, r)
    for wy in range(2):
        for wx in range(2):
            idx = np.array([(wy * 4 + a) * gridW + wx * 4 + b for a in range(4) for b in range(4)])
            q, k, v = (torch.tensor(t[idx]) for t in (Q, K, V))
            ref = torch.nn.functional.scaled_dot_product_attention(q[None], k[None], v[None])[0].numpy()
            np.testing.assert_allclose(O[idx], ref, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("kind,shift", KINDS)
def test_host_schedule_is_bit_exact_with_the_brute_force(kind, shift):
    for gridH, gridW, r, tiles in [(40, 56, 8, (16, 16, 8, 8)), (33, 17, 5, (16, 16, 8, 8)), (64, 64, 16, (16, 16, 8, 8)),
                                   (30, 30, 7, (8, 16, 4, 8)), (9, 70, 32, (16, 16, 8, 8))]:
        s = (r // 2) if (kind == orc.MASK_SWIN and shift) else 0
        got = ca.clear_attn_schedule_host_masked(gridH, gridW, r, kind, s, *tiles)
        with orc.mask_kind(kind, s):
            ref = orc.tile_schedule(gridH, gridW, r, *tiles)
        for a, b in zip(got, ref):
            assert a.shape == b.shape and (a == b).all(), (kind, s, gridH, gridW, r)


@pytest.mark.gpu
@pytest.mark.parametrize("kind,shift", KINDS)
@pytest.mark.parametrize("dtype,n_text,gridH,gridW,r,H", [
    ("f32", 8, 16, 16, 4, 1),
    ("f32", 5, 23, 9, 6, 2),
    ("bf16", 37, 40, 24, 8, 2),
    ("bf16", 0, 33, 50, 16, 1),
    ("bf16", 64, 48, 48, 16, 1),
])
def test_gpu_forward_other_masks(kind, shift, dtype, n_text, gridH, gridW, r, H):
    d = 128 if dtype == "bf16" else 64
    s = (r // 2) if (kind == orc.MASK_SWIN and shift) else 0
    Q, K, V = make_qkv_shape(1, H, n_text, gridH, gridW, d, dtype, seed=400 + r, device="cuda:0")
    ctx = ca.ClearAttn(n_text, gridH, gridW, d, r, ca._dtype_code(Q), mask_kind=kind, shift=s)
    try:
        O = ctx.forward(Q, K, V)
        torch.cuda.synchronize()
        # the context's schedule against the brute force over the element mask
        row_ptr, col_idx, flags = ctx.schedule_copy()
        qth, qtw, kth, ktw, *_ = ctx.schedule_size()
        with orc.mask_kind(kind, s):
            rp, ci, fl = orc.tile_schedule(gridH, gridW, r, qth, qtw, kth, ktw)
        assert (row_ptr == rp).all() and (col_idx == ci).all() and (flags == fl).all()
    finally:
        ctx.destroy()
    with orc.mask_kind(kind, s):
        ref = orc.attention(Q.float().cpu().numpy(), K.float().cpu().numpy(), V.float().cpu().numpy(), n_text, gridH, gridW, r)
    max_abs, rel_rms = error_metrics(O.float().cpu().numpy(), ref)
    assert max_abs <= TOL[dtype][0] and rel_rms <= TOL[dtype][1], (max_abs, rel_rms)


@pytest.mark.gpu
@pytest.mark.parametrize("kind,shift", KINDS)
def test_gpu_backward_other_masks(kind, shift):
    n_text, gridH, gridW, r, d = 37, 40, 24, 8, 128
    s = (r // 2) if (kind == orc.MASK_SWIN and shift) else 0
    Q, K, V = make_qkv_shape(1, 1, n_text, gridH, gridW, d, "bf16", seed=31, device="cuda:0")
    g = torch.Generator(device="cuda:0").manual_seed(32)
    dO = torch.randn(Q.shape, generator=g, device="cuda:0", dtype=torch.float32).to(torch.bfloat16)
    ctx = ca.ClearAttn(n_text, gridH, gridW, d, r, ca.CLEAR_BF16, mask_kind=kind, shift=s)
    try:
        O, lse = ctx.forward_lse(Q, K, V)
        dQ, dK, dV = ctx.backward(Q, K, V, O, dO, lse)
        torch.cuda.synchronize()
    finally:
        ctx.destroy()
    q, k, v, go = (t[0, 0].float().cpu().numpy() for t in (Q, K, V, dO))
    with orc.mask_kind(kind, s):
        rQ, rK, rV = orc.backward(q, k, v, go, n_text, gridH, gridW, r)
    for name, got, ref in (("dQ", dQ, rQ), ("dK", dK, rK), ("dV", dV, rV)):
        max_abs, rel_rms = error_metrics(got[0, 0].float().cpu().numpy(), ref)
        assert max_abs <= TOL["bf16"][0] * np.abs(ref).max() and rel_rms <= TOL["bf16"][1], (name, max_abs, rel_rms)
