"""Strided attention (the sparse mask of the paper's appendix on compared attentions): oracle pins (CPU) and
parity of the HIP path (GPU)."""
import numpy as np
import pytest
import torch

from oracle import clear_oracle as orc
from paper_2412_16112_amd import clear_attn as ca
from paper_2412_16112_amd.inputs import make_qkv_shape
from tests.parity_util import TOL, error_metrics


def strided_by_definition(n_text, gridH, gridW, r, layer):
    """The mask from its definition with numpy broadcasting (independent of the C oracle)."""
    N = n_text + gridH * gridW
    M = np.ones((N, N), dtype=bool)
    y, x = np.divmod(np.arange(gridH * gridW), gridW)
    rx, ry = layer % r, (layer // r) % r
    # offset = key - query; numpy's % gives the non-negative remainder
    M[n_text:, n_text:] = ((x[None, :] - x[:, None]) % r == rx) & ((y[None, :] - y[:, None]) % r == ry)
    return M


@pytest.mark.parametrize("n_text,gridH,gridW,r,layer", [(3, 8, 12, 4, 0), (3, 8, 12, 4, 6), (0, 10, 7, 3, 5), (2, 9, 13, 5, 24),
                                                          (2, 9, 13, 5, 27), (4, 6, 6, 8, 9)])
def test_oracle_mask_matches_the_definition_and_the_closed_form_count(n_text, gridH, gridW, r, layer):
    with orc.mask_kind(orc.MASK_STRIDED, layer):
        M = orc.mask_dense(n_text, gridH, gridW, r).astype(bool)
        total = orc.mask_count(n_text, gridH, gridW, r)
    ref = strided_by_definition(n_text, gridH, gridW, r, layer)
    assert (M == ref).all()
    # closed form: a query in column residue a sees the columns of residue (a + r_x) % r, likewise for rows
    rx, ry = layer % r, (layer // r) % r
    cols = np.bincount(np.arange(gridW) % r, minlength=r)
    rows = np.bincount(np.arange(gridH) % r, minlength=r)
    img = sum(int(cols[a] * cols[(a + rx) % r]) for a in range(r)) * sum(int(rows[b] * rows[(b + ry) % r]) for b in range(r))
    N = n_text + gridH * gridW
    assert total == N * N - (gridH * gridW) ** 2 + img == int(ref.sum())
    # each image query sees one key per r x r cell at most: never more than ceil(H/r) * ceil(W/r) image keys
    assert (M[n_text:, n_text:].sum(1) <= -(-gridH // r) * -(-gridW // r)).all()


def test_layers_cover_every_offset_once():
    """Over layers 0 .. r^2 - 1 every image key is attended by every image query exactly once."""
    n_text, gridH, gridW, r = 0, 6, 9, 3
    acc = np.zeros((gridH * gridW, gridH * gridW), dtype=int)
    for layer in range(r * r):
        with orc.mask_kind(orc.MASK_STRIDED, layer):
            acc += orc.mask_dense(n_text, gridH, gridW, r)
    assert (acc == 1).all()


def test_strided_attention_is_dense_attention_on_the_residue_classes():
    """Gathering the tokens by (y % r, x % r) turns the mask into full attention between one query class and
    one key class (plus the text keys): checked against the library's dense SDPA class by class."""
    n_text, gridH, gridW, r, d, layer = 3, 8, 12, 4, 8, 6
    rx, ry = layer % r, (layer // r) % r
    rng = np.random.default_rng(2)
    N = n_text + gridH * gridW
    Q, K, V = (rng.standard_normal((N, d)) for _ in range(3))
    with orc.mask_kind(orc.MASK_STRIDED, layer):
        O = orc.attention_rows(Q, K, V, np.arange(N), n_text, gridH, gridW, r)
    y, x = np.divmod(np.arange(gridH * gridW), gridW)
    text = np.arange(n_text)
    for b in range(r):
        for a in range(r):
            qi = n_text + np.nonzero((y % r == b) & (x % r == a))[0]
            ki = np.concatenate([text, n_text + np.nonzero((y % r == (b + ry) % r) & (x % r == (a + rx) % r))[0]])
            ref = torch.nn.functional.scaled_dot_product_attention(torch.tensor(Q[qi])[None], torch.tensor(K[ki])[None], torch.tensor(V[ki])[None])[0].numpy()
            np.testing.assert_allclose(O[qi], ref, rtol=1e-12, atol=1e-12)
    # text queries: everything
    ref = torch.nn.functional.scaled_dot_product_attention(torch.tensor(Q[:n_text])[None], torch.tensor(K)[None], torch.tensor(V)[None])[0].numpy()
    np.testing.assert_allclose(O[:n_text], ref, rtol=1e-12, atol=1e-12)


# ---- the library's host side

@pytest.mark.parametrize("n_text,gridH,gridW,r,layer", [(3, 8, 12, 4, 6), (0, 10, 7, 3, 5), (2, 9, 13, 5, 27), (512, 64, 64, 16, 100),
                                                          (7, 33, 50, 16, 17)])
def test_library_mask_count_equals_the_oracle(n_text, gridH, gridW, r, layer):
    with orc.mask_kind(orc.MASK_STRIDED, layer):
        ref = orc.mask_count(n_text, gridH, gridW, r)
    assert ca.clear_attn_mask_count_masked(n_text, gridH, gridW, r, ca.CLEAR_MASK_STRIDED, layer) == ref


def test_no_raster_schedule_for_the_strided_mask():
    with pytest.raises(ca.ClearAttnError) as e:
        ca.clear_attn_schedule_host_masked(32, 32, 4, ca.CLEAR_MASK_STRIDED, 0, 16, 16, 8, 8)
    assert e.value.status == ca.CLEAR_ERR_UNSUPPORTED


# ---- GPU parity

DEV = "cuda:0"


def gpu_compare(n_text, gridH, gridW, r, layer, H=1, d=128, seed=0, B=1):
    print(f"[case] strided n_text={n_text} grid={gridH}x{gridW} r={r} layer={layer} H={H} d={d}", flush=True)
    Q, K, V = make_qkv_shape(B, H, n_text, gridH, gridW, d, "bf16", seed, device="cpu")
    ctx = ca.ClearAttn(n_text, gridH, gridW, d, r, ca.CLEAR_BF16, ca.CLEAR_MASK_STRIDED, layer)
    try:
        O = torch.full(Q.shape, float("nan"), dtype=Q.dtype, device=DEV)
        ctx.forward(Q.to(DEV), K.to(DEV), V.to(DEV), O)
        torch.cuda.synchronize()
        executed = ctx.executed_pairs()
    finally:
        ctx.destroy()
    with orc.mask_kind(orc.MASK_STRIDED, layer):
        ref = orc.attention(Q, K, V, n_text, gridH, gridW, r)
        useful = orc.mask_count(n_text, gridH, gridW, r)
    O = O.float().cpu().numpy()
    assert np.isfinite(O).all()  # every row written
    mx, rms = error_metrics(O, ref)
    assert mx <= TOL["bf16"][0] and rms <= TOL["bf16"][1], (mx, rms)
    assert executed >= useful
    return executed, useful


@pytest.mark.gpu
@pytest.mark.parametrize("n_text,gridH,gridW,r,layer,H,d", [
    (8, 16, 16, 4, 0, 1, 128),       # layer 0: a query sees its own residue class
    (37, 21, 30, 4, 6, 2, 128),      # ragged classes (extents 5/6 and 7/8), ragged text tile
    (0, 16, 24, 8, 9, 1, 128),       # no text tokens
    (100, 64, 64, 16, 35, 1, 128),   # the paper's ratio: 4 x 4 keys per query, class grid smaller than one tile
    (64, 70, 45, 2, 3, 1, 128),      # class grid 35 x 23: several query tiles, border tiles
    (5, 9, 11, 1, 0, 1, 128),        # r = 1: full attention
    (20, 40, 40, 4, 21, 1, 128),     # layer beyond r^2: the row offset wraps
    (37, 21, 30, 4, 6, 2, 64),       # head_dim 64
    (333, 64, 64, 16, 35, 1, 64),
])
def test_gpu_forward_strided(n_text, gridH, gridW, r, layer, H, d):
    gpu_compare(n_text, gridH, gridW, r, layer, H=H, d=d, seed=400 + gridH)


@pytest.mark.gpu
def test_gpu_strided_batch_of_two():
    gpu_compare(16, 24, 24, 4, 5, H=2, d=128, seed=77, B=2)


@pytest.mark.gpu
def test_gpu_strided_executes_only_useful_pairs_on_an_even_shape():
    """64 x 64 grid, r = 4: every class is a 16 x 16 grid = one query tile and four whole key tiles; 64 text tokens
    = one whole tile: nothing is padded, so the executed pairs are exactly sum(M)."""
    executed, useful = gpu_compare(64, 64, 64, 4, 2, seed=78)
    assert executed == useful


@pytest.mark.gpu
def test_gpu_strided_with_lse_and_prologue():
    from oracle import prologue as pro
    from paper_2412_16112_amd.inputs import make_prologue_inputs
    n_text, gridH, gridW, r, layer, d = 30, 26, 19, 4, 7, 128
    Q, K, V = make_qkv_shape(1, 1, n_text, gridH, gridW, d, "bf16", seed=79, device=DEV, q_scale=2.0)
    gq, gk, ty, tx = make_prologue_inputs(gridH, gridW, d, seed=80, device=DEV)
    f64 = lambda t: t.detach().cpu().double().numpy()
    ctx = ca.ClearAttn(n_text, gridH, gridW, d, r, ca.CLEAR_BF16, ca.CLEAR_MASK_STRIDED, layer)
    try:
        O, lse = ctx.forward_lse(Q, K, V)
        Op = ctx.forward_prologue(Q, K, V, q_gain=gq, k_gain=gk, rope_y=ty, rope_x=tx, logit_scale=0.9)
        torch.cuda.synchronize()
    finally:
        ctx.destroy()
    N = n_text + gridH * gridW
    with orc.mask_kind(orc.MASK_STRIDED, layer):
        ref, m, l, _ = orc.attention_rows(f64(Q[0, 0]), f64(K[0, 0]), f64(V[0, 0]), np.arange(N), n_text, gridH, gridW, r, return_stats=True)
        qp = pro.qk_prologue(f64(Q[0, 0]), f64(gq), 1e-6, n_text, gridH, gridW, f64(ty), f64(tx))
        kp = pro.qk_prologue(f64(K[0, 0]), f64(gk), 1e-6, n_text, gridH, gridW, f64(ty), f64(tx))
        refp = orc.attention_rows(qp * 0.9, kp, f64(V[0, 0]), np.arange(N), n_text, gridH, gridW, r)
    mx, rms = error_metrics(f64(O[0, 0]), ref)
    assert mx <= TOL["bf16"][0] and rms <= TOL["bf16"][1], (mx, rms)
    assert np.abs(f64(lse[0, 0]) - (m + np.log(l))).max() <= 5e-3
    mx, rms = error_metrics(f64(Op[0, 0]), refp)
    assert mx <= TOL["bf16"][0] and rms <= TOL["bf16"][1], (mx, rms)


@pytest.mark.gpu
def test_gpu_strided_unsupported_combinations():
    with pytest.raises(ca.ClearAttnError) as e:
        ca.ClearAttn(8, 16, 16, 64, 4, ca.CLEAR_F32, ca.CLEAR_MASK_STRIDED, 0)
    assert e.value.status == ca.CLEAR_ERR_UNSUPPORTED
    with pytest.raises(ca.ClearAttnError) as e:
        ca.ClearAttn(8, 3, 16, 128, 4, ca.CLEAR_BF16, ca.CLEAR_MASK_STRIDED, 0)
    assert e.value.status == ca.CLEAR_ERR_UNSUPPORTED
    with pytest.raises(ca.ClearAttnError) as e:
        ca.ClearAttn(8, 16, 16, 128, 4, ca.CLEAR_BF16, ca.CLEAR_MASK_STRIDED, -1)
    assert e.value.status == ca.CLEAR_ERR_INVALID_ARG
    Q, K, V = make_qkv_shape(1, 1, 8, 16, 16, 128, "bf16", seed=81, device=DEV)
    ctx = ca.ClearAttn(8, 16, 16, 128, 4, ca.CLEAR_BF16, ca.CLEAR_MASK_STRIDED, 3)
    try:
        with pytest.raises(ca.ClearAttnError) as e:
            ctx.forward_band(Q, K, V, torch.empty_like(Q), 0, 16, True)
        assert e.value.status == ca.CLEAR_ERR_UNSUPPORTED
    finally:
        ctx.destroy()


@pytest.mark.gpu
@pytest.mark.parametrize("n_text,gridH,gridW,r,layer", [
    (37, 21, 30, 4, 6),     # ragged classes; the key class differs from the query class on both axes
    (8, 16, 16, 4, 0),      # layer 0: query class = key class
    (0, 16, 24, 8, 9),      # no text tokens
    (64, 70, 45, 2, 3),     # several row tiles per class, border tiles
    (20, 40, 40, 4, 21),    # layer beyond r^2
])
def test_gpu_backward_strided(n_text, gridH, gridW, r, layer):
    """The mask is not symmetric: a key's queries are those of the class moved back by (r_y, r_x)."""
    d = 128
    Q, K, V = make_qkv_shape(1, 1, n_text, gridH, gridW, d, "bf16", seed=500 + gridH, device=DEV)
    g = torch.Generator(device=DEV).manual_seed(501)
    dO = torch.randn(Q.shape, generator=g, device=DEV, dtype=torch.float32).to(torch.bfloat16)
    ctx = ca.ClearAttn(n_text, gridH, gridW, d, r, ca.CLEAR_BF16, ca.CLEAR_MASK_STRIDED, layer)
    try:
        O, lse = ctx.forward_lse(Q, K, V)
        dQ = dK = dV = None
        dQ, dK, dV = ctx.backward(Q, K, V, O, dO, lse)
        torch.cuda.synchronize()
    finally:
        ctx.destroy()
    q, k, v, go = (t[0, 0].float().cpu().numpy() for t in (Q, K, V, dO))
    with orc.mask_kind(orc.MASK_STRIDED, layer):
        rQ, rK, rV = orc.backward(q, k, v, go, n_text, gridH, gridW, r)
    for name, got, ref in (("dQ", dQ, rQ), ("dK", dK, rK), ("dV", dV, rV)):
        got = got[0, 0].float().cpu().numpy()
        assert np.isfinite(got).all()
        max_abs, rel_rms = error_metrics(got, ref)
        assert max_abs <= TOL["bf16"][0] * np.abs(ref).max() and rel_rms <= TOL["bf16"][1], (name, max_abs, rel_rms)


@pytest.mark.gpu
def test_gpu_autograd_with_a_mask_kind():
    from paper_2412_16112_amd.autograd import clear_attention, clear_context_cache
    n_text, gridH, gridW, r, layer, d = 16, 24, 24, 4, 5, 128
    Q, K, V = make_qkv_shape(1, 1, n_text, gridH, gridW, d, "bf16", seed=510, device=DEV)
    Q.requires_grad_(True); K.requires_grad_(True); V.requires_grad_(True)
    g = torch.Generator(device=DEV).manual_seed(511)
    dO = torch.randn(Q.shape, generator=g, device=DEV, dtype=torch.float32).to(torch.bfloat16)
    try:
        O = clear_attention(Q, K, V, n_text, gridH, gridW, r, ca.CLEAR_MASK_STRIDED, layer)
        O.backward(dO)
        torch.cuda.synchronize()
    finally:
        clear_context_cache()
    q, k, v, go = (t[0, 0].detach().float().cpu().numpy() for t in (Q, K, V, dO))
    with orc.mask_kind(orc.MASK_STRIDED, layer):
        rQ, rK, rV = orc.backward(q, k, v, go, n_text, gridH, gridW, r)
    for got, ref in ((Q.grad, rQ), (K.grad, rK), (V.grad, rV)):
        max_abs, rel_rms = error_metrics(got[0, 0].float().cpu().numpy(), ref)
        assert max_abs <= TOL["bf16"][0] * np.abs(ref).max() and rel_rms <= TOL["bf16"][1], (max_abs, rel_rms)
