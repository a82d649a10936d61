"""Row-band (patch-parallel) forward on one GPU: every band is run through the C ABI on its local tensors
(band + halo), the text rows are merged, and the result is compared with the CPU oracle of the UNDIVIDED
problem (image rows, exact text merge) or of Eq. 7 (average text merge)."""
import numpy as np
import pytest
import torch

from oracle import clear_oracle as orc
from oracle import patch_parallel as pp
from paper_2412_16112_amd import clear_attn as ca
from paper_2412_16112_amd.inputs import make_qkv_shape
from tests.parity_util import TOL, error_metrics

pytestmark = pytest.mark.gpu


def run_bands(Q, K, V, n_text, gridH, gridW, r, n_bands, mode, halo_align=1):
    """Returns O [B, H, N, d] assembled from n_bands band passes (each on its own local copy of the tokens).
    halo_align > 1: the top halo is widened to a multiple of that many rows (more neighbour rows than the r - 1
    the mask can reach, e.g. so that the owned rows start on a query-tile boundary)."""
    B, H, N, d = Q.shape
    dev = Q.device
    O = torch.zeros_like(Q)
    parts_o, parts_lse = [], []
    for band in range(n_bands):
        y0, y1, ht, hb = ca.clear_attn_band_layout(gridH, r, n_bands, band)
        if ht:
            ht = min(y0, -(-ht // halo_align) * halo_align)
        rows = slice(n_text + (y0 - ht) * gridW, n_text + (y1 + hb) * gridW)
        loc = [torch.cat([t[:, :, :n_text], t[:, :, rows]], dim=2).contiguous() for t in (Q, K, V)]
        Ol = torch.full_like(loc[0], float("nan"))
        ctx = ca.ClearAttn(n_text, ht + (y1 - y0) + hb, gridW, d, r, ca._dtype_code(Q))
        try:
            text_keys = True if mode == ca.CLEAR_MERGE_AVERAGE else band == 0
            _, to, tl = ctx.forward_band(loc[0], loc[1], loc[2], Ol, ht, ht + (y1 - y0), text_keys)
            torch.cuda.synchronize(dev)
        finally:
            ctx.destroy()
        own = Ol[:, :, n_text + ht * gridW: n_text + (ht + y1 - y0) * gridW]
        assert torch.isfinite(own.float()).all()
        # halo rows and text rows of the local output are not written
        assert torch.isnan(Ol[:, :, :n_text].float()).all()
        if ht:
            assert torch.isnan(Ol[:, :, n_text:n_text + ht * gridW].float()).all()
        if hb:
            assert torch.isnan(Ol[:, :, n_text + (ht + y1 - y0) * gridW:].float()).all()
        O[:, :, n_text + y0 * gridW: n_text + y1 * gridW] = own
        if n_text:
            parts_o.append(to)
            parts_lse.append(tl)
    if n_text:
        ca.clear_attn_merge_text(parts_o, parts_lse, O, n_text, mode)
        torch.cuda.synchronize(dev)
    return O


CASES = [
    # dtype, n_text, gridH, gridW, d, r, H, bands
    ("f32", 8, 16, 16, 64, 4, 1, 3),
    ("f32", 5, 23, 9, 64, 3, 2, 5),
    ("bf16", 64, 40, 24, 128, 8, 2, 2),
    ("bf16", 100, 64, 64, 128, 16, 1, 4),   # bands of 16 rows with 15 halo rows: the narrowest allowed
    ("bf16", 37, 50, 19, 128, 6, 1, 7),     # uneven bands, ragged tiles everywhere
    ("bf16", 0, 48, 32, 128, 8, 1, 3),      # no text tokens
]
# (head_dim 64 only against the undivided problem: its flatter softmax rows leave Eq. 7 too close to the exact merge
# for the test of the average to tell them apart)
CASES_D64 = [("bf16", 24, 40, 24, 64, 8, 2, 2)]


@pytest.mark.parametrize("dtype,n_text,gridH,gridW,d,r,H,n_bands", CASES + CASES_D64)
def test_bands_exact_equal_the_undivided_problem(dtype, n_text, gridH, gridW, d, r, H, n_bands):
    Q, K, V = make_qkv_shape(1, H, n_text, gridH, gridW, d, dtype, seed=100 + n_bands, device="cuda:0")
    O = run_bands(Q, K, V, n_text, gridH, gridW, r, n_bands, ca.CLEAR_MERGE_EXACT)
    ref = orc.attention(Q.float().cpu().numpy(), K.float().cpu().numpy(), V.float().cpu().numpy(), n_text, gridH, gridW, r)
    max_abs, rel_rms = error_metrics(O.float().cpu().numpy(), ref)
    assert max_abs <= TOL[dtype][0] and rel_rms <= TOL[dtype][1], (max_abs, rel_rms)


def test_bands_with_a_tile_aligned_halo():
    """A halo wider than r - 1 rows (here: widened to the 16 rows of a query tile) changes nothing: the extra
    rows are out of every owned query's reach."""
    n_text, gridH, gridW, d, r, H, n_bands = 64, 96, 40, 128, 8, 1, 3
    Q, K, V = make_qkv_shape(1, H, n_text, gridH, gridW, d, "bf16", seed=321, device="cuda:0")
    O = run_bands(Q, K, V, n_text, gridH, gridW, r, n_bands, ca.CLEAR_MERGE_EXACT, halo_align=16)
    ref = orc.attention(Q.float().cpu().numpy(), K.float().cpu().numpy(), V.float().cpu().numpy(), n_text, gridH, gridW, r)
    max_abs, rel_rms = error_metrics(O.float().cpu().numpy(), ref)
    assert max_abs <= TOL["bf16"][0] and rel_rms <= TOL["bf16"][1], (max_abs, rel_rms)


def _one_band_vs_oracle(ctx, Q, K, V, n_text, gridH, gridW, r, y0, y1, top):
    """Runs rows [y0, y1) of the undivided problem as a band whose local grid starts `top` rows above y0 and ends at
    the bottom halo; returns (max_abs, rel_rms) of the owned rows against the oracle of the undivided problem."""
    hb = min(r - 1, gridH - y1)
    rows = slice(n_text + (y0 - top) * gridW, n_text + (y1 + hb) * gridW)
    loc = [torch.cat([t[:, :, :n_text], t[:, :, rows]], dim=2).contiguous() for t in (Q, K, V)]
    Ol = torch.full_like(loc[0], float("nan"))
    ctx.forward_band(loc[0], loc[1], loc[2], Ol, top, top + (y1 - y0), True)
    torch.cuda.synchronize()
    own = Ol[0, :, n_text + top * gridW: n_text + (top + y1 - y0) * gridW].float().cpu().numpy()
    assert np.isfinite(own).all()
    assert torch.isnan(Ol[:, :, n_text:n_text + top * gridW].float()).all()
    assert torch.isnan(Ol[:, :, n_text + (top + y1 - y0) * gridW:].float()).all()
    idx = np.arange(n_text + y0 * gridW, n_text + y1 * gridW)
    ref = np.stack([orc.attention_rows(*(t[0, h].float().cpu().numpy() for t in (Q, K, V)), idx, n_text, gridH, gridW, r)
                    for h in range(Q.shape[1])])
    return error_metrics(own, ref)


def test_band_starting_off_the_tile_lattice():
    """Owned ranges whose first row is not a multiple of the 16-row query tile.  On one context: r - 1 or more halo
    rows above (the tile lists are then moved so that a tile row starts at the first owned row: two different moves,
    the first one used again, ranges ending on and inside a tile).  On another: fewer than r - 1 rows above because
    the image ends there (the tile lists of the grid as it is)."""
    n_text, gridH, gridW, d, r, H = 40, 88, 40, 128, 8, 2
    Q, K, V = make_qkv_shape(1, H, n_text, gridH, gridW, d, "bf16", seed=77, device="cuda:0")
    # every local grid has top + (y1 - y0) + 7 = 46 rows; the first owned local row is 7 or 10
    ctx = ca.ClearAttn(n_text, 46, gridW, d, r, ca.CLEAR_BF16)
    try:
        for y0, y1, top in [(23, 55, 7), (26, 55, 10), (23, 55, 7), (42, 71, 10)]:
            max_abs, rel_rms = _one_band_vs_oracle(ctx, Q, K, V, n_text, gridH, gridW, r, y0, y1, top)
            assert max_abs <= TOL["bf16"][0] and rel_rms <= TOL["bf16"][1], (y0, y1, top, max_abs, rel_rms)
    finally:
        ctx.destroy()
    # the band at the top of the image, queries from row 5 on: only 5 rows above, fewer than r - 1
    ctx = ca.ClearAttn(n_text, 5 + 21 + 7, gridW, d, r, ca.CLEAR_BF16)
    try:
        max_abs, rel_rms = _one_band_vs_oracle(ctx, Q, K, V, n_text, gridH, gridW, r, 5, 26, 5)
        assert max_abs <= TOL["bf16"][0] and rel_rms <= TOL["bf16"][1], (max_abs, rel_rms)
    finally:
        ctx.destroy()


@pytest.mark.parametrize("dtype,n_text,gridH,gridW,d,r,H,n_bands", [c for c in CASES if c[1] > 0])
def test_bands_average_is_eq7(dtype, n_text, gridH, gridW, d, r, H, n_bands):
    Q, K, V = make_qkv_shape(1, H, n_text, gridH, gridW, d, dtype, seed=200 + n_bands, device="cuda:0")
    O = run_bands(Q, K, V, n_text, gridH, gridW, r, n_bands, ca.CLEAR_MERGE_AVERAGE)
    bands = [ca.clear_attn_band_layout(gridH, r, n_bands, b)[:2] for b in range(n_bands)]
    assert bands == pp.band_rows(gridH, n_bands)
    tol = TOL[dtype]
    for h in range(H):
        q, k, v = (t[0, h].float().cpu().numpy() for t in (Q, K, V))
        ref = pp.text_rows_average(q, k, v, n_text, gridW, bands)
        max_abs, rel_rms = error_metrics(O[0, h, :n_text].float().cpu().numpy(), ref)
        assert max_abs <= tol[0] and rel_rms <= tol[1], (max_abs, rel_rms)
        # and it is NOT the exact result (the approximation is visible at these sizes), so the test can tell the modes apart
        exact = orc.attention_rows(q, k, v, np.arange(n_text), n_text, gridH, gridW, r)
        assert np.abs(ref - exact).max() > 2 * tol[0]


def test_merge_exact_against_numpy_merge():
    rng = np.random.default_rng(5)
    n_parts, B, H, n_text, d, N = 5, 1, 2, 7, 64, 50
    o = rng.standard_normal((n_parts, B, H, n_text, d)).astype(np.float32)
    lse = (rng.standard_normal((n_parts, B, H, n_text)) * 6).astype(np.float32)
    O = torch.zeros((B, H, N, d), dtype=torch.float32, device="cuda:0")
    to = [torch.from_numpy(o[i]).cuda() for i in range(n_parts)]
    tl = [torch.from_numpy(lse[i]).cuda() for i in range(n_parts)]
    ca.clear_attn_merge_text(to, tl, O, n_text, ca.CLEAR_MERGE_EXACT)
    torch.cuda.synchronize()
    ref = pp.merge_exact(o.reshape(n_parts, -1, d), lse.reshape(n_parts, -1)).reshape(B, H, n_text, d)
    np.testing.assert_allclose(O[:, :, :n_text].cpu().numpy(), ref, rtol=2e-5, atol=2e-6)
    assert (O[:, :, n_text:] == 0).all()
