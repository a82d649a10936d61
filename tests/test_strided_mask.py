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
