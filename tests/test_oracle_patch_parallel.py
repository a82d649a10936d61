"""Pins of the patch-parallel oracle (multi-GPU section, Eq. 7) against things other than itself."""
import numpy as np
import pytest

from oracle import clear_oracle as orc
from oracle import patch_parallel as pp


def _problem(seed, n_text, gridH, gridW, d):
    rng = np.random.default_rng(seed)
    N = n_text + gridH * gridW
    return tuple(rng.standard_normal((N, d)) for _ in range(3))


def test_band_rows_partition():
    for gridH, n in [(64, 8), (10, 3), (7, 7), (5, 1)]:
        b = pp.band_rows(gridH, n)
        assert b[0][0] == 0 and b[-1][1] == gridH and len(b) == n
        assert all(b[i][1] == b[i + 1][0] for i in range(n - 1))
        sizes = [y1 - y0 for y0, y1 in b]
        assert max(sizes) - min(sizes) <= 1


def test_one_band_is_the_plain_definition():
    # N = 1 in Eq. 7: no approximation is left; the text rows of the plain dense-masked definition (every key
    # is admitted for a text query, Eq. 3) computed by the C oracle must come out.
    n_text, gridH, gridW, d, r = 5, 6, 7, 8, 3
    Q, K, V = _problem(1, n_text, gridH, gridW, d)
    got = pp.text_rows_average(Q, K, V, n_text, gridW, [(0, gridH)])
    ref = orc.attention_rows(Q, K, V, np.arange(n_text), n_text, gridH, gridW, r)
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-12)


def test_zero_queries_give_means_of_means():
    # q = 0: every softmax weight inside a band is equal, so O_p is the plain mean of V over the band's keys
    # and Eq. 7 is the mean of those means: a closed form with no exponential in it.
    n_text, gridH, gridW, d = 3, 4, 5, 2
    _, K, V = _problem(2, n_text, gridH, gridW, d)
    Q = np.zeros_like(K)
    bands = [(0, 1), (1, 4)]
    expect = np.zeros(d)
    for y0, y1 in bands:
        rows = list(range(n_text)) + [n_text + y * gridW + x for y in range(y0, y1) for x in range(gridW)]
        expect += V[rows].mean(axis=0)
    expect /= len(bands)
    got = pp.text_rows_average(Q, K, V, n_text, gridW, bands)
    np.testing.assert_allclose(got, np.broadcast_to(expect, got.shape), rtol=1e-13, atol=1e-13)


def test_average_differs_from_exact_and_by_how_much_in_a_two_key_case():
    # One text token (q, k_t, v_t), two bands of one image token each, d = 1, values chosen by hand:
    # scores s = q * k; with q = 1: s_t = 0, s_1 = ln 3, s_2 = 0  (k = 0, ln 3, 0), v = (0, 1, 1).
    # Band 1 holds {t, 1}: weights 1 : 3 -> O_1 = 3/4.  Band 2 holds {t, 2}: weights 1 : 1 -> O_2 = 1/2.
    # Eq. 7: (3/4 + 1/2) / 2 = 5/8.  Exact softmax over {t, 1, 2}: weights 1 : 3 : 1 -> 4/5.
    n_text, gridW = 1, 1
    Q = np.array([[1.0], [0.0], [0.0]])
    K = np.array([[0.0], [np.log(3.0)], [0.0]])
    V = np.array([[0.0], [1.0], [1.0]])
    bands = [(0, 1), (1, 2)]
    got = pp.text_rows_average(Q, K, V, n_text, gridW, bands)
    assert got.shape == (1, 1)
    assert abs(got[0, 0] - 5.0 / 8.0) < 1e-14
    ref = orc.attention_rows(Q, K, V, np.arange(1), n_text, 2, 1, 1)
    assert abs(ref[0, 0] - 4.0 / 5.0) < 1e-14


@pytest.mark.parametrize("n_bands", [2, 3, 5])
def test_exact_merge_of_disjoint_bands_is_the_plain_definition(n_bands):
    # text keys counted in band 0 only -> the key sets are disjoint and cover every token; the weighted merge
    # must reproduce the undivided softmax (C oracle), whatever the number of bands.
    n_text, gridH, gridW, d, r = 4, 10, 6, 8, 4
    Q, K, V = _problem(3 + n_bands, n_text, gridH, gridW, d)
    Q *= 3.0  # sharp logits: the per-band denominators differ by orders of magnitude
    bands = pp.band_rows(gridH, n_bands)
    O_p, lse_p = pp.text_rows_per_band(Q, K, V, n_text, gridW, bands, text_in_band=[p == 0 for p in range(n_bands)])
    got = pp.merge_exact(O_p, lse_p)
    ref = orc.attention_rows(Q, K, V, np.arange(n_text), n_text, gridH, gridW, r)
    np.testing.assert_allclose(got, ref, rtol=1e-11, atol=1e-12)


def test_identical_bands_average_to_any_one_of_them():
    # the image rows of the two bands hold the same keys and values: O_1 = O_2, so their mean is O_1
    n_text, gridW, d = 3, 4, 4
    Q, K, V = _problem(9, n_text, 2, gridW, d)
    K[n_text + gridW:] = K[n_text:n_text + gridW]
    V[n_text + gridW:] = V[n_text:n_text + gridW]
    O_p, _ = pp.text_rows_per_band(Q, K, V, n_text, gridW, [(0, 1), (1, 2)])
    np.testing.assert_allclose(O_p[0], O_p[1], rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(pp.text_rows_average(Q, K, V, n_text, gridW, [(0, 1), (1, 2)]), O_p[0], rtol=1e-13, atol=1e-13)
