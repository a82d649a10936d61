"""Pins of the backward oracle: the hand-written gradient sums of oracle/clear_oracle.c against automatic
differentiation of the dense masked definition, finite differences, and closed forms."""
import numpy as np
import pytest
import torch

from oracle import clear_oracle as orc


def _problem(seed, n_text, gridH, gridW, d, scale=1.0):
    rng = np.random.default_rng(seed)
    N = n_text + gridH * gridW
    Q, K, V, dO = (rng.standard_normal((N, d)) for _ in range(4))
    return Q * scale, K, V, dO


def _autograd(Q, K, V, dO, n_text, gridH, gridW, r):
    """torch autograd (fp64) through softmax(QK^T/sqrt(d) + mask) V with the mask of Eq. 3 built element by element."""
    M = torch.from_numpy(orc.mask_dense(n_text, gridH, gridW, r).astype(bool))
    q, k, v = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (Q, K, V))
    s = (q @ k.T) / np.sqrt(Q.shape[1])
    s = s.masked_fill(~M, float("-inf"))
    o = torch.softmax(s, dim=1) @ v
    o.backward(torch.tensor(dO, dtype=torch.float64))
    return q.grad.numpy(), k.grad.numpy(), v.grad.numpy()


@pytest.mark.parametrize("n_text,gridH,gridW,d,r", [(3, 5, 4, 8, 2), (8, 16, 16, 16, 4), (0, 7, 9, 4, 3), (5, 6, 6, 8, 1), (4, 5, 7, 8, 100)])
def test_backward_matches_autograd_of_the_dense_masked_definition(n_text, gridH, gridW, d, r):
    Q, K, V, dO = _problem(11, n_text, gridH, gridW, d, scale=1.7)
    dQ, dK, dV = orc.backward(Q, K, V, dO, n_text, gridH, gridW, r)
    rQ, rK, rV = _autograd(Q, K, V, dO, n_text, gridH, gridW, r)
    np.testing.assert_allclose(dQ, rQ, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dK, rK, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dV, rV, rtol=1e-10, atol=1e-12)


def test_backward_matches_central_differences():
    n_text, gridH, gridW, d, r = 2, 4, 3, 4, 2
    Q, K, V, dO = _problem(5, n_text, gridH, gridW, d)
    N = Q.shape[0]
    idx = np.arange(N)

    def loss(q, k, v):
        return float((orc.attention_rows(q, k, v, idx, n_text, gridH, gridW, r) * dO).sum())

    dQ, dK, dV = orc.backward(Q, K, V, dO, n_text, gridH, gridW, r)
    eps = 1e-6
    rng = np.random.default_rng(0)
    for name, X, G in (("Q", Q, dQ), ("K", K, dK), ("V", V, dV)):
        for _ in range(6):
            i, c = int(rng.integers(N)), int(rng.integers(d))
            Xp, Xm = X.copy(), X.copy()
            Xp[i, c] += eps
            Xm[i, c] -= eps
            args_p = {"Q": (Xp, K, V), "K": (Q, Xp, V), "V": (Q, K, Xp)}[name]
            args_m = {"Q": (Xm, K, V), "K": (Q, Xm, V), "V": (Q, K, Xm)}[name]
            fd = (loss(*args_p) - loss(*args_m)) / (2 * eps)
            assert abs(fd - G[i, c]) < 1e-7 * max(1.0, abs(fd)), (name, i, c, fd, G[i, c])


def test_dv_for_unit_upstream_is_the_column_sum_of_the_probabilities():
    # dO = one-hot channel 0 for every row: dV[j, 0] = sum_i p_ij, and the column sums add up to N (rows sum to 1)
    n_text, gridH, gridW, d, r = 4, 6, 5, 8, 3
    Q, K, V, _ = _problem(7, n_text, gridH, gridW, d)
    N = Q.shape[0]
    dO = np.zeros((N, d))
    dO[:, 0] = 1.0
    _, _, dV = orc.backward(Q, K, V, dO, n_text, gridH, gridW, r)
    assert np.abs(dV[:, 1:]).max() == 0.0
    assert abs(dV[:, 0].sum() - N) < 1e-9
    # read the probability matrix out of the FORWARD oracle with one-hot values, d columns at a time
    P = np.zeros((N, N))
    for j0 in range(0, N, d):
        w = min(d, N - j0)
        Vh = np.zeros((N, d))
        Vh[j0 + np.arange(w), np.arange(w)] = 1.0
        P[:, j0:j0 + w] = orc.attention_rows(Q, K, Vh, np.arange(N), n_text, gridH, gridW, r)[:, :w]
    np.testing.assert_allclose(dV[:, 0], P.sum(axis=0), rtol=1e-12, atol=1e-12)


def test_zero_upstream_and_constant_values_give_zero_gradients_for_q_and_k():
    n_text, gridH, gridW, d, r = 3, 5, 5, 8, 2
    Q, K, V, dO = _problem(9, n_text, gridH, gridW, d)
    dQ, dK, dV = orc.backward(Q, K, V, np.zeros_like(dO), n_text, gridH, gridW, r)
    assert np.abs(dQ).max() == 0 and np.abs(dK).max() == 0 and np.abs(dV).max() == 0
    # every value row the same: O does not depend on the softmax weights, so dQ = dK = 0 for any dO
    Vc = np.tile(V[:1], (V.shape[0], 1))
    dQ, dK, _ = orc.backward(Q, K, Vc, dO, n_text, gridH, gridW, r)
    assert np.abs(dQ).max() < 1e-13 and np.abs(dK).max() < 1e-13


def test_sampled_rows_and_columns_equal_the_full_result():
    n_text, gridH, gridW, d, r = 6, 9, 8, 8, 3
    Q, K, V, dO = _problem(21, n_text, gridH, gridW, d)
    dQ, dK, dV = orc.backward(Q, K, V, dO, n_text, gridH, gridW, r)
    rows = np.array([0, 5, 6, 17, 40, 77])
    np.testing.assert_allclose(orc.backward_dq_rows(Q, K, V, dO, rows, n_text, gridH, gridW, r), dQ[rows], rtol=1e-13, atol=1e-14)
    cK, cV = orc.backward_dkv_cols(Q, K, V, dO, rows, n_text, gridH, gridW, r)
    np.testing.assert_allclose(cK, dK[rows], rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(cV, dV[rows], rtol=1e-13, atol=1e-14)
