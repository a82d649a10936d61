"""Pins of the CPU oracle against things that are NOT the oracle: numbers the paper prints,
closed forms, brute force written out here, library routines for special cases, invariants.

Each test is chosen so that a plausible slip in oracle/clear_oracle.c (<= instead of <, a
wrapped or shifted window at the border, a wrong text rule, swapped x/y strides, a missing
1/sqrt(d), softmax over the wrong axis, K and V swapped) makes it fail.
"""
import math
import os

import numpy as np
import pytest
import torch

from oracle import clear_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_attention_flops.txt")
C_MODEL = 3072  # feature dimension c of the FLOP estimate 4*sum(M)*c (Fig. 2 caption): 24 heads x 128
N_TEXT = 512


def lattice_sum_mask(n_text, gridH, gridW, r):
    """sum(M) from a lattice-point count, independent of the oracle's per-element loop:
    each offset (dy, dx) inside the open disc of radius r occurs (gridH-|dy|)*(gridW-|dx|) times."""
    n_img = gridH * gridW
    N = n_text + n_img
    img = 0
    for dy in range(-(r - 1), r):
        for dx in range(-(r - 1), r):
            if dx * dx + dy * dy < r * r:
                img += max(0, gridH - abs(dy)) * max(0, gridW - abs(dx))
    return n_text * N + n_img * n_text + img


def _golden_rows():
    rows = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                src, px, r, val, unit = line.split()
                rows.append((src, int(px), int(r), val, unit))
    return rows


@pytest.mark.parametrize("src,px,r,val,unit", _golden_rows())
def test_paper_flops_from_lattice(src, px, r, val, unit):
    """4*sum(M)*c reproduces every FLOP figure of Tables 2, 3, 7 to the printed digits."""
    g = px // 16
    sm = (N_TEXT + g * g) ** 2 if r == 0 else lattice_sum_mask(N_TEXT, g, g, r)
    flops = 4 * sm * C_MODEL / (1e9 if unit == "G" else 1e12)
    digits = len(val.split(".")[1])
    # half a unit of the last printed digit; 0.51 because Table 7 prints 13.09 for 8192 px, r=32 where
    # the definition gives 13.08497 (0.503 units off) -- every other entry is within 0.5
    assert abs(flops - float(val)) <= 0.51 * 10 ** (-digits), (src, px, r, flops, val)


@pytest.mark.parametrize("g,r", [(64, 8), (64, 16), (64, 32), (128, 8), (128, 16), (128, 32)])
def test_oracle_mask_count_matches_paper_and_lattice(g, r):
    """The oracle's element-by-element sum(M) equals the lattice count (hence the paper's tables)."""
    sm = orc.mask_count(N_TEXT, g, g, r)
    assert sm == lattice_sum_mask(N_TEXT, g, g, r)
    printed = {(src, px, rr): (val, unit) for src, px, rr, val, unit in _golden_rows()}
    key = ("table2" if g == 64 else "table3", g * 16, r)
    if key in printed:
        val, unit = printed[key]
        assert abs(4 * sm * C_MODEL / 1e9 - float(val)) <= 0.05 + 1e-9


def test_oracle_mask_count_le_would_not_match_paper():
    """The strict '<' of Eq. 3 matters: counting distance == r as inside misses the printed value."""
    g, r = 128, 16
    le = 0
    for dy in range(-r, r + 1):
        for dx in range(-r, r + 1):
            if dx * dx + dy * dy <= r * r:
                le += (g - abs(dy)) * (g - abs(dx))
    sm_le = N_TEXT * (N_TEXT + g * g) + g * g * N_TEXT + le
    assert abs(4 * sm_le * C_MODEL / 1e9 - 352.6) > 0.05
    assert abs(4 * orc.mask_count(N_TEXT, g, g, r) * C_MODEL / 1e9 - 352.6) <= 0.05


@pytest.mark.slow
def test_oracle_mask_count_4096():
    assert orc.mask_count(N_TEXT, 256, 256, 32) == lattice_sum_mask(N_TEXT, 256, 256, 32) == 255670316


@pytest.mark.parametrize("n_text,gh,gw,r", [(8, 16, 16, 4), (0, 5, 9, 3), (3, 7, 4, 1), (5, 6, 6, 20), (512, 192 // 8, 320 // 8, 5)])
def test_oracle_mask_count_small_and_nonsquare(n_text, gh, gw, r):
    assert orc.mask_count(n_text, gh, gw, r) == lattice_sum_mask(n_text, gh, gw, r)
    assert orc.mask_dense(n_text, gh, gw, r).sum() == lattice_sum_mask(n_text, gh, gw, r)


def test_tiny_sum_mask_value():
    assert orc.mask_count(8, 16, 16, 4) == 13484
    assert lattice_sum_mask(512, 512, 512, 16) == 471125568
    assert lattice_sum_mask(512, 192, 320, 32) == 238348332


@pytest.mark.parametrize("r,interior", [(4, 45), (8, 193), (16, 793), (32, 3205)])
def test_interior_and_corner_row_counts(r, interior):
    """Interior image rows see the full open disc (+ all text); the corner token sees the quarter disc."""
    n_text, g = 7, 2 * r + 5
    centre = n_text + (g // 2) * g + g // 2
    assert orc.row_count(centre, n_text, g, g, r) == interior + n_text
    quarter = sum(1 for dy in range(r) for dx in range(r) if dx * dx + dy * dy < r * r)
    assert orc.row_count(n_text, n_text, g, g, r) == quarter + n_text
    assert orc.row_count(0, n_text, g, g, r) == n_text + g * g  # text rows see everything
    # circle / square ratio tends to pi/4 (Sec. 3.2)
    ratio = interior / (2 * r + 1) ** 2
    assert ratio < math.pi / 4 and (r < 32 or ratio > 0.75)


def test_dense_mask_structure():
    n_text, gh, gw, r = 3, 6, 9, 3
    M = orc.mask_dense(n_text, gh, gw, r)
    N = n_text + gh * gw
    assert M[:n_text].all() and M[:, :n_text].all()
    Mi = M[n_text:, n_text:]
    assert (Mi == Mi.T).all() and np.diag(Mi).all()
    for i in range(gh * gw):  # written-out predicate, separate code
        for j in range(gh * gw):
            yi, xi, yj, xj = i // gw, i % gw, j // gw, j % gw
            assert Mi[i, j] == ((xi - xj) ** 2 + (yi - yj) ** 2 < r * r)
    # no wrap-around: first and last column of the same row are not neighbours
    assert Mi[0, gw - 1] == 0 and Mi[0, gw] == 1  # (0,0)-(0,gw-1) far apart; (0,0)-(1,0) adjacent
    assert N == M.shape[0]


def _rand(shape, seed):
    g = torch.Generator().manual_seed(seed)
    return torch.randn(shape, generator=g, dtype=torch.float32).numpy().astype(np.float64)


def test_attention_vs_python_triple_loop_tiny():
    """The tiny configuration (16x16 grid, 8 text tokens, r=4, d=64) against loops written out here."""
    n_text, gh, gw, r, d = 8, 16, 16, 4, 64
    N = n_text + gh * gw
    Q, K, V = _rand((N, d), 0), _rand((N, d), 1), _rand((N, d), 2)
    rows = np.arange(N)
    O, m, l, cnt = orc.attention_rows(Q, K, V, rows, n_text, gh, gw, r, return_stats=True)
    ref = np.zeros((N, d))
    for i in range(N):
        logits = {}
        for j in range(N):
            if i >= n_text and j >= n_text:
                yi, xi = divmod(i - n_text, gw)
                yj, xj = divmod(j - n_text, gw)
                if (xi - xj) ** 2 + (yi - yj) ** 2 >= r * r:
                    continue
            logits[j] = sum(Q[i, c] * K[j, c] for c in range(d)) / math.sqrt(d)
        mx = max(logits.values())
        den = sum(math.exp(v - mx) for v in logits.values())
        for j, v in logits.items():
            ref[i] += math.exp(v - mx) / den * V[j]
        assert cnt[i] == len(logits)
        assert abs(m[i] - mx) < 1e-12 and abs(l[i] - den) < 1e-9
    assert np.abs(O - ref).max() < 1e-12
    assert cnt.sum() == 13484


def test_large_r_is_full_attention_library():
    """r beyond the grid diagonal: every pair is unmasked, so the result is textbook attention."""
    n_text, gh, gw, d = 5, 7, 9, 32
    N = n_text + gh * gw
    r = int(math.sqrt((gh - 1) ** 2 + (gw - 1) ** 2)) + 1
    Q, K, V = _rand((N, d), 3), _rand((N, d), 4), _rand((N, d), 5)
    O = orc.attention_rows(Q, K, V, np.arange(N), n_text, gh, gw, r)
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(Q)[None], torch.from_numpy(K)[None], torch.from_numpy(V)[None])[0].numpy()
    assert np.abs(O - ref).max() < 1e-12
    # one step below the diagonal the two far corners stop seeing each other
    O2 = orc.attention_rows(Q, K, V, np.arange(N), n_text, gh, gw, r - 1)
    assert np.abs(O2[n_text] - ref[n_text]).max() > 1e-9
    assert np.abs(O2[:n_text] - ref[:n_text]).max() < 1e-12  # text rows are always dense


def test_masked_attention_vs_library_with_dense_mask():
    """General r: torch's fp64 SDPA with an explicit boolean mask built from the written-out predicate."""
    n_text, gh, gw, r, d = 4, 10, 13, 4, 16
    N = n_text + gh * gw
    Q, K, V = _rand((N, d), 6), _rand((N, d), 7), _rand((N, d), 8)
    ys, xs = np.divmod(np.arange(gh * gw), gw)
    Mi = (xs[:, None] - xs[None, :]) ** 2 + (ys[:, None] - ys[None, :]) ** 2 < r * r
    M = np.ones((N, N), dtype=bool)
    M[n_text:, n_text:] = Mi
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(Q)[None], torch.from_numpy(K)[None], torch.from_numpy(V)[None],
        attn_mask=torch.from_numpy(M)[None])[0].numpy()
    O = orc.attention_rows(Q, K, V, np.arange(N), n_text, gh, gw, r)
    assert np.abs(O - ref).max() < 1e-12


def test_probabilities_sum_to_one_and_vanish_outside_mask():
    n_text, gh, gw, r, d = 2, 6, 5, 3, 8
    N = n_text + gh * gw
    Q, K = _rand((N, d), 9), _rand((N, d), 10)
    ones = orc.attention_rows(Q, K, np.ones((N, d)), np.arange(N), n_text, gh, gw, r)
    assert np.abs(ones - 1.0).max() < 1e-14
    # one-hot V blocks read the probability matrix column block by column block
    P = np.zeros((N, N))
    for c0 in range(0, N, d):
        Vh = np.zeros((N, d))
        for c in range(min(d, N - c0)):
            Vh[c0 + c, c] = 1.0
        P[:, c0:c0 + d] = orc.attention_rows(Q, K, Vh, np.arange(N), n_text, gh, gw, r)[:, :min(d, N - c0)]
    M = orc.mask_dense(n_text, gh, gw, r).astype(bool)
    assert (P[~M] == 0.0).all() and (P[M] > 0.0).all()
    assert np.abs(P.sum(axis=1) - 1.0).max() < 1e-14
    S = Q @ K.T / math.sqrt(d)
    S[~M] = -np.inf
    ref = np.exp(S - S.max(axis=1, keepdims=True))
    ref /= ref.sum(axis=1, keepdims=True)
    assert np.abs(P - ref).max() < 1e-14


def test_key_shift_and_scale_properties():
    n_text, gh, gw, r, d = 3, 8, 8, 3, 16
    N = n_text + gh * gw
    # dyadic values so that K + u is exact in fp64
    Q = np.round(_rand((N, d), 11) * 8) / 8
    K = np.round(_rand((N, d), 12) * 8) / 8
    V = _rand((N, d), 13)
    u = np.round(_rand((1, d), 14) * 8) / 8
    rows = np.arange(N)
    O = orc.attention_rows(Q, K, V, rows, n_text, gh, gw, r)
    O_shift = orc.attention_rows(Q, K + u, V, rows, n_text, gh, gw, r)  # adds q.u to every logit of a row
    assert np.abs(O - O_shift).max() < 1e-12
    # the 1/sqrt(d) of Eq. 1: zero-padding the channels to 4d must equal scaling Q by 2 at width 4d
    # ... i.e. padding changes the scale, which a missing/incorrect scale would not notice:
    Qp = np.concatenate([Q, np.zeros((N, 3 * d))], axis=1)
    Kp = np.concatenate([K, np.zeros((N, 3 * d))], axis=1)
    Vp = np.concatenate([V, np.zeros((N, 3 * d))], axis=1)
    O_pad = orc.attention_rows(2 * Qp, Kp, Vp, rows, n_text, gh, gw, r)[:, :d]
    assert np.abs(O - O_pad).max() < 1e-12
    O_pad_unscaled = orc.attention_rows(Qp, Kp, Vp, rows, n_text, gh, gw, r)[:, :d]
    assert np.abs(O - O_pad_unscaled).max() > 1e-6


def test_r1_no_text_is_identity():
    gh, gw, d = 5, 6, 8
    N = gh * gw
    Q, K, V = _rand((N, d), 15), _rand((N, d), 16), _rand((N, d), 17)
    O = orc.attention_rows(Q, K, V, np.arange(N), 0, gh, gw, 1)
    assert np.abs(O - V).max() < 1e-15


def test_transpose_symmetry_nonsquare():
    """Eq. 3 is symmetric in x and y: transposing the raster transposes the result."""
    n_text, gh, gw, r, d = 3, 6, 11, 4, 8
    n_img = gh * gw
    N = n_text + n_img
    Q, K, V = _rand((N, d), 18), _rand((N, d), 19), _rand((N, d), 20)
    O = orc.attention_rows(Q, K, V, np.arange(N), n_text, gh, gw, r)
    perm = np.arange(n_img).reshape(gh, gw).T.reshape(-1)  # raster of the transposed (gw x gh) grid
    idx = np.concatenate([np.arange(n_text), n_text + perm])
    Ot = orc.attention_rows(Q[idx], K[idx], V[idx], np.arange(N), n_text, gw, gh, r)
    assert np.abs(Ot - O[idx]).max() < 1e-13
    # and it is NOT invariant if the grid shape is kept while tokens are transposed
    assert np.abs(orc.attention_rows(Q[idx], K[idx], V[idx], np.arange(N), n_text, gh, gw, r) - O[idx]).max() > 1e-6


def test_rows_subset_and_batched_front_end():
    n_text, gh, gw, r, d = 4, 6, 6, 3, 8
    N = n_text + gh * gw
    Q, K, V = (_rand((2, 3, N, d), s) for s in (21, 22, 23))
    O = orc.attention(Q, K, V, n_text, gh, gw, r)
    rows = np.array([0, 5, N - 1, 17])
    sub = orc.attention_rows(Q[1, 2], K[1, 2], V[1, 2], rows, n_text, gh, gw, r)
    assert np.array_equal(sub, O[1, 2][rows])


def _geometric_schedule(gh, gw, r, qth, qtw, kth, ktw):
    """Interval-distance rule, written independently of the element mask."""
    nqy, nqx, nky, nkx = -(-gh // qth), -(-gw // qtw), -(-gh // kth), -(-gw // ktw)
    row_ptr, col, flags = [0], [], []

    def gap(a0, a1, b0, b1):  # min and max |a-b| for a in [a0,a1], b in [b0,b1]
        return max(0, b0 - a1, a0 - b1), max(a1 - b0, b1 - a0)

    for qy in range(nqy):
        for qx in range(nqx):
            for ky in range(nky):
                for kx in range(nkx):
                    # clipped extents decide "listed"; unclipped ones decide FULL
                    q = (qy * qth, min(gh, (qy + 1) * qth) - 1, qx * qtw, min(gw, (qx + 1) * qtw) - 1)
                    k = (ky * kth, min(gh, (ky + 1) * kth) - 1, kx * ktw, min(gw, (kx + 1) * ktw) - 1)
                    dy0, dy1 = gap(q[0], q[1], k[0], k[1])
                    dx0, dx1 = gap(q[2], q[3], k[2], k[3])
                    if dy0 * dy0 + dx0 * dx0 < r * r:
                        col.append(ky * nkx + kx)
                        clipped = ((qy + 1) * qth > gh or (qx + 1) * qtw > gw or (ky + 1) * kth > gh or (kx + 1) * ktw > gw)
                        flags.append(int(not clipped and dy1 * dy1 + dx1 * dx1 < r * r))
            row_ptr.append(len(col))
    return np.array(row_ptr, np.int32), np.array(col, np.int32), np.array(flags, np.uint8)


@pytest.mark.parametrize("gh,gw,r,qt,kt", [(20, 28, 4, (4, 8), (4, 8)), (16, 16, 4, (8, 16), (8, 8)),
                                           (33, 17, 9, (16, 16), (8, 8)), (24, 40, 16, (16, 16), (4, 8)),
                                           (12, 12, 3, (2, 2), (1, 2)), (40, 40, 12, (4, 4), (2, 2))])
def test_bruteforce_schedule_vs_geometric_rule(gh, gw, r, qt, kt):
    rp, ci, fl = orc.tile_schedule(gh, gw, r, qt[0], qt[1], kt[0], kt[1])
    rp2, ci2, fl2 = _geometric_schedule(gh, gw, r, qt[0], qt[1], kt[0], kt[1])
    assert np.array_equal(rp, rp2) and np.array_equal(ci, ci2) and np.array_equal(fl, fl2)
    # nothing dropped: pair counts over listed tiles add up to the image-image part of sum(M)
    cnt = orc.tile_pair_counts(gh, gw, r, qt[0], qt[1], kt[0], kt[1])
    assert cnt.sum() == lattice_sum_mask(0, gh, gw, r)
    if qt == (4, 4):  # small tiles inside a radius-12 disc: some pairs must be FULL, some PARTIAL
        assert fl.any() and not fl.all()
