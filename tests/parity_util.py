"""Helpers of the GPU parity tests: row sampling plans and the error metrics of the acceptance bar."""
import numpy as np

from oracle import clear_oracle as orc

# Acceptance bar: bf16 inputs -> max-abs error <= 2e-2 and relative RMS <= 1e-2 against the fp64 oracle;
# fp32 inputs -> both <= 1e-4.  Relative RMS = ||O_gpu - O_ref||_F / ||O_ref||_F over the compared rows.
TOL = {"bf16": (2e-2, 1e-2), "f32": (1e-4, 1e-4)}


def max_abs_bar(dtype, ref):
    """The max-abs bar for outputs of any magnitude.  TOL's 2e-2 is meant for outputs of order one (a softmax average
    over many keys).  A row that averages two or three keys (r = 1, hardly any text) returns values as large as V's
    own, 4 and more, and there the rounding of the bf16 output alone is half an ulp = 2^-9 of the value, the
    rounding of the probabilities to bf16 as much again per term: 2^-7 of the largest reference value bounds both."""
    if dtype != "bf16":
        return TOL[dtype][0]
    return max(TOL[dtype][0], 2.0 ** -7 * float(np.abs(np.asarray(ref)).max()))


def error_metrics(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    diff = got - ref
    return float(np.abs(diff).max()), float(np.sqrt((diff ** 2).sum() / max((ref ** 2).sum(), 1e-300)))


def sample_rows(n_text, gridH, gridW, r, n_random, seed, n_text_rows=None, tile=(16, 16)):
    """Query rows worth checking: text rows, corners, edge midpoints, rows at distance r-1, r, r+1 from each
    border, both sides of query-tile boundaries, the last (possibly ragged) tile, plus seeded random rows."""
    rng = np.random.default_rng(seed)
    rows = set()
    if n_text:
        k = n_text if n_text_rows is None else min(n_text, n_text_rows)
        rows.update(int(x) for x in np.unique(np.concatenate([[0, n_text - 1], rng.integers(0, n_text, size=k)]))[:k + 2])
        if n_text_rows is None:
            rows.update(range(n_text))
    ys = {0, gridH - 1, gridH // 2, r - 1, r, r + 1, gridH - r, gridH - 1 - r, gridH - 2 - r, tile[0] - 1, tile[0],
          (gridH // tile[0]) * tile[0] - 1, (gridH // tile[0]) * tile[0]}
    xs = {0, gridW - 1, gridW // 2, r - 1, r, r + 1, gridW - r, gridW - 1 - r, gridW - 2 - r, tile[1] - 1, tile[1],
          (gridW // tile[1]) * tile[1] - 1, (gridW // tile[1]) * tile[1]}
    for y in ys:
        for x in xs:
            if 0 <= y < gridH and 0 <= x < gridW:
                rows.add(n_text + y * gridW + x)
    n_img = gridH * gridW
    rows.update(int(n_text + p) for p in rng.integers(0, n_img, size=n_random))
    return np.array(sorted(rows), dtype=np.int64)


def oracle_rows_for_heads(Q, K, V, heads, rows, n_text, gridH, gridW, r):
    """Oracle output [len(heads), len(rows), d] for batch item 0.  Q, K, V: torch tensors [B, H, N, d] (any device)."""
    out = []
    for h in heads:
        q, k, v = (t[0, h].detach().cpu().double().numpy() for t in (Q, K, V))
        out.append(orc.attention_rows(q, k, v, rows, n_text, gridH, gridW, r))
    return np.stack(out)
