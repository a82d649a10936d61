"""CPU oracle for row-band ("patch-parallel") inference of the CLEAR attention layer: the section on
multi-GPU parallel inference and its Eq. 7.

TEST INFRASTRUCTURE ONLY: imported by tests/ (and nothing else).  Plain numpy in fp64, no blocking, no
tricks; shares nothing with the HIP path and does not import it.

The feature map of gridH x gridW image tokens is cut along the vertical axis into bands of whole rows,
one per GPU; band p holds image rows [y0_p, y1_p).  Every GPU also holds the n_text text tokens.

* Image queries: the local window of Eq. 3 only ever reaches r - 1 rows beyond a band, so an image
  query's output under band parallelism is exactly its output in the undivided problem.  Nothing new
  to define: the plain definition (clear_oracle.attention_rows) is the oracle.

* Text queries need every image key.  Eq. 7 replaces that by the average over the bands of the softmax
  attention of the text queries over band p's own keys:
      O_text ~= (1/N) sum_p softmax(Q_text K_p^T / sqrt(c)) V_p.
  Reading taken here (the paper does not spell K_p out): K_p, V_p are the keys and values GPU p holds
  as its own, i.e. all text tokens followed by the image tokens of band p (no halo rows).

* The exact alternative: the same per-band softmax outputs combined with weights proportional to the
  per-band softmax denominators.  With a band's text keys counted once (in band 0 only) this equals the
  plain definition; `merge_exact` below is that combination written out, for testing a merge on its own.
"""
import numpy as np


def band_rows(gridH, n_bands):
    """Bands of whole rows, as even as possible, larger ones first: [(y0, y1), ...]."""
    base, extra = divmod(gridH, n_bands)
    out, y = [], 0
    for p in range(n_bands):
        h = base + (1 if p < extra else 0)
        out.append((y, y + h))
        y += h
    return out


def _band_keys(n_text, gridW, y0, y1, with_text=True):
    img = n_text + np.arange(y0 * gridW, y1 * gridW, dtype=np.int64)
    return np.concatenate([np.arange(n_text, dtype=np.int64), img]) if with_text else img


def text_rows_per_band(Q, K, V, n_text, gridW, bands, text_in_band=None):
    """Per band: softmax(Q_text K_p^T / sqrt(d)) V_p and the natural log of the softmax denominator.

    Q, K, V: [N, d] of one (batch, head), any float type (widened to fp64 exactly).
    text_in_band: for each band, whether its key set includes the text keys (default: all do).
    Returns (O_p [n_bands, n_text, d], lse_p [n_bands, n_text])."""
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    d = Q.shape[1]
    if text_in_band is None:
        text_in_band = [True] * len(bands)
    outs, lses = [], []
    for (y0, y1), with_text in zip(bands, text_in_band):
        keys = _band_keys(n_text, gridW, y0, y1, with_text)
        s = (Q[:n_text] @ K[keys].T) / np.sqrt(float(d))
        m = s.max(axis=1, keepdims=True)
        e = np.exp(s - m)
        den = e.sum(axis=1, keepdims=True)
        outs.append((e @ V[keys]) / den)
        lses.append((np.log(den) + m)[:, 0])
    return np.stack(outs), np.stack(lses)


def text_rows_average(Q, K, V, n_text, gridW, bands):
    """Eq. 7: the plain mean over the bands of the per-band softmax outputs (each band: text + own image keys)."""
    O_p, _ = text_rows_per_band(Q, K, V, n_text, gridW, bands)
    return O_p.mean(axis=0)


def merge_exact(O_p, lse_p):
    """Combination of per-band softmax outputs over DISJOINT key sets into the softmax over their union:
    weights exp(lse_p) / sum_p exp(lse_p).  O_p: [n_bands, rows, d], lse_p: [n_bands, rows]."""
    O_p = np.asarray(O_p, dtype=np.float64)
    lse_p = np.asarray(lse_p, dtype=np.float64)
    w = np.exp(lse_p - lse_p.max(axis=0, keepdims=True))
    w = w / w.sum(axis=0, keepdims=True)
    return (w[:, :, None] * O_p).sum(axis=0)
