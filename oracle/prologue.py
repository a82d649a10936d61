"""CPU oracle for the query/key prologue of a FLUX-style attention block: per-head RMS normalisation,
rotary position embedding on the two image axes, and a logit scale (Sec. 3.1 on the rotary embedding and
its relative distances on the two axes; Sec. 4.3 on the rotary frequencies and the attention scale used
for resolution extrapolation).

TEST INFRASTRUCTURE ONLY: imported by tests/ (and nothing else).  Plain numpy in fp64; shares nothing
with the HIP path and does not import it.

The paper names these steps but prints no formula for them; the definitions below are the published
ones of the components it cites, written out:

* RMS normalisation over the head's channels with a learned per-channel gain:
      y_c = x_c * g_c / sqrt(mean_c(x_c^2) + eps).
* Rotary embedding in its original form: channels are taken in adjacent pairs (2i, 2i+1), pair i of a
  token is turned by the token's angle theta_i:
      y_{2i} = cos(theta_i) x_{2i} - sin(theta_i) x_{2i+1},   y_{2i+1} = sin(theta_i) x_{2i} + cos(theta_i) x_{2i+1}.
  The angles arrive as tables, one per image axis: table_y[y, i] = (cos, sin) of the angle the row
  coordinate contributes, table_x[x, i] the same for the column; an image token at (y, x) is turned by
  the sum of the two angles, a text token is not turned at all (position 0 on every axis).  Which
  pairs an axis acts on, the frequencies and any NTK factor are the table maker's business: a pair an
  axis does not act on holds (1, 0).
* The results are rounded to bf16 (round to nearest even), the precision in which the block hands
  queries and keys to the attention operator; attention itself is then the plain definition
  (clear_oracle.attention_rows) on those values.
* The logit scale multiplies q.k / sqrt(c) before the softmax.
"""
import numpy as np


def rms_norm(x, gain, eps):
    """x: [..., c]; gain: [c]."""
    x = np.asarray(x, dtype=np.float64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x * np.asarray(gain, dtype=np.float64) / np.sqrt(ms + eps)


def rotate_pairs(x, cos, sin):
    """x: [..., c]; cos, sin: [..., c/2] (broadcast against x's leading axes)."""
    x = np.asarray(x, dtype=np.float64)
    even, odd = x[..., 0::2], x[..., 1::2]
    out = np.empty_like(x)
    out[..., 0::2] = cos * even - sin * odd
    out[..., 1::2] = sin * even + cos * odd
    return out


def token_rotation(n_text, gridH, gridW, table_y, table_x):
    """(cos, sin), each [N, c/2], of every token's angle: text tokens 0, image token (y, x) the sum of the
    row angle and the column angle (angle addition written out on the cos / sin pairs)."""
    ty = np.asarray(table_y, dtype=np.float64)  # [gridH, c/2, 2]
    tx = np.asarray(table_x, dtype=np.float64)  # [gridW, c/2, 2]
    half = ty.shape[1]
    cy, sy = ty[:, None, :, 0], ty[:, None, :, 1]
    cx, sx = tx[None, :, :, 0], tx[None, :, :, 1]
    cos_img = (cy * cx - sy * sx).reshape(gridH * gridW, half)
    sin_img = (sy * cx + cy * sx).reshape(gridH * gridW, half)
    cos = np.concatenate([np.ones((n_text, half)), cos_img])
    sin = np.concatenate([np.zeros((n_text, half)), sin_img])
    return cos, sin


def round_bf16(x):
    """fp64 -> nearest bf16 (ties to even), returned as fp64.  Values must be zero or normal in bf16."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    assert np.all((x == 0) | ((np.abs(x) > 1e-37) & (np.abs(x) < 1e38)))
    bits = x.view(np.uint64).copy()
    drop = np.uint64(45)  # fp64 keeps 52 fraction bits, bf16 7
    lsb = (bits >> drop) & np.uint64(1)
    bits += (np.uint64(1) << np.uint64(44)) - np.uint64(1) + lsb
    bits &= ~((np.uint64(1) << drop) - np.uint64(1))
    return bits.view(np.float64)


def qk_prologue(x, gain, eps, n_text, gridH, gridW, table_y, table_x):
    """One [N, c] slice of raw queries (or keys) -> what attention sees: normalised, turned, rounded to bf16.
    gain None: no normalisation; tables None: no rotation."""
    y = np.asarray(x, dtype=np.float64)
    if gain is not None:
        y = rms_norm(y, gain, eps)
    if table_y is not None:
        cos, sin = token_rotation(n_text, gridH, gridW, table_y, table_x)
        y = rotate_pairs(y, cos, sin)
    return round_bf16(y)
