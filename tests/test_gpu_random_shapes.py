"""Seeded random shapes through the C ABI against the fp64 oracle, every row of every head: text lengths, grid
extents and radii drawn so that ragged text tiles, ragged query and key tiles, windows cut on one or both sides,
r = 1 and r beyond the grid all turn up in combinations nobody wrote down by hand.  bf16 at both head
dimensions and the fp32 path; the forward pass, its log-sum-exp output, the variant that allocates nothing,
(bf16) the gradients of a few of the shapes, the other masks, and row bands.  CLEAR_RANDOM_SHAPES_FACTOR=k in the
environment draws k times as many cases of every kind (same seeds, so the default cases come first)."""
import os
import sys

import numpy as np
import pytest
import torch

from oracle import clear_oracle as orc
from paper_2412_16112_amd import clear_attn as ca
from paper_2412_16112_amd.inputs import make_qkv_shape
from tests.parity_util import TOL, error_metrics, max_abs_bar

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
FACTOR = max(1, int(os.environ.get("CLEAR_RANDOM_SHAPES_FACTOR", "1")))


def _shapes(seed, n, max_side):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        gh, gw = (int(x) for x in rng.integers(1, max_side + 1, size=2))
        n_text = int(rng.choice([0, 1, 7, 64, 65, 100, 256, 300])) if rng.random() < 0.7 else int(rng.integers(0, 400))
        r = int(rng.choice([1, 2, 3, 5, 8, 16, 17, 33, 100])) if rng.random() < 0.7 else int(rng.integers(1, 48))
        B, H = int(rng.integers(1, 3)), int(rng.integers(1, 4))
        out.append((B, H, n_text, gh, gw, r, 1000 * seed + i))
    return out


def _check_forward(dtype, d, B, H, n_text, gh, gw, r, seed):
    print(f"[case] random shape {dtype} d={d} B={B} H={H} n_text={n_text} grid={gh}x{gw} r={r} seed={seed}", flush=True)
    sys.stdout.flush()
    Q, K, V = make_qkv_shape(B, H, n_text, gh, gw, d, dtype, seed, device="cpu")
    Qd, Kd, Vd = Q.to(DEV), K.to(DEV), V.to(DEV)
    ctx = ca.ClearAttn(n_text, gh, gw, d, r, ca._dtype_code(Qd))
    try:
        O = torch.full_like(Qd, float("nan"))
        ctx.forward(Qd, Kd, Vd, O)
        O2, lse = ctx.forward_lse(Qd, Kd, Vd)
        O3 = torch.full_like(Qd, float("nan"))
        ctx.forward_noalloc(Qd, Kd, Vd, O3)
        torch.cuda.synchronize()
    finally:
        ctx.destroy()
    assert torch.equal(O, O2) and torch.equal(O, O3)
    tol = TOL[dtype]
    N = n_text + gh * gw
    for b in range(B):
        for h in range(H):
            q, k, v = (t[b, h].float().numpy() for t in (Q, K, V))
            ref, m, l, _ = orc.attention_rows(q, k, v, np.arange(N), n_text, gh, gw, r, return_stats=True)
            got = O[b, h].float().cpu().numpy()
            assert np.isfinite(got).all()
            max_abs, rel_rms = error_metrics(got, ref)
            assert max_abs <= max_abs_bar(dtype, ref) and rel_rms <= tol[1], (b, h, max_abs, rel_rms)
            np.testing.assert_allclose(lse[b, h].cpu().numpy(), m + np.log(l), rtol=0, atol=3e-3 if dtype == "bf16" else 1e-4)
    return Qd, Kd, Vd


@pytest.mark.parametrize("B,H,n_text,gh,gw,r,seed", _shapes(1, 14 * FACTOR, 56))
def test_random_shapes_bf16_d128(B, H, n_text, gh, gw, r, seed):
    _check_forward("bf16", 128, B, H, n_text, gh, gw, r, seed)


@pytest.mark.parametrize("B,H,n_text,gh,gw,r,seed", _shapes(2, 10 * FACTOR, 56))
def test_random_shapes_bf16_d64(B, H, n_text, gh, gw, r, seed):
    _check_forward("bf16", 64, B, H, n_text, gh, gw, r, seed)


@pytest.mark.parametrize("B,H,n_text,gh,gw,r,seed", _shapes(3, 6 * FACTOR, 40))
def test_random_shapes_f32(B, H, n_text, gh, gw, r, seed):
    _check_forward("f32", 64, B, H, n_text, gh, gw, r, seed)


@pytest.mark.parametrize("B,H,n_text,gh,gw,r,seed", _shapes(4, 6 * FACTOR, 36))
def test_random_shapes_backward(B, H, n_text, gh, gw, r, seed):
    d = 128
    print(f"[case] random shape backward B={B} H={H} n_text={n_text} grid={gh}x{gw} r={r} seed={seed}", flush=True)
    Q, K, V = make_qkv_shape(B, H, n_text, gh, gw, d, "bf16", seed, device=DEV)
    g = torch.Generator(device=DEV).manual_seed(seed + 7)
    dO = torch.randn(Q.shape, generator=g, device=DEV, dtype=torch.float32).to(torch.bfloat16)
    ctx = ca.ClearAttn(n_text, gh, gw, d, r, ca.CLEAR_BF16)
    try:
        O, lse = ctx.forward_lse(Q, K, V)
        dQ, dK, dV = ctx.backward(Q, K, V, O, dO, lse)
        torch.cuda.synchronize()
    finally:
        ctx.destroy()
    N = n_text + gh * gw
    idx = np.arange(N)
    for b in range(B):
        for h in range(H):
            q, k, v, go = (t[b, h].float().cpu().numpy() for t in (Q, K, V, dO))
            refs = (orc.backward_dq_rows(q, k, v, go, idx, n_text, gh, gw, r),) + tuple(orc.backward_dkv_cols(q, k, v, go, idx, n_text, gh, gw, r))
            for name, got, ref in zip(("dQ", "dK", "dV"), (dQ, dK, dV), refs):
                got = got[b, h].float().cpu().numpy()
                max_abs, rel_rms = error_metrics(got, ref)
                scale = float(np.abs(ref).max())
                assert np.isfinite(got).all()
                if scale < 1e-4:
                    # a gradient that vanishes identically (r = 1 without text: every token sees only itself, P = 1 and
                    # dS = dP - delta = 0): what is left is the rounding of two fp32 sums taken in different orders
                    assert max_abs <= 1e-4, (name, b, h, max_abs, scale)
                else:
                    assert max_abs <= TOL["bf16"][0] * scale and rel_rms <= TOL["bf16"][1], (name, b, h, max_abs, scale, rel_rms)


def _mask_shapes(seed, n, max_side):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        kind = int(rng.choice([orc.MASK_SQUARE, orc.MASK_SWIN, orc.MASK_STRIDED]))
        r = int(rng.choice([1, 2, 4, 5, 8, 16])) if kind != orc.MASK_STRIDED else int(rng.choice([1, 2, 3, 4, 8]))
        lo = r if kind == orc.MASK_STRIDED else 1  # the strided mask needs every residue class non-empty
        gh, gw = (int(x) for x in rng.integers(lo, max(lo, max_side) + 1, size=2))
        shift = int(rng.integers(0, r)) if kind == orc.MASK_SWIN else (int(rng.integers(0, 2 * r * r)) if kind == orc.MASK_STRIDED else 0)
        n_text = int(rng.choice([0, 5, 64, 130]))
        out.append((kind, shift, int(rng.integers(1, 3)), n_text, gh, gw, r, int(rng.choice([64, 128])), 7000 + 100 * seed + i))
    return out


@pytest.mark.parametrize("kind,shift,H,n_text,gh,gw,r,d,seed", _mask_shapes(5, 14 * FACTOR, 48))
def test_random_shapes_other_masks(kind, shift, H, n_text, gh, gw, r, d, seed):
    print(f"[case] random shape mask kind={kind} shift={shift} d={d} H={H} n_text={n_text} grid={gh}x{gw} r={r} seed={seed}", flush=True)
    Q, K, V = make_qkv_shape(1, H, n_text, gh, gw, d, "bf16", seed, device="cpu")
    ctx = ca.ClearAttn(n_text, gh, gw, d, r, ca.CLEAR_BF16, kind, shift)  # (the two sides number the mask kinds alike)
    try:
        O = torch.full(Q.shape, float("nan"), dtype=Q.dtype, device=DEV)
        ctx.forward(Q.to(DEV), K.to(DEV), V.to(DEV), O)
        torch.cuda.synchronize()
    finally:
        ctx.destroy()
    with orc.mask_kind(kind, shift):
        ref = orc.attention(Q, K, V, n_text, gh, gw, r)
    got = O.float().cpu().numpy()
    assert np.isfinite(got).all()
    max_abs, rel_rms = error_metrics(got, ref)
    assert max_abs <= max_abs_bar("bf16", ref) and rel_rms <= TOL["bf16"][1], (max_abs, rel_rms)


def _band_shapes(seed, n):
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < n:
        r = int(rng.choice([2, 3, 5, 8, 16]))
        n_bands = int(rng.integers(2, 6))
        gh = int(rng.integers(n_bands * max(r - 1, 1), n_bands * max(r - 1, 1) + 40))
        gw = int(rng.integers(1, 50))
        out.append((int(rng.choice([0, 9, 64, 100])), gh, gw, r, n_bands, int(rng.choice([64, 128])), 9000 + 100 * seed + len(out)))
    return out


@pytest.mark.parametrize("n_text,gh,gw,r,n_bands,d,seed", _band_shapes(6, 8 * FACTOR))
def test_random_shapes_row_bands(n_text, gh, gw, r, n_bands, d, seed):
    """Every band of a random cut, exact text merge, against the oracle of the undivided problem."""
    from tests.test_gpu_bands import run_bands
    print(f"[case] random bands n_text={n_text} grid={gh}x{gw} r={r} bands={n_bands} d={d} seed={seed}", flush=True)
    Q, K, V = make_qkv_shape(1, 2, n_text, gh, gw, d, "bf16", seed, device=DEV)
    O = run_bands(Q, K, V, n_text, gh, gw, r, n_bands, ca.CLEAR_MERGE_EXACT)
    ref = orc.attention(Q.float().cpu().numpy(), K.float().cpu().numpy(), V.float().cpu().numpy(), n_text, gh, gw, r)
    max_abs, rel_rms = error_metrics(O.float().cpu().numpy(), ref)
    assert max_abs <= max_abs_bar("bf16", ref) and rel_rms <= TOL["bf16"][1], (max_abs, rel_rms)
