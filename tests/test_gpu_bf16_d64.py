"""The bf16 kernels at head_dim 64 (an SD3.5-style head) against the fp64 oracle: the same code path as
head_dim 128 with 128-byte token rows, so the cases aim at what differs -- the LDS layout and swizzle of
staged tiles, operand addresses, the shorter matrix pipeline, four tiles per stage."""
import numpy as np
import pytest
import torch

from oracle import clear_oracle as orc
from oracle import prologue as pro
from paper_2412_16112_amd import clear_attn as ca
from paper_2412_16112_amd.inputs import WORKLOADS, make_prologue_inputs, make_qkv, make_qkv_shape
from tests.parity_util import TOL, error_metrics, oracle_rows_for_heads, sample_rows

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def full_compare(B, H, n_text, gh, gw, r, seed, q_scale=1.0, mask_kind=ca.CLEAR_MASK_DISC, shift=0):
    print(f"[case] d64 B={B} H={H} n_text={n_text} grid={gh}x{gw} r={r} seed={seed} mask={mask_kind}/{shift}", flush=True)
    Q, K, V = make_qkv_shape(B, H, n_text, gh, gw, 64, "bf16", seed, device="cpu", q_scale=q_scale)
    ctx = ca.ClearAttn(n_text, gh, gw, 64, r, ca.CLEAR_BF16, mask_kind, shift)
    try:
        O = ctx.forward(Q.to(DEV), K.to(DEV), V.to(DEV))
        torch.cuda.synchronize()
    finally:
        ctx.destroy()
    with orc.mask_kind(mask_kind, shift):
        ref = orc.attention(Q, K, V, n_text, gh, gw, r)
    O = O.float().cpu().numpy()
    assert np.isfinite(O).all()
    mx, rms = error_metrics(O, ref)
    assert mx <= TOL["bf16"][0] and rms <= TOL["bf16"][1], (mx, rms)


@pytest.mark.parametrize("B,H,n_text,gh,gw,r", [
    (1, 1, 8, 16, 16, 4),
    (2, 3, 40, 20, 28, 4),     # ragged text tile, ragged query and key tiles
    (1, 2, 0, 33, 17, 9),      # no text tokens
    (1, 2, 5, 7, 5, 1),        # r = 1
    (1, 1, 70, 24, 40, 100),   # full attention
    (1, 2, 300, 9, 70, 32),    # thin grid
    (1, 1, 1, 1, 1, 3),        # one image token
    (1, 2, 333, 48, 48, 16),   # SD3.5-like text length, several query tiles
    (1, 1, 64, 40, 72, 8),
    (1, 1, 1000, 24, 24, 6),   # long text part: many linear stages of four tiles, ragged last stage
])
def test_small_cases(B, H, n_text, gh, gw, r):
    full_compare(B, H, n_text, gh, gw, r, seed=300 + gh)


def test_sharp_logits():
    full_compare(1, 2, 96, 32, 32, 8, seed=7, q_scale=4.0)


@pytest.mark.parametrize("q_scale", [60.0, 400.0])
def test_extreme_logits_take_the_careful_pass(q_scale):
    full_compare(1, 2, 64, 24, 40, 6, seed=9, q_scale=q_scale)


@pytest.mark.parametrize("kind,shift", [(ca.CLEAR_MASK_SQUARE, 0), (ca.CLEAR_MASK_SWIN, 0), (ca.CLEAR_MASK_SWIN, 4)])
def test_other_masks(kind, shift):
    full_compare(1, 2, 21, 37, 29, 8, seed=17, mask_kind=kind, shift=shift)


def test_every_channel_and_key_slot_is_wired_right():
    """One-hot V rows: output channel c of a query is the softmax mass of the keys whose V row is e_c, so a
    misplaced chunk, slice or key slot shows up as mass in the wrong channel."""
    n_text, gh, gw, r = 64, 16, 16, 5
    Q, K, _ = make_qkv_shape(1, 1, n_text, gh, gw, 64, "bf16", seed=23, device="cpu")
    N = n_text + gh * gw
    V = torch.zeros(1, 1, N, 64, dtype=torch.bfloat16)
    V[0, 0, torch.arange(N), (torch.arange(N) * 7 + 3) % 64] = 1.0
    O = ca.clear_attn_forward_once(Q.to(DEV), K.to(DEV), V.to(DEV), n_text, gh, gw, r).float().cpu().numpy()
    ref = orc.attention(Q, K, V, n_text, gh, gw, r)
    mx, rms = error_metrics(O, ref)
    assert mx <= TOL["bf16"][0] and rms <= TOL["bf16"][1], (mx, rms)


def test_lse_and_bands_and_prologue_at_d64():
    n_text, gh, gw, r, H = 50, 40, 24, 8, 2
    Q, K, V = make_qkv_shape(1, H, n_text, gh, gw, 64, "bf16", seed=31, device=DEV, q_scale=2.0)
    gq, gk, ty, tx = make_prologue_inputs(gh, gw, 64, seed=32, device=DEV)
    f64 = lambda t: None if t is None else t.detach().cpu().double().numpy()
    ctx = ca.ClearAttn(n_text, gh, gw, 64, r, ca.CLEAR_BF16)
    try:
        O, lse = ctx.forward_lse(Q, K, V)
        Op = ctx.forward_prologue(Q, K, V, q_gain=gq, k_gain=gk, rope_y=ty, rope_x=tx, logit_scale=1.2)
        torch.cuda.synchronize()
    finally:
        ctx.destroy()
    N = n_text + gh * gw
    for h in range(H):
        ref, m, l, _ = orc.attention_rows(f64(Q[0, h]), f64(K[0, h]), f64(V[0, h]), np.arange(N), n_text, gh, gw, r, return_stats=True)
        mx, rms = error_metrics(f64(O[0, h]), ref)
        assert mx <= TOL["bf16"][0] and rms <= TOL["bf16"][1], (mx, rms)
        assert np.abs(f64(lse[0, h]) - (m + np.log(l))).max() <= 5e-3
        qp = pro.qk_prologue(f64(Q[0, h]), f64(gq), 1e-6, n_text, gh, gw, f64(ty), f64(tx))
        kp = pro.qk_prologue(f64(K[0, h]), f64(gk), 1e-6, n_text, gh, gw, f64(ty), f64(tx))
        refp = orc.attention_rows(qp * 1.2, kp, f64(V[0, h]), np.arange(N), n_text, gh, gw, r)
        mx, rms = error_metrics(f64(Op[0, h]), refp)
        assert mx <= TOL["bf16"][0] and rms <= TOL["bf16"][1], (mx, rms)


def sampled(name, heads, n_random, n_text_rows):
    w = WORKLOADS[name]
    print(f"[case] workload {name} heads={heads}", flush=True)
    Q, K, V = make_qkv(w, DEV)
    ctx = ca.ClearAttn(w.n_text, w.gridH, w.gridW, w.head_dim, w.r, ca.CLEAR_BF16)
    try:
        O = ctx.forward(Q, K, V)
        torch.cuda.synchronize()
        O2 = ctx.forward(Q, K, V)
        torch.cuda.synchronize()
        assert torch.equal(O.view(torch.int16), O2.view(torch.int16))
    finally:
        ctx.destroy()
    rows = sample_rows(w.n_text, w.gridH, w.gridW, w.r, n_random, seed=w.seed, n_text_rows=n_text_rows)
    ref = oracle_rows_for_heads(Q, K, V, heads, rows, w.n_text, w.gridH, w.gridW, w.r)
    got = O[0][heads][:, torch.from_numpy(rows).to(DEV)].float().cpu().numpy()
    mx, rms = error_metrics(got, ref)
    print(f"[result] {name}: rows={len(rows)} max_abs={mx:.3e} rel_rms={rms:.3e}", flush=True)
    assert mx <= TOL["bf16"][0] and rms <= TOL["bf16"][1], (mx, rms)
    assert torch.isfinite(O.float()).all()


def test_sd35l_1024_sampled():
    sampled("sd35l-1024-r16", [0, 19, 37], 600, None)


def test_sd35l_4096_sampled():
    sampled("sd35l-4096-r16", [0, 37], 1024, 64)


@pytest.mark.parametrize("n_text,gh,gw,r,H,kind,shift", [
    (37, 40, 24, 8, 2, ca.CLEAR_MASK_DISC, 0),
    (0, 33, 17, 9, 1, ca.CLEAR_MASK_DISC, 0),
    (333, 48, 48, 16, 1, ca.CLEAR_MASK_DISC, 0),
    (21, 37, 29, 8, 1, ca.CLEAR_MASK_SWIN, 4),
    (37, 21, 30, 4, 1, ca.CLEAR_MASK_STRIDED, 6),
])
def test_backward_at_d64(n_text, gh, gw, r, H, kind, shift):
    Q, K, V = make_qkv_shape(1, H, n_text, gh, gw, 64, "bf16", seed=600 + gh, device=DEV)
    g = torch.Generator(device=DEV).manual_seed(601)
    dO = torch.randn(Q.shape, generator=g, device=DEV, dtype=torch.float32).to(torch.bfloat16)
    ctx = ca.ClearAttn(n_text, gh, gw, 64, r, ca.CLEAR_BF16, kind, shift)
    try:
        O, lse = ctx.forward_lse(Q, K, V)
        dQ, dK, dV = ctx.backward(Q, K, V, O, dO, lse)
        torch.cuda.synchronize()
    finally:
        ctx.destroy()
    for h in range(H):
        q, k, v, go = (t[0, h].float().cpu().numpy() for t in (Q, K, V, dO))
        with orc.mask_kind(kind, shift):
            rQ, rK, rV = orc.backward(q, k, v, go, n_text, gh, gw, r)
        for name, got, ref in (("dQ", dQ, rQ), ("dK", dK, rK), ("dV", dV, rV)):
            got = got[0, h].float().cpu().numpy()
            assert np.isfinite(got).all()
            mx, rms = error_metrics(got, ref)
            assert mx <= TOL["bf16"][0] * np.abs(ref).max() and rms <= TOL["bf16"][1], (name, h, mx, rms)
