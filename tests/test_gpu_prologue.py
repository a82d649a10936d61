"""Query/key prologue on the GPU (RMS norm, rotary embedding, bf16 hand-over, logit scale) against the CPU
oracle: the pass of its own element by element, and the fused forward pass on sampled and on all rows."""
import numpy as np
import pytest
import torch

from oracle import clear_oracle as orc
from oracle import prologue as pro
from paper_2412_16112_amd import clear_attn as ca
from paper_2412_16112_amd.inputs import make_prologue_inputs, make_qkv_shape
from tests.parity_util import TOL, error_metrics, sample_rows

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
BF16_ULP = 2.0 ** -7  # spacing of bf16 relative to the binade's lower end


def tables(gridH, gridW, d, seed, ntk=1.0):
    return make_prologue_inputs(gridH, gridW, d, seed, ntk_factor=ntk, device=DEV)


def np64(t):
    return None if t is None else t.detach().cpu().double().numpy()


def check_rounded(got, ref):
    """The device works in fp32 and rounds once to bf16; the oracle in fp64 and rounds once: values may differ by
    one bf16 step where the exact value lies next to a rounding boundary, nowhere by more."""
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    step = BF16_ULP * np.maximum(np.abs(ref), 2.0 ** -20)
    assert np.all(np.abs(got - ref) <= step * 1.001)
    assert np.mean(got != ref) < 0.02


@pytest.mark.parametrize("d", [128, 64])
@pytest.mark.parametrize("norm,rope", [(True, True), (True, False), (False, True), (False, False)])
def test_qk_prologue_pass(d, norm, rope):
    n_text, gridH, gridW, B, H = 37, 19, 23, 2, 3
    X, _, _ = make_qkv_shape(B, H, n_text, gridH, gridW, d, "bf16", seed=21, device=DEV, q_scale=3.0)
    gq, _, ty, tx = tables(gridH, gridW, d, 22, ntk=10.0)
    g = gq if norm else None
    ry, rx = (ty, tx) if rope else (None, None)
    Y = ca.clear_attn_qk_prologue(X, n_text, gridH, gridW, gain=g, norm_eps=1e-6, rope_y=ry, rope_x=rx)
    torch.cuda.synchronize()
    for b in range(B):
        for h in range(H):
            ref = pro.qk_prologue(np64(X[b, h]), np64(g), 1e-6, n_text, gridH, gridW, np64(ry), np64(rx))
            if not norm and not rope:
                assert np.array_equal(np64(Y[b, h]), ref)
            else:
                check_rounded(np64(Y[b, h]), ref)
    # in place
    Z = X.clone()
    ca.clear_attn_qk_prologue(Z, n_text, gridH, gridW, gain=g, norm_eps=1e-6, rope_y=ry, rope_x=rx, out=Z)
    torch.cuda.synchronize()
    assert torch.equal(Z, Y)


FWD_CASES = [
    # n_text, gridH, gridW, r, H, norm, rope, logit_scale, ntk
    (64, 40, 24, 8, 2, True, True, 1.0, 1.0),
    (77, 37, 53, 6, 1, True, True, 1.25, 10.0),
    (0, 48, 32, 8, 1, True, True, 1.0, 1.0),
    (33, 32, 32, 16, 1, True, False, 0.8, 1.0),
    (33, 32, 32, 16, 1, False, True, 1.0, 1.0),
    (33, 32, 32, 16, 1, False, False, 1.5, 1.0),
]


@pytest.mark.parametrize("n_text,gridH,gridW,r,H,norm,rope,logit_scale,ntk", FWD_CASES)
def test_forward_prologue_all_rows(n_text, gridH, gridW, r, H, norm, rope, logit_scale, ntk):
    d = 128
    Q, K, V = make_qkv_shape(1, H, n_text, gridH, gridW, d, "bf16", seed=31 + n_text, device=DEV, q_scale=2.0)
    gq, gk, ty, tx = tables(gridH, gridW, d, 32, ntk)
    if not norm:
        gq = gk = None
        # without the normalisation raw N(0, 4) queries would give logits in the hundreds: scale them down
        Q = (Q.float() * 0.5).to(torch.bfloat16)
    ry, rx = (ty, tx) if rope else (None, None)
    ctx = ca.ClearAttn(n_text, gridH, gridW, d, r, ca.CLEAR_BF16)
    try:
        K_before = K.clone()
        O = ctx.forward_prologue(Q, K, V, q_gain=gq, k_gain=gk, norm_eps=1e-6, rope_y=ry, rope_x=rx, logit_scale=logit_scale)
        torch.cuda.synchronize()
        assert torch.equal(K, K_before)
        # a second call on the same context (workspace reuse) gives the same bits
        O2 = ctx.forward_prologue(Q, K, V, q_gain=gq, k_gain=gk, norm_eps=1e-6, rope_y=ry, rope_x=rx, logit_scale=logit_scale)
        torch.cuda.synchronize()
        assert torch.equal(O, O2)
    finally:
        ctx.destroy()
    N = n_text + gridH * gridW
    tol_abs, tol_rms = TOL["bf16"]
    for h in range(H):
        qp = pro.qk_prologue(np64(Q[0, h]), np64(gq), 1e-6, n_text, gridH, gridW, np64(ry), np64(rx))
        kp = pro.qk_prologue(np64(K[0, h]), np64(gk), 1e-6, n_text, gridH, gridW, np64(ry), np64(rx))
        ref = orc.attention_rows(qp * logit_scale, kp, np64(V[0, h]), np.arange(N), n_text, gridH, gridW, r)
        mx, rms = error_metrics(np64(O[0, h]), ref)
        assert mx <= tol_abs and rms <= tol_rms, (h, mx, rms)


def test_forward_prologue_flux_1024_sampled():
    n_text, gridH, gridW, d, r, H = 512, 64, 64, 128, 16, 24
    Q, K, V = make_qkv_shape(1, H, n_text, gridH, gridW, d, "bf16", seed=41, device=DEV, q_scale=2.0)
    gq, gk, ty, tx = tables(gridH, gridW, d, 42, ntk=10.0)
    scale = float(np.sqrt(np.log(n_text + gridH * gridW) / np.log(n_text + 64 * 64)))  # a log-ratio factor; 1 at the native size
    scale = 1.1 * scale
    ctx = ca.ClearAttn(n_text, gridH, gridW, d, r, ca.CLEAR_BF16)
    try:
        O = ctx.forward_prologue(Q, K, V, q_gain=gq, k_gain=gk, rope_y=ty, rope_x=tx, logit_scale=scale)
        torch.cuda.synchronize()
    finally:
        ctx.destroy()
    rows = sample_rows(n_text, gridH, gridW, r, n_random=150, seed=43, n_text_rows=24)
    tol_abs, tol_rms = TOL["bf16"]
    for h in (0, 11, 23):
        qp = pro.qk_prologue(np64(Q[0, h]), np64(gq), 1e-6, n_text, gridH, gridW, np64(ty), np64(tx))
        kp = pro.qk_prologue(np64(K[0, h]), np64(gk), 1e-6, n_text, gridH, gridW, np64(ty), np64(tx))
        ref = orc.attention_rows(qp * scale, kp, np64(V[0, h]), rows, n_text, gridH, gridW, r)
        mx, rms = error_metrics(np64(O[0, h])[rows], ref)
        assert mx <= tol_abs and rms <= tol_rms, (h, mx, rms)


def test_forward_prologue_matches_the_two_pass_route():
    """Fused call against: prologue pass on Q and on K, then the plain forward (logit scale 1)."""
    n_text, gridH, gridW, d, r = 50, 33, 47, 128, 8
    Q, K, V = make_qkv_shape(1, 2, n_text, gridH, gridW, d, "bf16", seed=51, device=DEV, q_scale=2.0)
    gq, gk, ty, tx = tables(gridH, gridW, d, 52)
    ctx = ca.ClearAttn(n_text, gridH, gridW, d, r, ca.CLEAR_BF16)
    try:
        O1 = ctx.forward_prologue(Q, K, V, q_gain=gq, k_gain=gk, rope_y=ty, rope_x=tx)
        Qp = ca.clear_attn_qk_prologue(Q, n_text, gridH, gridW, gain=gq, rope_y=ty, rope_x=tx)
        Kp = ca.clear_attn_qk_prologue(K, n_text, gridH, gridW, gain=gk, rope_y=ty, rope_x=tx)
        O2 = ctx.forward(Qp, Kp, V)
        torch.cuda.synchronize()
    finally:
        ctx.destroy()
    # same arithmetic on both routes up to the compiler's choice of fused multiply-adds
    mx, rms = error_metrics(np64(O1), np64(O2))
    assert mx <= 2e-2 and rms <= 2e-3, (mx, rms)


def test_forward_prologue_argument_checks():
    n_text, gridH, gridW, r = 8, 16, 16, 4
    Q, K, V = make_qkv_shape(1, 1, n_text, gridH, gridW, 128, "bf16", seed=61, device=DEV)
    gq, gk, ty, tx = tables(gridH, gridW, 128, 62)
    ctx = ca.ClearAttn(n_text, gridH, gridW, 128, r, ca.CLEAR_BF16)
    try:
        with pytest.raises(ca.ClearAttnError) as e:
            ctx.forward_prologue(Q, K, V, rope_y=ty)
        assert e.value.status == ca.CLEAR_ERR_INVALID_ARG
        with pytest.raises(ca.ClearAttnError) as e:
            ctx.forward_prologue(Q, K, V, q_gain=gq, logit_scale=0.0)
        assert e.value.status == ca.CLEAR_ERR_INVALID_ARG
        with pytest.raises(ca.ClearAttnError):
            ctx.forward_prologue(Q, K, V, rope_y=ty[:, :32], rope_x=tx)
    finally:
        ctx.destroy()
    Qf, Kf, Vf = make_qkv_shape(1, 1, n_text, gridH, gridW, 64, "f32", seed=63, device=DEV)
    ctx = ca.ClearAttn(n_text, gridH, gridW, 64, r, ca.CLEAR_F32)
    try:
        with pytest.raises(ca.ClearAttnError) as e:
            ctx.forward_prologue(Qf, Kf, Vf, logit_scale=1.0)
        assert e.value.status == ca.CLEAR_ERR_UNSUPPORTED
    finally:
        ctx.destroy()
