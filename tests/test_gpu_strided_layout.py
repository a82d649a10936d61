"""Tensors in other layouts through clear_attn_forward_strided: [B, N, H, d] storage seen as [B, H, N, d] views, slices
of a packed QKV tensor, keys shared by all heads.  The kernels only change their address arithmetic, so the results
must equal the plain-layout results bit for bit; one case is also held against the oracle directly."""
import numpy as np
import pytest
import torch

from oracle import clear_oracle as orc
from paper_2412_16112_amd import clear_attn as ca
from paper_2412_16112_amd.inputs import make_prologue_inputs, make_qkv_shape
from tests.parity_util import TOL, error_metrics

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def token_major(t):
    """A [B, H, N, d] view of a fresh [B, N, H, d] tensor holding the same values."""
    return t.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)


@pytest.mark.parametrize("d,B,H,n_text,gh,gw,r,kind,shift", [
    (128, 2, 3, 40, 20, 28, 4, ca.CLEAR_MASK_DISC, 0),
    (128, 1, 2, 96, 33, 47, 8, ca.CLEAR_MASK_DISC, 0),
    (64, 1, 3, 77, 37, 29, 6, ca.CLEAR_MASK_DISC, 0),
    (128, 1, 2, 21, 37, 29, 8, ca.CLEAR_MASK_SWIN, 4),
    (128, 1, 2, 37, 21, 30, 4, ca.CLEAR_MASK_STRIDED, 6),
])
def test_token_major_storage_matches_plain_layout(d, B, H, n_text, gh, gw, r, kind, shift):
    Q, K, V = make_qkv_shape(B, H, n_text, gh, gw, d, "bf16", seed=700 + gh, device=DEV)
    Qs, Ks, Vs = token_major(Q), token_major(K), token_major(V)
    assert not Qs.is_contiguous() and Qs.stride(2) == H * d
    ctx = ca.ClearAttn(n_text, gh, gw, d, r, ca.CLEAR_BF16, kind, shift)
    try:
        O = ctx.forward(Q, K, V)
        Os = ctx.forward_strided(Qs, Ks, Vs)
        torch.cuda.synchronize()
    finally:
        ctx.destroy()
    assert Os.stride() == Qs.stride()
    assert torch.equal(O.view(torch.int16), Os.contiguous().view(torch.int16))
    with orc.mask_kind(kind, shift):
        ref = orc.attention(Q, K, V, n_text, gh, gw, r)
    mx, rms = error_metrics(Os.float().cpu().numpy(), ref)
    assert mx <= TOL["bf16"][0] and rms <= TOL["bf16"][1], (mx, rms)


def test_slices_of_a_packed_qkv_tensor_and_shared_keys():
    B, H, n_text, gh, gw, d, r = 1, 4, 50, 24, 40, 128, 8
    N = n_text + gh * gw
    Q, K, V = make_qkv_shape(B, H, n_text, gh, gw, d, "bf16", seed=710, device=DEV)
    packed = torch.empty(B, N, 3, H, d, dtype=torch.bfloat16, device=DEV)
    for i, t in enumerate((Q, K, V)):
        packed[:, :, i] = t.permute(0, 2, 1, 3)
    Qs, Ks, Vs = (packed[:, :, i].permute(0, 2, 1, 3) for i in range(3))
    assert Qs.stride(2) == 3 * H * d
    out = torch.full((B, N, H, d), float("nan"), dtype=torch.bfloat16, device=DEV)
    ctx = ca.ClearAttn(n_text, gh, gw, d, r, ca.CLEAR_BF16)
    try:
        O = ctx.forward(Q, K, V)
        Os = ctx.forward_strided(Qs, Ks, Vs, out.permute(0, 2, 1, 3))
        # keys and values of head 0 used by every head (head stride 0)
        K0, V0 = K[:, :1].expand(B, H, N, d), V[:, :1].expand(B, H, N, d)
        assert K0.stride(1) == 0
        Oshared = ctx.forward_strided(Q, K0, V0)
        Oshared_ref = ctx.forward(Q, K0.contiguous(), V0.contiguous())
        torch.cuda.synchronize()
    finally:
        ctx.destroy()
    assert torch.equal(O, out.permute(0, 2, 1, 3).contiguous())
    assert torch.equal(Oshared, Oshared_ref)


def test_strided_layout_with_the_prologue():
    B, H, n_text, gh, gw, d, r = 1, 2, 33, 26, 19, 128, 6
    Q, K, V = make_qkv_shape(B, H, n_text, gh, gw, d, "bf16", seed=720, device=DEV, q_scale=2.0)
    gq, gk, ty, tx = make_prologue_inputs(gh, gw, d, seed=721, device=DEV)
    ctx = ca.ClearAttn(n_text, gh, gw, d, r, ca.CLEAR_BF16)
    try:
        O = ctx.forward_prologue(Q, K, V, q_gain=gq, k_gain=gk, rope_y=ty, rope_x=tx, logit_scale=1.1)
        Os = ctx.forward_strided(token_major(Q), token_major(K), token_major(V), q_gain=gq, k_gain=gk, rope_y=ty, rope_x=tx, logit_scale=1.1)
        torch.cuda.synchronize()
    finally:
        ctx.destroy()
    assert torch.equal(O, Os.contiguous())


def test_stride_argument_checks():
    B, H, n_text, gh, gw, d, r = 1, 2, 8, 16, 16, 128, 4
    N = n_text + gh * gw
    Q, K, V = make_qkv_shape(B, H, n_text, gh, gw, d, "bf16", seed=730, device=DEV)
    ctx = ca.ClearAttn(n_text, gh, gw, d, r, ca.CLEAR_BF16)
    try:
        # token stride that is not a multiple of 8 elements
        buf = torch.zeros(B * H * N * (d + 4) + 64, dtype=torch.bfloat16, device=DEV)
        odd = buf.as_strided((B, H, N, d), (H * N * (d + 4), N * (d + 4), d + 4, 1))
        with pytest.raises(ca.ClearAttnError) as e:
            ctx.forward_strided(odd, K, V)
        assert e.value.status == ca.CLEAR_ERR_INVALID_ARG
        # O inside the span of Q
        with pytest.raises(ca.ClearAttnError) as e:
            ctx.forward_strided(Q, K, V, Q)
        assert e.value.status == ca.CLEAR_ERR_INVALID_ARG
        # channels not contiguous: refused by the binding
        with pytest.raises(ca.ClearAttnError):
            ctx.forward_strided(Q.transpose(2, 3).contiguous().transpose(2, 3), K, V)
    finally:
        ctx.destroy()
    Qf, Kf, Vf = make_qkv_shape(1, 1, n_text, gh, gw, 64, "f32", seed=731, device=DEV)
    ctx = ca.ClearAttn(n_text, gh, gw, 64, r, ca.CLEAR_F32)
    try:
        with pytest.raises(ca.ClearAttnError) as e:
            ctx.forward_strided(Qf, Kf, Vf)
        assert e.value.status == ca.CLEAR_ERR_UNSUPPORTED
    finally:
        ctx.destroy()


@pytest.mark.parametrize("d", [128, 64])
def test_training_pair_in_token_major_storage(d):
    """forward with log-sum-exp + backward on [B, N, H, d] storage: same bits as the plain layout."""
    B, H, n_text, gh, gw, r = 2, 2, 40, 24, 28, 6
    Q, K, V = make_qkv_shape(B, H, n_text, gh, gw, d, "bf16", seed=740 + d, device=DEV)
    g = torch.Generator(device=DEV).manual_seed(741)
    dO = torch.randn(Q.shape, generator=g, device=DEV, dtype=torch.float32).to(torch.bfloat16)
    ctx = ca.ClearAttn(n_text, gh, gw, d, r, ca.CLEAR_BF16)
    try:
        O, lse = ctx.forward_lse(Q, K, V)
        dQ, dK, dV = ctx.backward(Q, K, V, O, dO, lse)
        Qs, Ks, Vs, dOs = (token_major(t) for t in (Q, K, V, dO))
        lse_s = torch.empty_like(lse)
        Os = ctx.forward_strided(Qs, Ks, Vs, lse=lse_s)
        dQs, dKs, dVs = ctx.backward_strided(Qs, Ks, Vs, Os, dOs, lse_s)
        torch.cuda.synchronize()
    finally:
        ctx.destroy()
    assert dQs.stride() == Qs.stride() and not dQs.is_contiguous()
    assert torch.equal(O, Os.contiguous()) and torch.equal(lse, lse_s)
    for a, b in ((dQ, dQs), (dK, dKs), (dV, dVs)):
        assert torch.equal(a, b.contiguous())


def test_training_pair_in_token_major_storage_many_workgroups():
    """The same at a size where the backward pass sends its kernels out one after the other (more than 64 image
    workgroups per CU) and the dQ kernels form delta from the O rows themselves, through O's strides."""
    B, H, n_text, gh, gw, r, d = 1, 96, 64, 224, 224, 8, 128
    Q, K, V = make_qkv_shape(B, H, n_text, gh, gw, d, "bf16", seed=760, device=DEV)
    g = torch.Generator(device=DEV).manual_seed(761)
    dO = torch.randn(Q.shape, generator=g, device=DEV, dtype=torch.float32).to(torch.bfloat16)
    ctx = ca.ClearAttn(n_text, gh, gw, d, r, ca.CLEAR_BF16)
    try:
        O, lse = ctx.forward_lse(Q, K, V)
        dQ, dK, dV = ctx.backward(Q, K, V, O, dO, lse)
        Qs, Ks, Vs, dOs, Os = (token_major(t) for t in (Q, K, V, dO, O))
        dQs, dKs, dVs = ctx.backward_strided(Qs, Ks, Vs, Os, dOs, lse)
        torch.cuda.synchronize()
    finally:
        ctx.destroy()
    assert not dQs.is_contiguous()
    for a, b in ((dQ, dQs), (dK, dKs), (dV, dVs)):
        assert torch.equal(a, b.contiguous())


def test_autograd_takes_transposed_views():
    from paper_2412_16112_amd.autograd import clear_attention, clear_context_cache
    B, H, n_text, gh, gw, d, r = 1, 2, 16, 24, 24, 128, 5
    Q, K, V = make_qkv_shape(B, H, n_text, gh, gw, d, "bf16", seed=750, device=DEV)
    g = torch.Generator(device=DEV).manual_seed(751)
    dO = torch.randn(Q.shape, generator=g, device=DEV, dtype=torch.float32).to(torch.bfloat16)
    leaves = [t.permute(0, 2, 1, 3).contiguous().requires_grad_(True) for t in (Q, K, V)]  # [B, N, H, d] parameters' outputs
    try:
        O = clear_attention(*(t.permute(0, 2, 1, 3) for t in leaves), n_text, gh, gw, r)
        O.backward(dO)
        torch.cuda.synchronize()
    finally:
        clear_context_cache()
    q, k, v, go = (t[0, 0].float().cpu().numpy() for t in (Q, K, V, dO))
    rQ, rK, rV = orc.backward(q, k, v, go, n_text, gh, gw, r)
    for leaf, ref in zip(leaves, (rQ, rK, rV)):
        got = leaf.grad.permute(0, 2, 1, 3)[0, 0].float().cpu().numpy()
        mx, rms = error_metrics(got, ref)
        assert mx <= TOL["bf16"][0] * np.abs(ref).max() and rms <= TOL["bf16"][1], (mx, rms)
