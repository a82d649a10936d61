"""Pins of the prologue oracle (oracle/prologue.py): each step against a closed form, an invariant, or a
library routine that computes the same published definition another way."""
import numpy as np
import pytest
import torch

from oracle import clear_oracle as orc
from oracle import prologue as pro
from paper_2412_16112_amd.inputs import make_prologue_inputs


def test_rms_norm_unit_rms_and_scale_invariance():
    rng = np.random.default_rng(0)
    x = rng.normal(size=(7, 128)) * 3.0
    y = pro.rms_norm(x, np.ones(128), 0.0)
    assert np.allclose(np.mean(y * y, axis=-1), 1.0, rtol=0, atol=1e-13)
    assert np.allclose(pro.rms_norm(5.0 * x, np.ones(128), 0.0), y, rtol=0, atol=1e-13)
    # with eps: |y|^2 = c * ss / (ss + c eps), ss = |x|^2
    eps = 0.37
    ss = (x * x).sum(-1)
    y = pro.rms_norm(x, np.ones(128), eps)
    assert np.allclose((y * y).sum(-1), 128 * ss / (ss + 128 * eps), rtol=1e-13)


def test_rms_norm_against_torch():
    rng = np.random.default_rng(1)
    x = rng.normal(size=(5, 64))
    g = rng.normal(size=64)
    ref = torch.nn.functional.rms_norm(torch.from_numpy(x), (64,), torch.from_numpy(g), 1e-6).numpy()
    assert np.allclose(pro.rms_norm(x, g, 1e-6), ref, rtol=0, atol=1e-13)


def test_rotate_pairs_quarter_turn_fixes_the_sign():
    x = np.array([1.0, 0.0, 0.0, 2.0])
    c, s = np.zeros(2), np.ones(2)  # 90 degrees on both pairs
    assert np.allclose(pro.rotate_pairs(x, c, s), [0.0, 1.0, -2.0, 0.0], atol=1e-15)


def test_rotate_pairs_is_complex_multiplication():
    rng = np.random.default_rng(2)
    x = rng.normal(size=(9, 32))
    ang = rng.uniform(-7, 7, size=(9, 16))
    z = (x[:, 0::2] + 1j * x[:, 1::2]) * np.exp(1j * ang)
    y = pro.rotate_pairs(x, np.cos(ang), np.sin(ang))
    assert np.allclose(y[:, 0::2], z.real, atol=1e-14) and np.allclose(y[:, 1::2], z.imag, atol=1e-14)
    assert np.allclose((y * y).sum(-1), (x * x).sum(-1), rtol=1e-13)


def test_rotated_dot_product_depends_on_the_angle_difference_only():
    rng = np.random.default_rng(3)
    q, k = rng.normal(size=16), rng.normal(size=16)
    a, b = rng.uniform(-3, 3, size=8), rng.uniform(-3, 3, size=8)
    lhs = pro.rotate_pairs(q, np.cos(a), np.sin(a)) @ pro.rotate_pairs(k, np.cos(b), np.sin(b))
    rhs = pro.rotate_pairs(q, np.cos(a - b), np.sin(a - b)) @ k
    assert abs(lhs - rhs) < 1e-13


def test_token_rotation_adds_the_axis_angles_and_leaves_text_alone():
    rng = np.random.default_rng(4)
    n_text, gridH, gridW, half = 3, 4, 5, 6
    ay, ax = rng.uniform(-9, 9, size=(gridH, half)), rng.uniform(-9, 9, size=(gridW, half))
    ty = np.stack([np.cos(ay), np.sin(ay)], -1)
    tx = np.stack([np.cos(ax), np.sin(ax)], -1)
    cos, sin = pro.token_rotation(n_text, gridH, gridW, ty, tx)
    assert cos.shape == (n_text + gridH * gridW, half)
    assert np.all(cos[:n_text] == 1.0) and np.all(sin[:n_text] == 0.0)
    for y in range(gridH):
        for x in range(gridW):
            t = n_text + y * gridW + x
            assert np.allclose(cos[t], np.cos(ay[y] + ax[x]), atol=1e-14)
            assert np.allclose(sin[t], np.sin(ay[y] + ax[x]), atol=1e-14)


def test_round_bf16_ties_and_against_torch():
    # spacing of bf16 in [1, 2) is 2^-7: ties go to the even neighbour
    assert pro.round_bf16(np.array([1.0 + 2.0 ** -8]))[0] == 1.0
    assert pro.round_bf16(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6
    assert pro.round_bf16(np.array([1.0 + 2.0 ** -8 + 2.0 ** -30]))[0] == 1.0 + 2.0 ** -7
    assert pro.round_bf16(np.array([-0.0, 0.0])).tolist() == [0.0, 0.0]
    g = torch.Generator().manual_seed(5)
    x = torch.randn(4096, generator=g, dtype=torch.float32) * torch.logspace(-6, 6, 4096)
    ref = x.to(torch.bfloat16).double().numpy()
    assert np.array_equal(pro.round_bf16(x.double().numpy()), ref)


def test_prologue_tables_of_the_input_recipe():
    gq, gk, ty, tx = make_prologue_inputs(6, 9, 128, seed=7, ntk_factor=10.0)
    assert gq.shape == (128,) and ty.shape == (6, 64, 2) and tx.shape == (9, 64, 2)
    ty, tx = ty.double().numpy(), tx.double().numpy()
    assert np.allclose(ty[..., 0] ** 2 + ty[..., 1] ** 2, 1.0, atol=1e-6)
    # 8 constant pairs, 28 row pairs, 28 column pairs
    assert np.all(ty[:, :8, 0] == 1) and np.all(ty[:, 36:, 0] == 1) and np.all(tx[:, :36, 0] == 1)
    assert np.all(ty[0, :, 1] == 0) and np.all(tx[0, :, 1] == 0)
    assert abs(ty[1, 8, 1] - np.sin(1.0)) < 1e-6 and abs(tx[2, 36, 0] - np.cos(2.0)) < 1e-6


def test_whole_prologue_against_a_torch_pipeline():
    """RMS norm -> rotary (complex form) -> masked SDPA in torch fp64 against oracle prologue + oracle attention
    (without the bf16 rounding, which has its own pin)."""
    n_text, gridH, gridW, d, r = 5, 6, 7, 32, 3
    N = n_text + gridH * gridW
    g = torch.Generator().manual_seed(11)
    q, k, v = (torch.randn(N, d, generator=g, dtype=torch.float64) for _ in range(3))
    gq, gk, ty, tx = make_prologue_inputs(gridH, gridW, d, seed=12)
    logit_scale = 1.3

    def torch_side(x, gain):
        x = torch.nn.functional.rms_norm(x, (d,), gain.double(), 1e-6)
        ang_y = torch.atan2(ty[..., 1], ty[..., 0]).double()
        ang_x = torch.atan2(tx[..., 1], tx[..., 0]).double()
        ang = torch.cat([torch.zeros(n_text, d // 2, dtype=torch.float64), (ang_y[:, None] + ang_x[None, :]).reshape(-1, d // 2)])
        z = torch.view_as_complex(x.reshape(N, d // 2, 2).contiguous()) * torch.polar(torch.ones_like(ang), ang)
        return torch.view_as_real(z).reshape(N, d)

    qt, kt = torch_side(q, gq), torch_side(k, gk)
    M = torch.from_numpy(orc.mask_dense(n_text, gridH, gridW, r).astype(bool))
    ref = torch.nn.functional.scaled_dot_product_attention(qt[None], kt[None], v[None], attn_mask=M[None], scale=logit_scale / d ** 0.5)[0].numpy()

    def oracle_side(x, gain):
        y = pro.rms_norm(x.numpy(), gain.numpy(), 1e-6)
        cos, sin = pro.token_rotation(n_text, gridH, gridW, ty.numpy(), tx.numpy())
        return pro.rotate_pairs(y, cos, sin)

    got = orc.attention_rows(oracle_side(q, gq) * logit_scale, oracle_side(k, gk), v.numpy(), np.arange(N), n_text, gridH, gridW, r)
    assert np.allclose(got, ref, rtol=0, atol=1e-7)  # tables are fp32: atan2 of rounded (cos, sin) pairs


def test_qk_prologue_switches():
    rng = np.random.default_rng(13)
    x = rng.normal(size=(2 + 3 * 4, 16))
    assert np.array_equal(pro.qk_prologue(x, None, 0.0, 2, 3, 4, None, None), pro.round_bf16(x))
    gq, gk, ty, tx = make_prologue_inputs(3, 4, 16, seed=14)
    full = pro.qk_prologue(x, gq.numpy(), 1e-6, 2, 3, 4, ty.numpy(), tx.numpy())
    cos, sin = pro.token_rotation(2, 3, 4, ty.numpy(), tx.numpy())
    assert np.array_equal(full, pro.round_bf16(pro.rotate_pairs(pro.rms_norm(x, gq.numpy(), 1e-6), cos, sin)))
    assert np.array_equal(full[:2], pro.round_bf16(pro.rms_norm(x[:2], gq.numpy(), 1e-6)))  # text rows are not turned
