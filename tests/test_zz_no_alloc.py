"""clear_attn_forward_noalloc (the forward pass for callers that cannot allocate device memory), called through
the C ABI: its output against clear_attn_forward's on the same inputs, and against the fp64 oracle, on two calls
in a row that share the library's static scratch array, the second with a smaller input."""
import sys

import numpy as np
import pytest
import torch

from oracle import clear_oracle as orc
from paper_2412_16112_amd import clear_attn as ca
from paper_2412_16112_amd.inputs import make_qkv_shape
from tests.parity_util import TOL, error_metrics

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _announce(msg):
    print("[case] " + msg, flush=True)
    sys.stdout.flush()


def _both(B, H, n_text, gh, gw, d, r, dtype, seed):
    """(noalloc output, forward output, oracle) for one seeded problem."""
    Q, K, V = make_qkv_shape(B, H, n_text, gh, gw, d, dtype, seed, device="cpu")
    ref = orc.attention(Q, K, V, n_text, gh, gw, r)
    Qd, Kd, Vd = Q.to(DEV), K.to(DEV), V.to(DEV)
    code = ca.CLEAR_BF16 if dtype == "bf16" else ca.CLEAR_F32
    ctx = ca.ClearAttn(n_text, gh, gw, d, r, code)
    try:
        O_na = torch.full_like(Qd, float("nan"))
        ctx.forward_noalloc(Qd, Kd, Vd, O_na)
        torch.cuda.synchronize()
        O_fw = ctx.forward(Qd, Kd, Vd)
        torch.cuda.synchronize()
    finally:
        ctx.destroy()
    return O_na, O_fw, ref


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("bf16", 64), ("f32", 64)])
def test_noalloc_equals_forward_twice_in_a_row_second_call_smaller(dtype, d):
    # first call: several key splits and query tiles, ragged grid; second call: fewer heads, fewer text tokens, smaller
    # grid, so that it uses a prefix of what the first call left in the scratch array
    for (B, H, n_text, gh, gw, r, seed) in [(1, 3, 300, 40, 56, 8, 31), (1, 2, 70, 20, 28, 4, 32)]:
        _announce(f"noalloc vs forward B={B} H={H} n_text={n_text} grid={gh}x{gw} d={d} r={r} {dtype} seed={seed}")
        O_na, O_fw, ref = _both(B, H, n_text, gh, gw, d, r, dtype, seed)
        assert torch.isfinite(O_na.float()).all()
        # same kernels, same key splits: the two entry points agree bit for bit
        assert torch.equal(O_na, O_fw)
        max_abs, rel_rms = error_metrics(O_na.float().cpu().numpy(), ref)
        tol = TOL[dtype]
        assert max_abs <= tol[0] and rel_rms <= tol[1], (max_abs, rel_rms)


def test_noalloc_without_text_tokens_needs_no_scratch():
    _announce("noalloc, n_text = 0")
    O_na, O_fw, ref = _both(1, 2, 0, 33, 17, 128, 9, "bf16", 33)
    assert torch.equal(O_na, O_fw)
    max_abs, rel_rms = error_metrics(O_na.float().cpu().numpy(), ref)
    assert max_abs <= TOL["bf16"][0] and rel_rms <= TOL["bf16"][1]


def test_noalloc_rejects_what_does_not_fit_and_launches_nothing():
    """B*H * splits * n_text * (d + 2) floats beyond the 112 MiB array: CLEAR_ERR_UNSUPPORTED with the sizes, O untouched."""
    _announce("noalloc, too large for the scratch array")
    n_text, gh, gw, d, r = 512, 64, 64, 128, 16
    B, H = 8, 96  # 768 (batch, head) pairs x >= 1 split x 512 rows x 130 floats = 204 MB
    ctx = ca.ClearAttn(n_text, gh, gw, d, r, ca.CLEAR_BF16)
    try:
        N = n_text + gh * gw
        Q = torch.zeros((B, H, N, d), dtype=torch.bfloat16, device=DEV)
        O = torch.full_like(Q, 7.0)
        with pytest.raises(ca.ClearAttnError) as ei:
            ctx.forward_noalloc(Q, Q.clone(), Q.clone(), O)
        assert ei.value.status == ca.CLEAR_ERR_UNSUPPORTED
        assert "scratch" in str(ei.value) and str(112 << 20) in str(ei.value)
        torch.cuda.synchronize()
        assert bool((O == 7.0).all())
        # the same context still serves a call that fits
        Qs, Ks, Vs = (t.to(DEV) for t in make_qkv_shape(1, 2, n_text, gh, gw, d, "bf16", 34, device="cpu"))
        O_na = torch.empty_like(Qs)
        ctx.forward_noalloc(Qs, Ks, Vs, O_na)
        O_fw = ctx.forward(Qs, Ks, Vs)
        torch.cuda.synchronize()
        assert torch.equal(O_na, O_fw)
    finally:
        ctx.destroy()


def test_noalloc_argument_checks():
    _announce("noalloc, argument checks")
    ctx = ca.ClearAttn(8, 16, 16, 128, 4, ca.CLEAR_BF16)
    try:
        Q = torch.zeros((1, 1, 8 + 256, 128), dtype=torch.bfloat16, device=DEV)
        O = torch.empty_like(Q)
        L = ca.lib()
        import ctypes
        rc = L.clear_attn_forward_noalloc(ctx._ctx, Q.data_ptr(), Q.data_ptr(), Q.data_ptr(), None, 1, 1, 8, 16, 16, 128, 4, None)
        assert rc == ca.CLEAR_ERR_INVALID_ARG
        rc = L.clear_attn_forward_noalloc(ctx._ctx, Q.data_ptr(), Q.data_ptr(), Q.data_ptr(), O.data_ptr(), 1, 1, 8, 16, 17, 128, 4, None)
        assert rc == ca.CLEAR_ERR_MISMATCH
        rc = L.clear_attn_forward_noalloc(None, Q.data_ptr(), Q.data_ptr(), Q.data_ptr(), O.data_ptr(), 1, 1, 8, 16, 16, 128, 4, None)
        assert rc == ca.CLEAR_ERR_INVALID_ARG
    finally:
        ctx.destroy()
