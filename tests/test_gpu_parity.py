"""GPU parity: the HIP path, called through the C ABI, against the fp64 CPU oracle on the same seeded
inputs -- element by element on small cases, on sampled rows at the full workload sizes."""
import sys

import numpy as np
import pytest
import torch

from oracle import clear_oracle as orc
from paper_2412_16112_amd import clear_attn as ca
from paper_2412_16112_amd.inputs import WORKLOADS, make_qkv, make_qkv_shape
from tests.parity_util import TOL, error_metrics, oracle_rows_for_heads, sample_rows

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _announce(msg):
    print("[case] " + msg, flush=True)
    sys.stdout.flush()


def _run_full_compare(B, H, n_text, gh, gw, d, r, dtype, seed, q_scale=1.0):
    _announce(f"full compare B={B} H={H} n_text={n_text} grid={gh}x{gw} d={d} r={r} {dtype} seed={seed}")
    Q, K, V = make_qkv_shape(B, H, n_text, gh, gw, d, dtype, seed, device="cpu", q_scale=q_scale)
    O = ca.clear_attn_forward_once(Q.to(DEV), K.to(DEV), V.to(DEV), n_text, gh, gw, r).float().cpu().numpy()
    ref = orc.attention(Q, K, V, n_text, gh, gw, r)
    assert np.isfinite(O).all()
    max_abs, rel_rms = error_metrics(O, ref)
    tol = TOL[dtype]
    assert max_abs <= tol[0] and rel_rms <= tol[1], (max_abs, rel_rms)
    return max_abs, rel_rms


def test_tiny_fp32_workload():
    w = WORKLOADS["tiny"]
    Q, K, V = make_qkv(w, "cpu")
    _announce("tiny fp32")
    O = ca.clear_attn_forward_once(Q.to(DEV), K.to(DEV), V.to(DEV), w.n_text, w.gridH, w.gridW, w.r).cpu().numpy()
    ref = orc.attention(Q, K, V, w.n_text, w.gridH, w.gridW, w.r)
    max_abs, rel_rms = error_metrics(O, ref)
    assert max_abs <= 1e-4 and rel_rms <= 1e-4, (max_abs, rel_rms)


@pytest.mark.parametrize("B,H,n_text,gh,gw,r", [
    (1, 1, 8, 16, 16, 4),      # tiny shape
    (2, 3, 40, 20, 28, 4),     # ragged text tile, ragged query and key tiles
    (1, 2, 0, 33, 17, 9),      # no text tokens
    (1, 2, 5, 7, 5, 1),        # r = 1: image queries see themselves + text
    (1, 1, 70, 24, 40, 100),   # r beyond the diagonal: full attention
    (1, 2, 300, 9, 70, 32),    # thin grid, window cut on both sides
    (1, 1, 1, 1, 1, 3),        # one image token
])
def test_f32_small_cases(B, H, n_text, gh, gw, r):
    _run_full_compare(B, H, n_text, gh, gw, 64, r, "f32", seed=100 + gh)


@pytest.mark.parametrize("B,H,n_text,gh,gw,r", [
    (1, 1, 8, 16, 16, 4),
    (2, 3, 40, 20, 28, 4),
    (1, 2, 0, 33, 17, 9),
    (1, 2, 5, 7, 5, 1),
    (1, 1, 70, 24, 40, 100),
    (1, 2, 300, 9, 70, 32),
    (1, 1, 1, 1, 1, 3),
    (1, 2, 512, 48, 48, 16),   # FLUX-like text length, several query tiles, r = 16
    (1, 1, 64, 40, 72, 8),
    (1, 2, 24, 40, 300, 6),    # more than 16 query tiles across: the tiles are dealt to the workgroups in 2 x 16 blocks
])
def test_bf16_small_cases(B, H, n_text, gh, gw, r):
    _run_full_compare(B, H, n_text, gh, gw, 128, r, "bf16", seed=200 + gh)


def test_bf16_sharp_logits():
    """Q scaled by 4: peaked softmax rows stress the running-maximum handling."""
    _run_full_compare(1, 2, 96, 32, 32, 128, 8, "bf16", seed=7, q_scale=4.0)


@pytest.mark.parametrize("q_scale", [60.0, 400.0])
def test_bf16_extreme_logits(q_scale):
    """Logits spread over hundreds of powers of two: exponentials relative to the first tile's maximum leave
    the fp32 range for some rows, so the kernel has to fall back to its exact-maximum pass."""
    _run_full_compare(1, 2, 64, 24, 40, 128, 6, "bf16", seed=9, q_scale=q_scale)


def test_bf16_first_tile_far_above_the_rest():
    """Text keys with huge logits, image keys with ordinary ones: everything after the first tile underflows."""
    B, H, n_text, gh, gw, d, r = 1, 1, 64, 16, 24, 128, 5
    Q, K, V = make_qkv_shape(B, H, n_text, gh, gw, d, "bf16", seed=21, device="cpu")
    K = K.float()
    K[:, :, :n_text] *= 50.0
    K = K.to(torch.bfloat16)
    _announce("first tile dominates")
    O = ca.clear_attn_forward_once(Q.to(DEV), K.to(DEV), V.to(DEV), n_text, gh, gw, r).float().cpu().numpy()
    ref = orc.attention(Q, K, V, n_text, gh, gw, r)
    max_abs, rel_rms = error_metrics(O, ref)
    assert np.isfinite(O).all() and max_abs <= TOL["bf16"][0] and rel_rms <= TOL["bf16"][1], (max_abs, rel_rms)


def test_schedule_from_context_equals_host_schedule_and_oracle():
    ctx = ca.ClearAttn(40, 20, 28, 128, 4, ca.CLEAR_BF16)
    try:
        qth, qtw, kth, ktw, nq, npairs = ctx.schedule_size()
        got = ctx.schedule_copy()
        host = ca.clear_attn_schedule_host(20, 28, 4, qth, qtw, kth, ktw)
        ref = orc.tile_schedule(20, 28, 4, qth, qtw, kth, ktw)
        for a, b, c in zip(got, host, ref):
            assert np.array_equal(a, b) and np.array_equal(a, c)
        assert nq == len(got[0]) - 1 and npairs == len(got[1])
        assert ctx.executed_pairs() >= ca.clear_attn_mask_count(40, 20, 28, 4)
    finally:
        ctx.destroy()


def test_forward_rejects_mismatch_and_bad_pointers():
    import ctypes
    ctx = ca.ClearAttn(8, 16, 16, 64, 4, ca.CLEAR_F32)
    try:
        Q, K, V = (t.to(DEV) for t in make_qkv(WORKLOADS["tiny"], "cpu"))
        O = torch.empty_like(Q)
        L = ca.lib()
        args = lambda **kw: [ctx._ctx, Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), 1, 1,
                             kw.get("n_text", 8), 16, 16, 64, kw.get("r", 4), None]
        assert L.clear_attn_forward(*args(r=5)) == ca.CLEAR_ERR_MISMATCH
        assert L.clear_attn_forward(*args(n_text=9)) == ca.CLEAR_ERR_MISMATCH
        a = args(); a[4] = None
        assert L.clear_attn_forward(*a) == ca.CLEAR_ERR_INVALID_ARG
        a = args(); a[4] = Q.data_ptr()
        assert L.clear_attn_forward(*a) == ca.CLEAR_ERR_INVALID_ARG  # O aliases Q
        a = args(); a[1] = Q.data_ptr() + 4
        assert L.clear_attn_forward(*a) == ca.CLEAR_ERR_INVALID_ARG  # misaligned
        a = args(); a[5] = 0
        assert L.clear_attn_forward(*a) == ca.CLEAR_ERR_INVALID_ARG
        assert L.clear_attn_forward(*args()) == ca.CLEAR_OK
        torch.cuda.synchronize()
    finally:
        ctx.destroy()


def _sampled_workload_check(name, heads, n_random, n_text_rows):
    w = WORKLOADS[name]
    _announce(f"workload {name} heads={heads} random_rows={n_random}")
    Q, K, V = make_qkv(w, DEV)
    ctx = ca.ClearAttn(w.n_text, w.gridH, w.gridW, w.head_dim, w.r, ca.CLEAR_BF16)
    try:
        O = ctx.forward(Q, K, V)
        torch.cuda.synchronize()
        O2 = ctx.forward(Q, K, V)  # run-to-run determinism, bit for bit
        torch.cuda.synchronize()
        assert torch.equal(O.view(torch.int16), O2.view(torch.int16))
        del O2
    finally:
        ctx.destroy()
    rows = sample_rows(w.n_text, w.gridH, w.gridW, w.r, n_random, seed=w.seed, n_text_rows=n_text_rows)
    ref = oracle_rows_for_heads(Q, K, V, heads, rows, w.n_text, w.gridH, w.gridW, w.r)
    got = O[0][heads][:, torch.from_numpy(rows).to(DEV)].float().cpu().numpy()
    assert np.isfinite(got).all()
    max_abs, rel_rms = error_metrics(got, ref)
    print(f"[result] {name}: rows={len(rows)} heads={heads} max_abs={max_abs:.3e} rel_rms={rel_rms:.3e}", flush=True)
    assert max_abs <= TOL["bf16"][0] and rel_rms <= TOL["bf16"][1], (max_abs, rel_rms)
    # properties that hold at any size: finite everywhere, |O| bounded by max |V| (convex combination)
    assert torch.isfinite(O.float()).all()
    assert O.float().abs().max() <= V.float().abs().max() * 1.01


def test_flux_1024_all_rows_two_heads():
    w = WORKLOADS["flux-1024"]
    _announce("flux-1024 all rows, heads 0 and 23")
    Q, K, V = make_qkv(w, "cpu")
    O = ca.clear_attn_forward_once(Q.to(DEV), K.to(DEV), V.to(DEV), w.n_text, w.gridH, w.gridW, w.r)
    rows = np.arange(w.N)
    heads = [0, 23]
    ref = oracle_rows_for_heads(Q, K, V, heads, rows, w.n_text, w.gridH, w.gridW, w.r)
    got = O[0][heads].float().cpu().numpy()
    max_abs, rel_rms = error_metrics(got, ref)
    print(f"[result] flux-1024: max_abs={max_abs:.3e} rel_rms={rel_rms:.3e}", flush=True)
    assert max_abs <= TOL["bf16"][0] and rel_rms <= TOL["bf16"][1], (max_abs, rel_rms)


def test_flux_2048_r16_sampled():
    _sampled_workload_check("flux-2048-r16", [0, 11, 23], 1024, None)


def test_flux_2048_r8_sampled():
    _sampled_workload_check("flux-2048-r8", [5], 1024, 64)


def test_flux_4096_r32_sampled():
    _sampled_workload_check("flux-4096-r32", [0, 12, 23], 1024, 96)


def test_flux_4096_nonsquare_sampled():
    _sampled_workload_check("flux-4096-192x320-r32", [7], 1024, 64)


def test_flux_8k_r16_sampled():
    _sampled_workload_check("flux-8k-r16", [0, 12, 23], 2048, 48)


def test_small_problem_on_a_side_stream_back_to_back():
    """Small problems fork their text-query kernels onto a stream the context owns.  Three calls in a row on a
    caller's side stream, each with its own inputs and output, synchronising that stream only: every output
    must be complete and correct (the calls share the context's text-query workspace)."""
    n_text, gh, gw, d, r, H = 96, 32, 40, 128, 8, 2
    ctx = ca.ClearAttn(n_text, gh, gw, d, r, ca.CLEAR_BF16)
    side = torch.cuda.Stream(device=DEV)
    ins = [make_qkv_shape(1, H, n_text, gh, gw, d, "bf16", seed=900 + i, device=DEV) for i in range(3)]
    torch.cuda.synchronize()
    try:
        with torch.cuda.stream(side):
            outs = [ctx.forward(Q, K, V, stream=side.cuda_stream) for Q, K, V in ins]
        side.synchronize()
    finally:
        ctx.destroy()
    for (Q, K, V), O in zip(ins, outs):
        ref = orc.attention(Q, K, V, n_text, gh, gw, r)
        max_abs, rel_rms = error_metrics(O.float().cpu().numpy(), ref)
        assert max_abs <= TOL["bf16"][0] and rel_rms <= TOL["bf16"][1], (max_abs, rel_rms)


def test_bf16_many_launches_give_the_same_bits():
    """The staged tiles pass from the loading waves to the computing waves once per stage; a missed hand-over
    would show as a run-to-run difference.  Thirty launches in a row, interleaved with a poisoned output."""
    w = WORKLOADS["flux-1024"]
    _announce("workload flux-1024, 30 launches")
    Q, K, V = make_qkv(w, DEV)
    ctx = ca.ClearAttn(w.n_text, w.gridH, w.gridW, w.head_dim, w.r, ca.CLEAR_BF16)
    try:
        ref = ctx.forward(Q, K, V).clone()
        O = torch.empty_like(ref)
        for _ in range(30):
            O.fill_(float("nan"))
            ctx.forward(Q, K, V, O)
            assert torch.equal(O.view(torch.int16), ref.view(torch.int16))
    finally:
        ctx.destroy()
