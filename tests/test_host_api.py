"""Host-side checks that need no GPU: exported symbols, argument validation, sum(M), and the tile
schedule of the library against the oracle's brute-force schedule (bit-exact)."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import clear_oracle as orc
from paper_2412_16112_amd import clear_attn as ca
from paper_2412_16112_amd.inputs import WORKLOADS

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "clear_attn.h")).read()
    declared = sorted(set(re.findall(r"\b(clear_attn_[a-z_]+)\s*\(", header)))
    assert declared == sorted(ca.EXPORTS)
    L = ctypes.CDLL(ca.LIB_PATH)
    for name in declared:
        assert hasattr(L, name), name


@pytest.mark.parametrize("name", list(WORKLOADS))
def test_mask_count_matches_known_values(name):
    w = WORKLOADS[name]
    expected = {"tiny": 13484, "flux-1024": 7051328, "flux-2048-r16": 28693056, "flux-2048-r8": 20038564,
                "flux-4096-r32": 255670316, "flux-4096-192x320-r32": 238348332, "flux-8k-r16": 471125568,
                # (each of these reproduces the figure the paper prints for it: 4 * sum(M) * 3072, tests/golden/)
                "flux-1024-r8": 5166500, "flux-1024-r32": 12541484, "flux-2048-r32": 58940460, "flux-4096-r8": 79691684,
                "flux-4096-r16": 116631104, "flux-8k-r8": 318633892, "flux-8k-r32": 1064857644,
                # 333 text tokens: the image-image part is that of the 512-text-token workload of the same grid
                "sd35l-1024-r16": 5433705, "sd35l-4096-r16": 93017961}[name]
    assert ca.clear_attn_mask_count(w.n_text, w.gridH, w.gridW, w.r) == expected


@pytest.mark.parametrize("n_text,gh,gw,r", [(8, 16, 16, 4), (0, 5, 9, 3), (3, 7, 4, 1), (5, 6, 6, 20), (512, 64, 64, 16), (17, 40, 23, 9)])
def test_mask_count_vs_oracle(n_text, gh, gw, r):
    assert ca.clear_attn_mask_count(n_text, gh, gw, r) == orc.mask_count(n_text, gh, gw, r)


def test_argument_validation_without_gpu():
    L = ca.lib()
    out = ctypes.c_ulonglong(0)
    assert L.clear_attn_mask_count(-1, 4, 4, 2, ctypes.byref(out)) == ca.CLEAR_ERR_INVALID_ARG
    assert L.clear_attn_mask_count(0, 0, 4, 2, ctypes.byref(out)) == ca.CLEAR_ERR_INVALID_ARG
    assert L.clear_attn_mask_count(0, 4, 4, 0, ctypes.byref(out)) == ca.CLEAR_ERR_INVALID_ARG
    assert L.clear_attn_mask_count(0, 4, 4, 2, None) == ca.CLEAR_ERR_INVALID_ARG
    assert b"NULL" in L.clear_attn_last_error(None)
    ctx = ctypes.c_void_p(None)
    # rejected before any device work
    assert L.clear_attn_create(ctypes.byref(ctx), 8, 16, 16, 64, 0, ca.CLEAR_F32) == ca.CLEAR_ERR_INVALID_ARG
    assert L.clear_attn_create(ctypes.byref(ctx), 8, 16, 16, 96, 4, ca.CLEAR_BF16) == ca.CLEAR_ERR_UNSUPPORTED
    assert L.clear_attn_create(ctypes.byref(ctx), 8, 16, 16, 64, 4, 7) == ca.CLEAR_ERR_INVALID_ARG
    assert L.clear_attn_create(None, 8, 16, 16, 64, 4, ca.CLEAR_F32) == ca.CLEAR_ERR_INVALID_ARG
    assert not ctx.value
    assert L.clear_attn_forward(None, None, None, None, None, 1, 1, 8, 16, 16, 64, 4, None) == ca.CLEAR_ERR_INVALID_ARG
    L.clear_attn_destroy(None)  # no-op
    with pytest.raises(ca.ClearAttnError):
        ca.clear_attn_tile_shape(128, ca.CLEAR_F32)
    assert ca.clear_attn_tile_shape(128, ca.CLEAR_BF16) == (16, 16, 8, 8)
    assert ca.clear_attn_tile_shape(64, ca.CLEAR_F32) == (16, 16, 8, 8)


SCHED_CASES = [(16, 16, 4), (20, 28, 4), (64, 64, 16), (33, 17, 9), (24, 40, 16), (7, 5, 1), (9, 70, 32), (128, 128, 8)]


@pytest.mark.parametrize("gh,gw,r", SCHED_CASES)
def test_schedule_bit_exact_vs_oracle_bruteforce(gh, gw, r):
    qth, qtw, kth, ktw = ca.clear_attn_tile_shape(128, ca.CLEAR_BF16)
    rp, ci, fl = ca.clear_attn_schedule_host(gh, gw, r, qth, qtw, kth, ktw)
    rp2, ci2, fl2 = orc.tile_schedule(gh, gw, r, qth, qtw, kth, ktw)
    assert rp.dtype == rp2.dtype and np.array_equal(rp, rp2)
    assert np.array_equal(ci, ci2)
    assert np.array_equal(fl, fl2)


@pytest.mark.parametrize("qt,kt", [((4, 8), (4, 8)), ((2, 2), (1, 2)), ((8, 16), (8, 8)), ((4, 4), (2, 2))])
def test_schedule_other_tile_shapes_vs_oracle(qt, kt):
    for gh, gw, r in [(20, 28, 4), (40, 40, 12), (13, 31, 6)]:
        got = ca.clear_attn_schedule_host(gh, gw, r, qt[0], qt[1], kt[0], kt[1])
        ref = orc.tile_schedule(gh, gw, r, qt[0], qt[1], kt[0], kt[1])
        for a, b in zip(got, ref):
            assert np.array_equal(a, b)


@pytest.mark.slow
@pytest.mark.parametrize("name", ["flux-2048-r16", "flux-4096-r32", "flux-4096-192x320-r32", "flux-8k-r16"])
def test_schedule_bit_exact_large(name):
    w = WORKLOADS[name]
    qth, qtw, kth, ktw = ca.clear_attn_tile_shape(128, ca.CLEAR_BF16)
    got = ca.clear_attn_schedule_host(w.gridH, w.gridW, w.r, qth, qtw, kth, ktw)
    ref = orc.tile_schedule(w.gridH, w.gridW, w.r, qth, qtw, kth, ktw)
    for a, b in zip(got, ref):
        assert np.array_equal(a, b)
    assert got[2].any() == (w.r >= 32)


def test_band_layout_partitions_and_halos():
    from oracle import patch_parallel as pp
    for gridH, r, n in [(512, 16, 8), (64, 16, 4), (50, 6, 7), (23, 3, 5), (16, 4, 3), (9, 1, 9), (12, 5, 1)]:
        rows = [ca.clear_attn_band_layout(gridH, r, n, b) for b in range(n)]
        assert [x[:2] for x in rows] == pp.band_rows(gridH, n)
        for y0, y1, ht, hb in rows:
            assert ht == min(r - 1, y0) and hb == min(r - 1, gridH - y1)


def test_band_layout_rejects_bands_narrower_than_the_halo():
    # 64 rows in 8 bands of 8 with r = 16: the 15 halo rows would reach across two neighbours
    with pytest.raises(ca.ClearAttnError) as e:
        ca.clear_attn_band_layout(64, 16, 8, 0)
    assert e.value.status == ca.CLEAR_ERR_UNSUPPORTED
    with pytest.raises(ca.ClearAttnError) as e:
        ca.clear_attn_band_layout(4, 2, 5, 0)
    assert e.value.status == ca.CLEAR_ERR_UNSUPPORTED
    for bad in [(0, 4, 1, 0), (8, 0, 1, 0), (8, 4, 0, 0), (8, 4, 2, 2), (8, 4, 2, -1)]:
        with pytest.raises(ca.ClearAttnError) as e:
            ca.clear_attn_band_layout(*bad)
        assert e.value.status == ca.CLEAR_ERR_INVALID_ARG
