#!/usr/bin/env python3
"""Benchmark of the CLEAR local-attention forward pass on one MI355X.

A "step" is one whole forward pass (image-query kernel + text-query kernel + merge) over one
synthetic batch of the FLUX-8K shape (B=1, H=24, head_dim=128, 512x512 token grid + 512 text
tokens, r=16, bf16), inputs resident in HBM before the timed region.  Prints ONE JSON line:
useful TFLOP/s = 4*sum(M)*d*H*B / time (the paper's FLOP estimate, Fig. 2 caption), plus executed
TFLOP/s (tile waste included), the roofline of the dominant kernel, and the CPU oracle timed on a
bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 matrix peak


def forward_kernel_sources_digest():
    """SHA-256 over the sources the forward kernels and their launch shape are built from: a stored counter reading
    (profiles/hbm_traffic.json) carries the digest it was taken on, so a reading that the kernels have moved away from
    shows in the bench line instead of going stale silently."""
    import hashlib
    h = hashlib.sha256()
    for name in ("kernels_bf16.hip", "kernels_bf16_d64.hip", "bf16_common.h", "block_class.h", "clear_internal.h", "schedule.cpp", "clear_attn_api.cpp"):
        with open(os.path.join(ROOT, "paper_2412_16112_amd", "csrc", name), "rb") as f:
            h.update(name.encode() + b"\0" + f.read() + b"\0")
    return h.hexdigest()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="flux-8k-r16")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-image-rows", type=int, default=131072)
    ap.add_argument("--cpu-text-rows", type=int, default=512)
    ap.add_argument("--bands", type=int, default=0,
                    help="row-band mode: time ONE band of the workload cut into this many bands (one GPU's share of a "
                         "patch-parallel run; no second GPU is used)")
    ap.add_argument("--band", type=int, default=-1, help="which band (default: a middle one, halo on both sides)")
    ap.add_argument("--halo-align", type=int, default=1,
                    help="row-band mode: widen the top halo to a multiple of this many rows (16 = the query tile: the owned rows then start on a tile boundary)")
    ap.add_argument("--backward", action="store_true",
                    help="time the backward pass (dQ, dK, dV from dO and the forward pass's log-sum-exp) instead of the forward pass")
    ap.add_argument("--mask", default="disc", choices=["disc", "square", "swin", "strided"],
                    help="image-image mask of the forward bench: the paper's disc (default) or one of the compared local masks")
    ap.add_argument("--shift", type=int, default=0, help="Swin: window shift (0 <= shift < r); strided: layer index")
    ap.add_argument("--layout", default="bhnd", choices=["bhnd", "bnhd"],
                    help="storage of Q, K, V, O in the forward bench: [B, H, N, d] (default) or [B, N, H, d] passed with strides "
                         "(what a projection produces; no transposing copy)")
    ap.add_argument("--prologue", action="store_true",
                    help="time the forward pass with the query/key prologue (RMS norm, rotary embedding, logit scale) fused in, "
                         "against the plain forward pass and against the prologue as two passes of their own")
    ap.add_argument("--no-also", action="store_true",
                    help="skip the short timings of the other paths (backward, head_dim 64, smaller images, one row band) that the "
                         "default run appends to its line as `also_measured`")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain 1 GiB device-to-device copy a few times (reference for HBM byte counters)")
    ap.add_argument("--kernel-sources-digest", action="store_true",
                    help="print the digest of the forward kernels' sources (what a new entry of profiles/hbm_traffic.json records) and exit")
    args = ap.parse_args()
    if args.kernel_sources_digest:
        print(forward_kernel_sources_digest())
        return
    if args.copy_calibration:
        import torch
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes": 1 << 30, "copies": 3}))
        return
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); --gpus %d is not supported. "
              "Heads are independent, so N GPUs would each take H/N heads with no communication inside the op." % args.gpus,
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2412_16112_amd import clear_attn as ca
    from paper_2412_16112_amd.inputs import WORKLOADS, make_qkv

    w = WORKLOADS[args.workload]
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.bands > 0:
        bench_band(args, w, dev)
        return
    if args.backward:
        bench_backward(args, w, dev)
        return
    if args.prologue:
        bench_prologue(args, w, dev)
        return
    Q, K, V = make_qkv(w, dev)
    O = torch.empty_like(Q)
    dtype_code = ca.CLEAR_BF16 if w.dtype == "bf16" else ca.CLEAR_F32
    mask_kind = {"disc": ca.CLEAR_MASK_DISC, "square": ca.CLEAR_MASK_SQUARE, "swin": ca.CLEAR_MASK_SWIN,
                 "strided": ca.CLEAR_MASK_STRIDED}[args.mask]
    ctx = ca.ClearAttn(w.n_text, w.gridH, w.gridW, w.head_dim, w.r, dtype_code, mask_kind, args.shift)
    ctx.reserve(w.B * w.H)

    if args.layout == "bnhd":
        # the same values stored token-major; the library gets [B, H, N, d] views and their strides
        Qs, Ks, Vs = (t.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3) for t in (Q, K, V))
        Os = torch.empty_like(Qs.permute(0, 2, 1, 3)).permute(0, 2, 1, 3)
        step = lambda: ctx.forward_strided(Qs, Ks, Vs, Os)
    else:
        step = lambda: ctx.forward(Q, K, V, O)
    for _ in range(args.warmup):
        step()
    # Exactly `steps` timed calls between two synchronisations: `ms_per_step` is the wall-clock mean over them.
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    # Then the same calls once more with a HIP event on the launch stream before and after each (the stream the
    # library launches on: torch's current one): the median, minimum and maximum of the per-call times are reported
    # beside the mean.  (The events stay out of the loop above: between calls of a tenth of a millisecond they
    # cost a tenth of the call.)
    events = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    events[0].record()
    for i in range(args.steps):
        step()
        events[i + 1].record()
    torch.cuda.synchronize()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    per_call_ms = sorted(events[i].elapsed_time(events[i + 1]) for i in range(args.steps))
    ms_median = per_call_ms[len(per_call_ms) // 2] if len(per_call_ms) % 2 else 0.5 * (per_call_ms[len(per_call_ms) // 2 - 1] + per_call_ms[len(per_call_ms) // 2])
    if args.layout == "bnhd":
        O.copy_(Os)  # for the check against the oracle below

    # per-kernel durations, HIP events on the launch stream
    phase_ms = ctx.forward_profile(Q, K, V, O, reps=min(256, max(3, args.steps)))

    BH = w.B * w.H
    sum_m = ca.clear_attn_mask_count_masked(w.n_text, w.gridH, w.gridW, w.r, mask_kind, args.shift)
    useful_flop = 4.0 * sum_m * w.head_dim * BH
    exec_pairs = ctx.executed_pairs()
    executed_flop = 4.0 * exec_pairs * w.head_dim * BH
    useful_tflops = useful_flop / (ms_per_step * 1e-3) / 1e12
    executed_tflops = executed_flop / (ms_per_step * 1e-3) / 1e12

    # dominant kernel: the image-query kernel.  Algorithmic work = 4*d FLOP per unmasked pair of its rows.
    sum_m_image_rows = sum_m - w.n_text * w.N
    img_flop = 4.0 * sum_m_image_rows * w.head_dim * BH
    img_ms = phase_ms[0]
    # HBM-side bytes of the dominant kernel: counter readings of separate rocprofv3 runs (FETCH_SIZE, then WRITE_SIZE), kept
    # with the commit they were taken at; stale once that kernel changes, which is why the commit is printed beside them
    # (and the digest of the kernel sources they were taken on, compared below with the sources as they are now)
    traffic, traffic_at, traffic_current = None, None, None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):
        with open(tpath) as f:
            entry = json.load(f).get(w.name if args.mask == "disc" else "", {})
        traffic, traffic_at = entry.get("image_query_kernel_bytes_per_launch"), entry.get("measured_at")
        if traffic is not None and entry.get("forward_kernel_sources_sha256"):
            traffic_current = entry["forward_kernel_sources_sha256"] == forward_kernel_sources_digest()
    roofline = {
        "bound": "mfma", "kernel": "clear_fwd_bf16_kernel<image queries>",
        "achieved": img_flop / (img_ms * 1e-3) / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
        "frac": img_flop / (img_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, "traffic": traffic, "traffic_measured_at_commit": traffic_at,
        "traffic_measured_on_current_kernel_sources": traffic_current,
        "traffic_over_algorithmic": (traffic / (w.B * w.H * 2.0 * (w.N + w.gridH * w.gridW) * w.head_dim * 2.0)) if traffic else None,
        "kernel_ms": {"image_query": phase_ms[0], "text_query": phase_ms[1], "text_merge": phase_ms[2]},
    }

    # what the matrix pipeline alone sustains on this device right now (data-sheet peak: 2.5 PFLOP/s at 2.4 GHz)
    mfma_tflops, mfma_mhz = ca.clear_attn_measure_mfma_peak(0.5)
    roofline["measured_mfma_only"] = {"tflops": mfma_tflops, "shader_mhz": mfma_mhz,
                                      "executed_frac_of_measured": executed_tflops / mfma_tflops}

    result = {
        "metric": "local-attn useful TFLOP/s (4*sumM*d)", "value": useful_tflops, "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "ms_per_step_median": ms_median, "ms_per_step_min": per_call_ms[0], "ms_per_step_max": per_call_ms[-1],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": (w.name if args.mask == "disc" else "%s mask=%s shift=%d" % (w.name, args.mask, args.shift))
                               + ("" if args.layout == "bhnd" else " layout=[B,N,H,d]"),
                   "B": w.B, "H": w.H, "head_dim": w.head_dim, "n_text": w.n_text,
                   "gridH": w.gridH, "gridW": w.gridW, "r": w.r, "sum_M_per_head": sum_m},
        "useful_tflops": useful_tflops, "executed_tflops": executed_tflops,
        "useful_frac_of_mfma_peak": useful_tflops / MFMA_BF16_PEAK_TFLOPS,
        "executed_frac_of_mfma_peak": executed_tflops / MFMA_BF16_PEAK_TFLOPS,
        "executed_over_useful": executed_flop / useful_flop,
        "roofline": roofline,
    }

    if not args.no_cpu_baseline:
        from oracle import clear_oracle as orc
        rng = np.random.default_rng(12345)
        rows_t = rng.choice(w.n_text, size=min(w.n_text, args.cpu_text_rows), replace=False) if w.n_text else np.zeros(0, int)
        rows_i = w.n_text + rng.choice(w.gridH * w.gridW, size=min(w.gridH * w.gridW, args.cpu_image_rows), replace=False)
        rows = np.sort(np.concatenate([rows_t, rows_i])).astype(np.int64)
        h = w.H // 2
        q, k, v = (t[0, h].float().cpu().double().numpy() for t in (Q, K, V))
        tc0 = time.perf_counter()
        with orc.mask_kind(mask_kind, args.shift):  # (the two sides number the mask kinds alike)
            ref, _, _, cnt = orc.attention_rows(q, k, v, rows, w.n_text, w.gridH, w.gridW, w.r, return_stats=True)
        tc1 = time.perf_counter()
        got = O[0, h][torch.from_numpy(rows).to(dev)].float().cpu().numpy()
        diff = got - ref
        cpu_flop = 4.0 * float(cnt.sum()) * w.head_dim
        result["cpu_baseline"] = {
            "value": cpu_flop / (tc1 - tc0) / 1e12, "unit": "TFLOP/s", "cores": orc.num_threads(), "kind": "oracle",
            "sample": "%d text rows + %d image rows of head %d (fp64 dense-masked loop over all %d keys per row), %.1f s"
                      % (len(rows_t), len(rows_i), h, w.N, tc1 - tc0),
            "us_per_query_row": (tc1 - tc0) * 1e6 / len(rows),
        }
        result["check_vs_oracle"] = {"rows": int(len(rows)), "max_abs": float(np.abs(diff).max()),
                                     "rel_rms": float(np.sqrt((diff ** 2).sum() / (ref ** 2).sum()))}
    ctx.destroy()
    if args.workload == "flux-8k-r16" and args.mask == "disc" and args.layout == "bhnd" and not args.no_also:
        del Q, K, V, O
        torch.cuda.empty_cache()
        result["also_measured"] = also_measured(w, dev)
    print(json.dumps(result))


def also_measured(w, dev):
    """Short timings of the other paths of the library, appended to the default run's line so that every round's
    record holds them: wall-clock mean per call between two synchronisations, inputs resident, nothing skipped.  They
    are not checked against the oracle here (the -m gpu tests and each path's own bench mode do that)."""
    import dataclasses
    import torch
    from paper_2412_16112_amd import clear_attn as ca
    from paper_2412_16112_amd.inputs import WORKLOADS, make_qkv

    def timed(step, warmup, steps):
        for _ in range(warmup):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            step()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps

    out = {}
    # forward pass on the smaller images of the paper's tables and on a head_dim-64 shape (many calls where a call is
    # short: a few dozen of them are over before the clock has settled)
    for name, warmup, steps in [("flux-1024", 100, 400), ("flux-2048-r16", 50, 200), ("flux-4096-r16", 10, 40), ("sd35l-4096-r16", 10, 40)]:
        wl = WORKLOADS[name]
        Q, K, V = make_qkv(wl, dev)
        O = torch.empty_like(Q)
        ctx = ca.ClearAttn(wl.n_text, wl.gridH, wl.gridW, wl.head_dim, wl.r, ca.CLEAR_BF16)
        ms = timed(lambda: ctx.forward(Q, K, V, O), warmup, steps)
        useful = 4.0 * ca.clear_attn_mask_count(wl.n_text, wl.gridH, wl.gridW, wl.r) * wl.head_dim * wl.B * wl.H
        out["forward " + name] = {"ms_per_step": ms, "steps": steps, "useful_tflops": useful / (ms * 1e-3) / 1e12}
        ctx.destroy()
        del Q, K, V, O
    # backward pass on the headline shape
    Q, K, V = make_qkv(w, dev)
    g = torch.Generator(device=dev).manual_seed(w.seed + 1000)
    dO = torch.randn(Q.shape, generator=g, device=dev, dtype=torch.float32).to(Q.dtype)
    ctx = ca.ClearAttn(w.n_text, w.gridH, w.gridW, w.head_dim, w.r, ca.CLEAR_BF16)
    O, lse = ctx.forward_lse(Q, K, V)
    ms = timed(lambda: ctx.backward(Q, K, V, O, dO, lse), 2, 5)
    useful = 10.0 * ca.clear_attn_mask_count(w.n_text, w.gridH, w.gridW, w.r) * w.head_dim * w.B * w.H
    out["backward " + w.name] = {"ms_per_step": ms, "steps": 5, "useful_tflops": useful / (ms * 1e-3) / 1e12}
    ctx.destroy()
    del Q, K, V, O, dO, lse
    torch.cuda.empty_cache()
    # one row band of eight (its image queries with the r - 1 halo rows, its text queries, the merge of eight partials)
    n_bands = 8
    y0, y1, ht, hb = ca.clear_attn_band_layout(w.gridH, w.r, n_bands, n_bands // 2)
    rows = ht + (y1 - y0) + hb
    Q, K, V = make_qkv(dataclasses.replace(w, gridH=rows), dev)
    O = torch.empty_like(Q)
    ctx = ca.ClearAttn(w.n_text, rows, w.gridW, w.head_dim, w.r, ca.CLEAR_BF16)
    to = torch.empty((w.B, w.H, w.n_text, w.head_dim), dtype=torch.float32, device=dev)
    tl = torch.empty((w.B, w.H, w.n_text), dtype=torch.float32, device=dev)

    def band_step():
        ctx.forward_band(Q, K, V, O, ht, ht + (y1 - y0), True, to, tl)
        ca.clear_attn_merge_text([to] * n_bands, [tl] * n_bands, O, w.n_text, ca.CLEAR_MERGE_AVERAGE)

    out["forward %s, one row band of %d" % (w.name, n_bands)] = {"ms_per_step": timed(band_step, 20, 100), "steps": 100}
    ctx.destroy()
    return out


def bench_prologue(args, w, dev):
    """Forward pass with the query/key prologue.  Three routes over the same raw Q, K: (a) the plain forward pass
    on them (no prologue; the floor), (b) fused: Q transformed as it is loaded, K by one pass into the context's
    buffer, (c) a prologue pass over Q and one over K, then the plain forward pass.  `value` is route (b)."""
    import numpy as np
    import torch
    from paper_2412_16112_amd import clear_attn as ca
    from paper_2412_16112_amd.inputs import make_prologue_inputs, make_qkv

    Q, K, V = make_qkv(w, dev)
    O = torch.empty_like(Q)
    gq, gk, ty, tx = make_prologue_inputs(w.gridH, w.gridW, w.head_dim, w.seed + 2000, ntk_factor=10.0, device=dev)
    logit_scale = 1.1
    ctx = ca.ClearAttn(w.n_text, w.gridH, w.gridW, w.head_dim, w.r, ca.CLEAR_BF16)
    ctx.reserve(w.B * w.H)
    Qp, Kp = torch.empty_like(Q), torch.empty_like(K)

    def plain():
        ctx.forward(Q, K, V, O)

    def fused():
        ctx.forward_prologue(Q, K, V, O, q_gain=gq, k_gain=gk, rope_y=ty, rope_x=tx, logit_scale=logit_scale)

    def two_pass():
        ca.clear_attn_qk_prologue(Q, w.n_text, w.gridH, w.gridW, gain=gq, rope_y=ty, rope_x=tx, out=Qp)
        ca.clear_attn_qk_prologue(K, w.n_text, w.gridH, w.gridW, gain=gk, rope_y=ty, rope_x=tx, out=Kp)
        ctx.forward(Qp, Kp, V, O)

    def one_pass_only():
        ca.clear_attn_qk_prologue(K, w.n_text, w.gridH, w.gridW, gain=gk, rope_y=ty, rope_x=tx, out=Kp)

    def timed(fn):
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / args.steps

    ms_plain, ms_fused, ms_two, ms_pass = timed(plain), timed(fused), timed(two_pass), timed(one_pass_only)
    sum_m = ca.clear_attn_mask_count(w.n_text, w.gridH, w.gridW, w.r)
    useful = 4.0 * sum_m * w.head_dim * w.B * w.H
    tensor_bytes = Q.numel() * 2
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):
        with open(tpath) as f:
            traffic = json.load(f).get(w.name + " + prologue", {}).get("qk_prologue_kernel_bytes_per_launch")
    result = {
        "metric": "local-attn forward with fused q/k prologue, useful TFLOP/s (4*sumM*d)", "value": useful / (ms_fused * 1e-3) / 1e12,
        "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_fused, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name + " + prologue", "B": w.B, "H": w.H, "head_dim": w.head_dim, "n_text": w.n_text, "gridH": w.gridH,
                   "gridW": w.gridW, "r": w.r, "logit_scale": logit_scale},
        "routes_ms": {"plain_forward_no_prologue": ms_plain, "fused": ms_fused, "two_prologue_passes_then_forward": ms_two,
                      "one_prologue_pass": ms_pass},
        # the pass of its own is the HBM-bound kernel here: one tensor read, one written
        "roofline": {"bound": "hbm", "kernel": "qk_prologue_kernel<128>", "achieved": 2 * tensor_bytes / (ms_pass * 1e-3) / 1e9, "peak": 8000.0,
                     "unit": "GB/s", "frac": 2 * tensor_bytes / (ms_pass * 1e-3) / 1e9 / 8000.0, "traffic": traffic},
    }
    if not args.no_cpu_baseline:
        from oracle import clear_oracle as orc
        from oracle import prologue as pro
        fused()
        torch.cuda.synchronize()
        h = w.H // 2
        f64 = lambda t: None if t is None else t.detach().cpu().double().numpy()
        rng = np.random.default_rng(777)
        rows = np.sort(np.concatenate([rng.choice(w.n_text, size=min(w.n_text, 64), replace=False),
                                       w.n_text + rng.choice(w.gridH * w.gridW, size=4096, replace=False)])).astype(np.int64)
        tc0 = time.perf_counter()
        qp = pro.qk_prologue(f64(Q[0, h]), f64(gq), 1e-6, w.n_text, w.gridH, w.gridW, f64(ty), f64(tx))
        kp = pro.qk_prologue(f64(K[0, h]), f64(gk), 1e-6, w.n_text, w.gridH, w.gridW, f64(ty), f64(tx))
        tc1 = time.perf_counter()
        ref = orc.attention_rows(qp * logit_scale, kp, f64(V[0, h]), rows, w.n_text, w.gridH, w.gridW, w.r)
        got = O[0, h][torch.from_numpy(rows).to(dev)].float().cpu().numpy()
        diff = got - ref
        result["cpu_baseline"] = {"value": (tc1 - tc0) * 1e6 / (2 * w.N), "unit": "us per prologue row", "cores": 1, "kind": "oracle",
                                  "sample": "prologue of Q and K of head %d (%d rows each, numpy fp64), %.1f s" % (h, w.N, tc1 - tc0)}
        result["check_vs_oracle"] = {"rows": int(len(rows)), "max_abs": float(np.abs(diff).max()),
                                     "rel_rms": float(np.sqrt((diff ** 2).sum() / (ref ** 2).sum()))}
    ctx.destroy()
    print(json.dumps(result))


def bench_backward(args, w, dev):
    """Backward pass on the workload's shape.  Useful work: the five matrix products of attention's backward
    pass over the unmasked pairs, 10*sumM*d FLOP per head (the kernels execute seven: the scores are
    recomputed once for dQ and once for dK/dV, and dV has its own pass)."""
    import numpy as np
    import torch
    from paper_2412_16112_amd import clear_attn as ca
    from paper_2412_16112_amd.inputs import make_qkv

    Q, K, V = make_qkv(w, dev)
    g = torch.Generator(device=dev).manual_seed(w.seed + 1000)
    dO = torch.randn(Q.shape, generator=g, device=dev, dtype=torch.float32).to(Q.dtype)
    ctx = ca.ClearAttn(w.n_text, w.gridH, w.gridW, w.head_dim, w.r, ca.CLEAR_BF16)
    ctx.reserve(w.B * w.H)
    O, lse = ctx.forward_lse(Q, K, V)
    for _ in range(args.warmup):
        grads = ctx.backward(Q, K, V, O, dO, lse)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        grads = ctx.backward(Q, K, V, O, dO, lse)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    sum_m = ca.clear_attn_mask_count(w.n_text, w.gridH, w.gridW, w.r)
    useful = 10.0 * sum_m * w.head_dim * w.B * w.H
    result = {
        "metric": "local-attn backward useful TFLOP/s (10*sumM*d)", "value": useful / (ms * 1e-3) / 1e12, "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name + " backward", "B": w.B, "H": w.H, "head_dim": w.head_dim, "n_text": w.n_text,
                   "gridH": w.gridH, "gridW": w.gridW, "r": w.r, "sum_M_per_head": sum_m},
        "roofline": {"bound": "mfma", "kernel": "clear_bwd_bf16_kernel (dQ, dK, dV passes)", "achieved": useful / (ms * 1e-3) / 1e12,
                     "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": useful / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, "traffic": None},
    }
    if not args.no_cpu_baseline:
        from oracle import clear_oracle as orc
        rng = np.random.default_rng(4321)
        h = w.H // 2
        q, k, v, go = (t[0, h].float().cpu().double().numpy() for t in (Q, K, V, dO))
        rows = np.sort(rng.choice(w.N, size=min(w.N, 65536), replace=False)).astype(np.int64)
        tc0 = time.perf_counter()
        ref = orc.backward_dq_rows(q, k, v, go, rows, w.n_text, w.gridH, w.gridW, w.r)
        tc1 = time.perf_counter()
        got = grads[0][0, h][torch.from_numpy(rows).to(dev)].float().cpu().numpy()
        diff = got - ref
        result["cpu_baseline"] = {"value": (tc1 - tc0) * 1e6 / len(rows), "unit": "us per dQ row", "cores": orc.num_threads(), "kind": "oracle",
                                  "sample": "dQ of %d random rows of head %d (fp64, two dense-masked passes over all %d keys per row), %.1f s"
                                            % (len(rows), h, w.N, tc1 - tc0)}
        result["check_vs_oracle"] = {"rows": int(len(rows)), "max_abs": float(np.abs(diff).max()), "ref_max_abs": float(np.abs(ref).max()),
                                     "rel_rms": float(np.sqrt((diff ** 2).sum() / (ref ** 2).sum()))}
    ctx.destroy()
    print(json.dumps(result))


def bench_band(args, w, dev):
    """One band of a patch-parallel run: the band's image queries (with halo rows as extra keys) and the text
    queries over the band's own keys, plus the merge of n_bands text partials.  Synthetic tensors of the band's
    local shape; `value` is the useful TFLOP/s of this one GPU's share."""
    import dataclasses
    import numpy as np
    import torch
    from paper_2412_16112_amd import clear_attn as ca
    from paper_2412_16112_amd.inputs import make_qkv

    band = args.band if args.band >= 0 else args.bands // 2
    y0, y1, ht, hb = ca.clear_attn_band_layout(w.gridH, w.r, args.bands, band)
    if ht:
        ht = min(y0, -(-ht // args.halo_align) * args.halo_align)
    rows = ht + (y1 - y0) + hb
    wl = dataclasses.replace(w, name="%s band %d/%d" % (w.name, band, args.bands), gridH=rows)
    Q, K, V = make_qkv(wl, dev)
    O = torch.empty_like(Q)
    dtype_code = ca.CLEAR_BF16 if w.dtype == "bf16" else ca.CLEAR_F32
    ctx = ca.ClearAttn(w.n_text, rows, w.gridW, w.head_dim, w.r, dtype_code)
    ctx.reserve(w.B * w.H)
    to = torch.empty((w.B, w.H, w.n_text, w.head_dim), dtype=torch.float32, device=dev)
    tl = torch.empty((w.B, w.H, w.n_text), dtype=torch.float32, device=dev)
    parts_o, parts_l = [to] * args.bands, [tl] * args.bands  # stand-ins for the gathered partials of the other bands

    def step():
        ctx.forward_band(Q, K, V, O, ht, ht + (y1 - y0), True, to, tl)
        ca.clear_attn_merge_text(parts_o, parts_l, O, w.n_text, ca.CLEAR_MERGE_AVERAGE)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    # useful pairs of this band: its image queries in the undivided problem + text queries over text and own image keys
    BH = w.B * w.H
    full = ca.clear_attn_mask_count(w.n_text, w.gridH, w.gridW, w.r)
    img_rows_all = full - w.n_text * (w.n_text + w.gridH * w.gridW)
    # image-query pairs of rows y0..y1-1: count by difference of two prefix problems is not exact near the cut, so count directly
    r2 = w.r * w.r
    offs = [(dy, dx) for dy in range(-w.r + 1, w.r) for dx in range(-w.r + 1, w.r) if dx * dx + dy * dy < r2]
    dyc = np.bincount(np.array([dy for dy, _ in offs]) + w.r - 1, minlength=2 * w.r - 1)  # offsets per dy, dx unrestricted
    pairs_img = 0
    for dy in range(-w.r + 1, w.r):
        n_y = sum(1 for y in range(y0, y1) if 0 <= y + dy < w.gridH)
        for ddy, dx in offs:
            if ddy == dy:
                pairs_img += n_y * max(0, w.gridW - abs(dx))
    del dyc, img_rows_all
    pairs = pairs_img + (y1 - y0) * w.gridW * w.n_text + w.n_text * (w.n_text + (y1 - y0) * w.gridW)
    useful = 4.0 * pairs * w.head_dim * BH
    ctx.destroy()
    print(json.dumps({
        "metric": "local-attn useful TFLOP/s (4*sumM*d), one band of a patch-parallel run", "value": useful / (ms * 1e-3) / 1e12,
        "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True,
        "scaling": "strong", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": wl.name, "B": w.B, "H": w.H, "head_dim": w.head_dim, "n_text": w.n_text, "band_rows": [y0, y1],
                   "halo_rows": [ht, hb], "gridW": w.gridW, "r": w.r, "n_bands": args.bands, "pairs_per_head": int(pairs),
                   "text_merge": "average (Eq. 7) over %d partials" % args.bands},
    }))


if __name__ == "__main__":
    main()
