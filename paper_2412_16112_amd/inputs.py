"""Seeded synthetic inputs and workload shapes.

This module holds no arithmetic of the attention method: it only names the workload shapes and
draws Q, K, V.  Both the GPU path and the CPU oracle are fed from here so that they see identical
bits.  The tensors stand in for post-RoPE FLUX.1-dev activations at the resolutions the paper
evaluates (Sec. 4.1, Tables 2, 3 and 7): the shapes (512 text tokens, 24 heads x 128 channels,
one latent token per 16x16 pixels) are the ones the paper's printed FLOP counts imply; the
values are i.i.d. N(0,1), rounded once to the storage dtype.
"""
from dataclasses import dataclass

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    H: int
    n_text: int
    gridH: int
    gridW: int
    head_dim: int
    r: int
    dtype: str  # "bf16" or "f32"
    seed: int
    per_head_q_scale: bool = False  # Q of head h multiplied by s_h ~ U[0.5, 2] (varies logit sharpness)

    @property
    def N(self):
        return self.n_text + self.gridH * self.gridW

    @property
    def torch_dtype(self):
        return torch.bfloat16 if self.dtype == "bf16" else torch.float32


WORKLOADS = {
    w.name: w
    for w in [
        Workload("tiny", 1, 1, 8, 16, 16, 64, 4, "f32", 0),
        Workload("flux-1024", 1, 24, 512, 64, 64, 128, 16, "bf16", 1),
        Workload("flux-2048-r16", 1, 24, 512, 128, 128, 128, 16, "bf16", 2),
        Workload("flux-2048-r8", 1, 24, 512, 128, 128, 128, 8, "bf16", 2),
        Workload("flux-4096-r32", 1, 24, 512, 256, 256, 128, 32, "bf16", 3),
        Workload("flux-4096-192x320-r32", 1, 24, 512, 192, 320, 128, 32, "bf16", 4),
        Workload("flux-8k-r16", 1, 24, 512, 512, 512, 128, 16, "bf16", 5, per_head_q_scale=True),
        # the remaining (resolution, r) pairs of the paper's efficiency tables (Tables 2, 3 and 7)
        Workload("flux-1024-r8", 1, 24, 512, 64, 64, 128, 8, "bf16", 11),
        Workload("flux-1024-r32", 1, 24, 512, 64, 64, 128, 32, "bf16", 12),
        Workload("flux-2048-r32", 1, 24, 512, 128, 128, 128, 32, "bf16", 13),
        Workload("flux-4096-r8", 1, 24, 512, 256, 256, 128, 8, "bf16", 14),
        Workload("flux-4096-r16", 1, 24, 512, 256, 256, 128, 16, "bf16", 15),
        Workload("flux-8k-r8", 1, 24, 512, 512, 512, 128, 8, "bf16", 16, per_head_q_scale=True),
        Workload("flux-8k-r32", 1, 24, 512, 512, 512, 128, 32, "bf16", 17, per_head_q_scale=True),
        # head_dim 64: the geometry of an SD3.5-Large-style block (38 heads of 64 channels, 333 text tokens; the
        # paper deploys CLEAR on that model with r = 16 but does not print its shapes)
        Workload("sd35l-1024-r16", 1, 38, 333, 64, 64, 64, 16, "bf16", 6),
        Workload("sd35l-4096-r16", 1, 38, 333, 256, 256, 64, 16, "bf16", 7),
    ]
}


def make_qkv(w, device="cpu"):
    """Draw Q, K, V of shape [B, H, N, head_dim] for workload `w` on `device`, head by head.

    The generator lives on `device`; CPU and GPU streams differ, so draw once and hand the same
    tensors (or copies of them) to every consumer."""
    dev = torch.device(device)
    g = torch.Generator(device=dev)
    g.manual_seed(w.seed)
    shape = (w.B, w.H, w.N, w.head_dim)
    out = [torch.empty(shape, dtype=w.torch_dtype, device=dev) for _ in range(3)]
    q_scale = torch.ones(w.H, dtype=torch.float32, device=dev)
    if w.per_head_q_scale:
        q_scale = 0.5 + 1.5 * torch.rand(w.H, generator=g, dtype=torch.float32, device=dev)
    for b in range(w.B):
        for h in range(w.H):
            for t, dst in enumerate(out):
                x = torch.randn((w.N, w.head_dim), generator=g, dtype=torch.float32, device=dev)
                if t == 0:
                    x = x * q_scale[h]
                dst[b, h].copy_(x)  # one round-to-nearest-even into the storage dtype
    return out[0], out[1], out[2]


def make_qkv_shape(B, H, n_text, gridH, gridW, head_dim, dtype, seed, device="cpu", q_scale=1.0):
    """Same recipe for an ad-hoc shape (edge-case tests)."""
    w = Workload("adhoc", B, H, n_text, gridH, gridW, head_dim, 1, dtype, seed)
    Q, K, V = make_qkv(w, device)
    if q_scale != 1.0:
        Q = (Q.float() * q_scale).to(Q.dtype)
    return Q, K, V


def make_prologue_inputs(gridH, gridW, head_dim, seed, ntk_factor=1.0, theta=10000.0, device="cpu"):
    """Inputs of the query/key prologue for a FLUX-style block: per-channel RMS-norm gains for Q and K
    (1 + 0.1 N(0,1), fp32) and the rotary tables of the two image axes, fp32 [grid, head_dim/2, 2] = (cos, sin).

    The channel pairs are split over three position axes in the proportion 1 : 3.5 : 3.5 (16 / 56 / 56
    channels at head_dim 128); the first axis is constant over the sequence, so its pairs hold (1, 0) in
    both tables; the second follows the row, the third the column.  Pair j of an axis with n pairs has the
    frequency (theta * ntk_factor) ** (-j / n) (ntk_factor 1: the native setting; 10: the resolution-
    extrapolation setting of Sec. 4.3)."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    half = head_dim // 2
    n_row = n_col = (half * 7) // 16
    n_const = half - n_row - n_col
    gain_q = (1.0 + 0.1 * torch.randn(head_dim, generator=g, dtype=torch.float32))
    gain_k = (1.0 + 0.1 * torch.randn(head_dim, generator=g, dtype=torch.float32))

    def table(n_pos, first, n):
        t = torch.zeros(n_pos, half, 2, dtype=torch.float64)
        t[:, :, 0] = 1.0
        freq = (theta * ntk_factor) ** (-torch.arange(n, dtype=torch.float64) / n)
        ang = torch.arange(n_pos, dtype=torch.float64)[:, None] * freq[None, :]
        t[:, first:first + n, 0] = torch.cos(ang)
        t[:, first:first + n, 1] = torch.sin(ang)
        return t.float()

    table_y = table(gridH, n_const, n_row)
    table_x = table(gridW, n_const + n_row, n_col)
    dev = torch.device(device)
    return gain_q.to(dev), gain_k.to(dev), table_y.to(dev), table_x.to(dev)
