"""torch.autograd entry point for the CLEAR local attention (argument marshalling only: forward and backward
both run in the HIP library).

    from paper_2412_16112_amd.autograd import clear_attention
    O = clear_attention(Q, K, V, n_text=512, gridH=64, gridW=64, r=16)   # [B, H, N, 128] bf16, differentiable

Contexts (tile schedule, mask table, workspaces) are cached per (device, shape, mask); the cache keeps the
`MAX_CACHED_CONTEXTS` most recently used ones (an evicted context is destroyed once no pending backward holds it) and
`clear_context_cache()` empties it.  Gradients need bf16 tensors: the backward kernels are built for bf16 only, and
a call that asks for gradients of fp32 tensors is refused in the forward pass, not later inside `loss.backward()`.
"""
import torch

from . import clear_attn as ca

MAX_CACHED_CONTEXTS = 16
_contexts = {}  # insertion order = least recently used first


def _context(device, n_text, gridH, gridW, head_dim, r, dtype_code, mask_kind=ca.CLEAR_MASK_DISC, shift=0):
    key = (device.index, n_text, gridH, gridW, head_dim, r, dtype_code, mask_kind, shift)
    ctx = _contexts.pop(key, None)
    if ctx is None:
        with torch.cuda.device(device):
            ctx = ca.ClearAttn(n_text, gridH, gridW, head_dim, r, dtype_code, mask_kind, shift)
    _contexts[key] = ctx  # most recently used last
    while len(_contexts) > MAX_CACHED_CONTEXTS:
        # dropped, not destroyed: a saved-for-backward reference may still use it; ClearAttn.__del__ frees it with
        # the last reference (its kernels have been enqueued by then, and the free waits for the device)
        _contexts.pop(next(iter(_contexts)))
    return ctx


def clear_context_cache():
    _contexts.clear()


class ClearAttentionFunction(torch.autograd.Function):
    @staticmethod
    def forward(fctx, Q, K, V, n_text, gridH, gridW, r, mask_kind=ca.CLEAR_MASK_DISC, shift=0):
        # bf16 tensors go in with whatever batch / head / token strides they have (transposed views of a projection's
        # [B, N, H, d] output included); only the channels must be contiguous
        strided = Q.dtype == torch.bfloat16
        if any(fctx.needs_input_grad[:3]) and not strided:
            raise ca.ClearAttnError(ca.CLEAR_ERR_UNSUPPORTED, "gradients need bf16 tensors: the backward pass is built for bf16 only "
                                    "(detach the fp32 inputs or cast them to bfloat16)")
        fix = (lambda t: t if t.stride(-1) == 1 else t.contiguous()) if strided else (lambda t: t.contiguous())
        Q, K, V = fix(Q), fix(K), fix(V)
        ctx = _context(Q.device, n_text, gridH, gridW, Q.shape[-1], r, ca._dtype_code(Q), mask_kind, shift)
        needs_grad = any(fctx.needs_input_grad[:3])
        with torch.cuda.device(Q.device):
            if strided:
                lse = torch.empty(Q.shape[:3], dtype=torch.float32, device=Q.device) if needs_grad else None
                O = ctx.forward_strided(Q, K, V, lse=lse)
            elif needs_grad:
                O, lse = ctx.forward_lse(Q, K, V)
            else:
                O = ctx.forward(Q, K, V)
            if needs_grad:
                fctx.save_for_backward(Q, K, V, O, lse)
                fctx.clear_ctx = ctx
        return O

    @staticmethod
    def backward(fctx, dO):
        Q, K, V, O, lse = fctx.saved_tensors
        dO = dO.to(Q.dtype)
        with torch.cuda.device(Q.device):
            if Q.dtype == torch.bfloat16:
                dQ, dK, dV = fctx.clear_ctx.backward_strided(Q, K, V, O, dO if dO.stride(-1) == 1 else dO.contiguous(), lse)
            else:
                dQ, dK, dV = fctx.clear_ctx.backward(Q, K, V, O, dO.contiguous(), lse)
        return dQ, dK, dV, None, None, None, None, None, None


def clear_attention(Q, K, V, n_text, gridH, gridW, r, mask_kind=ca.CLEAR_MASK_DISC, shift=0):
    """softmax(Q K^T / sqrt(d) under the CLEAR mask) V for [B, H, n_text + gridH*gridW, d] device tensors.
    mask_kind / shift select one of the compared local masks instead of the disc (clear_attn_create_masked)."""
    return ClearAttentionFunction.apply(Q, K, V, n_text, gridH, gridW, r, mask_kind, shift)
