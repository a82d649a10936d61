"""Thin ctypes binding of libclear_attn.so: the same names as include/clear_attn.h, argument
marshalling only.  PyTorch tensors are used for device memory and streams; every step of the
attention runs in the HIP kernels.  There is no fallback: a missing library raises."""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libclear_attn.so")

CLEAR_OK, CLEAR_ERR_INVALID_ARG, CLEAR_ERR_UNSUPPORTED, CLEAR_ERR_ALLOC, CLEAR_ERR_HIP, CLEAR_ERR_MISMATCH = range(6)
CLEAR_BF16, CLEAR_F32 = 0, 1
CLEAR_MERGE_EXACT, CLEAR_MERGE_AVERAGE = 0, 1
CLEAR_MASK_DISC, CLEAR_MASK_SQUARE, CLEAR_MASK_SWIN, CLEAR_MASK_STRIDED = 0, 1, 2, 3
CLEAR_TILE_PARTIAL, CLEAR_TILE_FULL = 0, 1

EXPORTS = [
    "clear_attn_create", "clear_attn_create_masked", "clear_attn_mask_count_masked", "clear_attn_schedule_host_masked", "clear_attn_reserve", "clear_attn_forward", "clear_attn_forward_profile",
    "clear_attn_destroy", "clear_attn_forward_lse", "clear_attn_backward", "clear_attn_reserve_backward",
    "clear_attn_forward_band", "clear_attn_band_layout", "clear_attn_merge_text",
    "clear_attn_mask_count", "clear_attn_tile_shape", "clear_attn_schedule_host",
    "clear_attn_schedule_size", "clear_attn_schedule_copy", "clear_attn_executed_pairs",
    "clear_attn_measure_mfma_peak", "clear_attn_last_error",
    "clear_attn_forward_prologue", "clear_attn_reserve_prologue", "clear_attn_qk_prologue",
    "clear_attn_forward_strided", "clear_attn_forward_prologue_strided", "clear_attn_backward_strided",
    "clear_attn_forward_noalloc",
]

_lib = None


class ClearAttnError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("clear_attn status %d: %s" % (status, message))
        self.status = status


def lib():
    """The loaded C library (raises if it has not been built: python -m paper_2412_16112_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libclear_attn.so is not built (run: python -m paper_2412_16112_amd.build); "
                              "there is no non-HIP fallback")
        L = ctypes.CDLL(LIB_PATH)
        i, vp, ip = ctypes.c_int, ctypes.c_void_p, ctypes.POINTER(ctypes.c_int)
        ullp, llp = ctypes.POINTER(ctypes.c_ulonglong), ctypes.POINTER(ctypes.c_longlong)
        L.clear_attn_create.argtypes = [ctypes.POINTER(vp), i, i, i, i, i, i]
        L.clear_attn_create_masked.argtypes = [ctypes.POINTER(vp), i, i, i, i, i, i, i, i]
        L.clear_attn_mask_count_masked.argtypes = [i, i, i, i, i, i, ullp]
        L.clear_attn_reserve.argtypes = [vp, i]
        L.clear_attn_forward.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, i, i, i, vp]
        L.clear_attn_forward_noalloc.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, i, i, i, vp]
        L.clear_attn_forward_profile.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, i, i, i, vp, i, ctypes.POINTER(ctypes.c_float)]
        L.clear_attn_destroy.argtypes = [vp]
        L.clear_attn_destroy.restype = None
        L.clear_attn_mask_count.argtypes = [i, i, i, i, ullp]
        L.clear_attn_tile_shape.argtypes = [i, i, ip, ip, ip, ip]
        L.clear_attn_schedule_host.argtypes = [i, i, i, i, i, i, i, ip, llp, vp, vp, vp]
        L.clear_attn_schedule_host_masked.argtypes = [i, i, i, i, i, i, i, i, i, ip, llp, vp, vp, vp]
        L.clear_attn_schedule_size.argtypes = [vp, ip, ip, ip, ip, ip, llp]
        L.clear_attn_schedule_copy.argtypes = [vp, vp, vp, vp]
        L.clear_attn_executed_pairs.argtypes = [vp, ullp]
        L.clear_attn_forward_lse.argtypes = [vp, vp, vp, vp, vp, vp, i, i, i, i, i, i, i, vp]
        L.clear_attn_backward.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i, i, i, i, i, i, i, vp]
        L.clear_attn_reserve_backward.argtypes = [vp, i]
        L.clear_attn_forward_band.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, i, i, i, i, i, i, vp, vp, vp]
        L.clear_attn_band_layout.argtypes = [i, i, i, i, ip, ip, ip, ip]
        L.clear_attn_merge_text.argtypes = [i, vp, vp, i, i, i, ctypes.c_longlong, i, i, vp, i, vp]
        L.clear_attn_measure_mfma_peak.argtypes = [ctypes.c_double, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
        f = ctypes.c_float
        L.clear_attn_forward_prologue.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, i, i, i, vp, vp, f, vp, vp, f, vp]
        L.clear_attn_reserve_prologue.argtypes = [vp, i]
        L.clear_attn_qk_prologue.argtypes = [vp, vp, i, i, i, i, i, i, vp, f, vp, vp, vp]
        L.clear_attn_forward_strided.argtypes = [vp, vp, vp, vp, vp, vp, llp, i, i, i, i, i, i, i, vp]
        L.clear_attn_backward_strided.argtypes = [vp] * 10 + [llp] + [i] * 7 + [vp]
        L.clear_attn_forward_prologue_strided.argtypes = [vp, vp, vp, vp, vp, llp, i, i, i, i, i, i, i, vp, vp, f, vp, vp, f, vp]
        L.clear_attn_last_error.argtypes = [vp]
        L.clear_attn_last_error.restype = ctypes.c_char_p
        for name in EXPORTS:
            if name not in ("clear_attn_destroy", "clear_attn_last_error"):
                getattr(L, name).restype = i
        _lib = L
    return _lib


def _check(status, ctx=None):
    if status != CLEAR_OK:
        raise ClearAttnError(status, lib().clear_attn_last_error(ctx).decode())


def clear_attn_mask_count(n_text, gridH, gridW, r):
    out = ctypes.c_ulonglong(0)
    _check(lib().clear_attn_mask_count(n_text, gridH, gridW, r, ctypes.byref(out)))
    return int(out.value)


def clear_attn_measure_mfma_peak(seconds=0.5):
    """(sustained dense bf16 MFMA TFLOP/s, shader clock in MHz) of the current device."""
    tf, mhz = ctypes.c_double(0), ctypes.c_double(0)
    _check(lib().clear_attn_measure_mfma_peak(ctypes.c_double(seconds), ctypes.byref(tf), ctypes.byref(mhz)))
    return float(tf.value), float(mhz.value)


def clear_attn_mask_count_masked(n_text, gridH, gridW, r, mask_kind, shift=0):
    out = ctypes.c_ulonglong(0)
    _check(lib().clear_attn_mask_count_masked(n_text, gridH, gridW, r, mask_kind, shift, ctypes.byref(out)))
    return int(out.value)


def clear_attn_tile_shape(head_dim, dtype):
    v = [ctypes.c_int(0) for _ in range(4)]
    _check(lib().clear_attn_tile_shape(head_dim, dtype, *[ctypes.byref(x) for x in v]))
    return tuple(int(x.value) for x in v)


def clear_attn_schedule_host(gridH, gridW, r, q_tile_h, q_tile_w, k_tile_h, k_tile_w):
    """Returns (row_ptr int32[n_q_tiles+1], col_idx int32[n_pairs], flags uint8[n_pairs])."""
    nq, npairs = ctypes.c_int(0), ctypes.c_longlong(0)
    args = (gridH, gridW, r, q_tile_h, q_tile_w, k_tile_h, k_tile_w)
    _check(lib().clear_attn_schedule_host(*args, ctypes.byref(nq), ctypes.byref(npairs), None, None, None))
    row_ptr = np.zeros(nq.value + 1, dtype=np.int32)
    col_idx = np.zeros(max(1, npairs.value), dtype=np.int32)
    flags = np.zeros(max(1, npairs.value), dtype=np.uint8)
    _check(lib().clear_attn_schedule_host(*args, ctypes.byref(nq), ctypes.byref(npairs), row_ptr.ctypes.data,
                                          col_idx.ctypes.data, flags.ctypes.data))
    return row_ptr, col_idx[:npairs.value], flags[:npairs.value]


def clear_attn_schedule_host_masked(gridH, gridW, r, mask_kind, shift, q_tile_h, q_tile_w, k_tile_h, k_tile_w):
    """clear_attn_schedule_host for a mask kind."""
    nq, npairs = ctypes.c_int(0), ctypes.c_longlong(0)
    args = (gridH, gridW, r, mask_kind, shift, q_tile_h, q_tile_w, k_tile_h, k_tile_w)
    _check(lib().clear_attn_schedule_host_masked(*args, ctypes.byref(nq), ctypes.byref(npairs), None, None, None))
    row_ptr = np.zeros(nq.value + 1, dtype=np.int32)
    col_idx = np.zeros(max(1, npairs.value), dtype=np.int32)
    flags = np.zeros(max(1, npairs.value), dtype=np.uint8)
    _check(lib().clear_attn_schedule_host_masked(*args, ctypes.byref(nq), ctypes.byref(npairs), row_ptr.ctypes.data,
                                                 col_idx.ctypes.data, flags.ctypes.data))
    return row_ptr, col_idx[:npairs.value], flags[:npairs.value]


def _dtype_code(t):
    import torch
    if t.dtype == torch.bfloat16:
        return CLEAR_BF16
    if t.dtype == torch.float32:
        return CLEAR_F32
    raise ClearAttnError(CLEAR_ERR_UNSUPPORTED, "tensors must be bfloat16 or float32")


def _check_plain(ref, named, what="tensors"):
    """The plain-layout entry points read their tensors as packed [B, H, N, head_dim] arrays: every tensor in `named`
    (name -> tensor, None entries skipped) must be a contiguous device tensor on ref's device with ref's shape and dtype."""
    for name, t in named.items():
        if t is None:
            continue
        if not (t.is_cuda and t.device == ref.device and t.is_contiguous() and t.dim() == 4 and t.dtype == ref.dtype and t.shape == ref.shape):
            raise ClearAttnError(CLEAR_ERR_INVALID_ARG, "%s: %s must be a contiguous device tensor with the shape, dtype and device of Q "
                                 "(use the *_strided entry points for transposed or sliced views)" % (what, name))


def _check_f32(ref, name, t, shape):
    import torch
    if t is not None and not (t.is_cuda and t.device == ref.device and t.is_contiguous() and t.dtype == torch.float32 and tuple(t.shape) == tuple(shape)):
        raise ClearAttnError(CLEAR_ERR_INVALID_ARG, "%s must be a contiguous fp32 device tensor of shape %s" % (name, tuple(shape)))


class ClearAttn:
    """Owns one clear_attn_ctx (clear_attn_create / clear_attn_forward / clear_attn_destroy)."""

    def __init__(self, n_text, gridH, gridW, head_dim, r, dtype, mask_kind=CLEAR_MASK_DISC, shift=0):
        self._ctx = ctypes.c_void_p(None)
        self.shape = (n_text, gridH, gridW, head_dim, r)
        self.dtype = dtype
        self.mask = (mask_kind, shift)
        if mask_kind == CLEAR_MASK_DISC and shift == 0:
            _check(lib().clear_attn_create(ctypes.byref(self._ctx), n_text, gridH, gridW, head_dim, r, dtype))
        else:
            _check(lib().clear_attn_create_masked(ctypes.byref(self._ctx), n_text, gridH, gridW, head_dim, r, dtype, mask_kind, shift))

    def reserve(self, BH):
        _check(lib().clear_attn_reserve(self._ctx, BH), self._ctx)

    def forward(self, Q, K, V, O=None, stream=None):
        """Q, K, V: contiguous device tensors [B, H, N, head_dim]; enqueues on `stream` (default: torch's current)."""
        import torch
        n_text, gridH, gridW, head_dim, r = self.shape
        B, H, N, d = self._check_call(Q, {"Q": Q, "K": K, "V": V, "O": O}, "forward")
        if O is None:
            O = torch.empty_like(Q)
        s = torch.cuda.current_stream(Q.device).cuda_stream if stream is None else stream
        _check(lib().clear_attn_forward(self._ctx, Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), B, H,
                                        n_text, gridH, gridW, head_dim, r, ctypes.c_void_p(s)), self._ctx)
        return O

    def _check_call(self, Q, named, what):
        """Shape / dtype of Q against the context, then the plain-layout checks on every tensor of `named`."""
        n_text, gridH, gridW, head_dim, r = self.shape
        if Q.dim() != 4:
            raise ClearAttnError(CLEAR_ERR_INVALID_ARG, "%s: Q must be [B, H, N, head_dim]" % what)
        if _dtype_code(Q) != self.dtype:
            raise ClearAttnError(CLEAR_ERR_MISMATCH, "tensor dtype differs from the context's")
        B, H, N, d = Q.shape
        if N != n_text + gridH * gridW or d != head_dim:
            raise ClearAttnError(CLEAR_ERR_MISMATCH, "tensor shape differs from the context's")
        _check_plain(Q, named, what)
        return B, H, N, d

    def forward_noalloc(self, Q, K, V, O, stream=None):
        """clear_attn_forward_noalloc: the forward pass without any device allocation (O is the caller's)."""
        import torch
        n_text, gridH, gridW, head_dim, r = self.shape
        B, H, N, d = self._check_call(Q, {"Q": Q, "K": K, "V": V, "O": O}, "forward_noalloc")
        s = torch.cuda.current_stream(Q.device).cuda_stream if stream is None else stream
        _check(lib().clear_attn_forward_noalloc(self._ctx, Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), B, H,
                                                n_text, gridH, gridW, head_dim, r, ctypes.c_void_p(s)), self._ctx)
        return O

    def forward_prologue(self, Q, K, V, O=None, q_gain=None, k_gain=None, norm_eps=1e-6, rope_y=None, rope_x=None, logit_scale=1.0,
                         stream=None):
        """clear_attn_forward_prologue: Q, K raw; gains fp32 [head_dim]; rope tables fp32 [grid, head_dim/2, 2]."""
        import torch
        n_text, gridH, gridW, head_dim, r = self.shape
        B, H, N, d = self._check_call(Q, {"Q": Q, "K": K, "V": V, "O": O}, "forward_prologue")
        _check_prologue_tables(Q.device, head_dim, gridH, gridW, (q_gain, k_gain), rope_y, rope_x)
        if O is None:
            O = torch.empty_like(Q)
        s = torch.cuda.current_stream(Q.device).cuda_stream if stream is None else stream
        ptr = lambda t: None if t is None else t.data_ptr()
        _check(lib().clear_attn_forward_prologue(self._ctx, Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), B, H, n_text, gridH, gridW,
                                                 head_dim, r, ptr(q_gain), ptr(k_gain), norm_eps, ptr(rope_y), ptr(rope_x), logit_scale,
                                                 ctypes.c_void_p(s)), self._ctx)
        return O

    def forward_strided(self, Q, K, V, O=None, stream=None, q_gain=None, k_gain=None, norm_eps=1e-6, rope_y=None, rope_x=None,
                        logit_scale=None, lse=None):
        """clear_attn_forward_strided (or, with any prologue argument, clear_attn_forward_prologue_strided): Q, K, V, O are
        [B, H, N, head_dim] views with any batch / head / token strides and contiguous channels, e.g. transposed views
        of [B, N, H, head_dim] tensors or slices of a packed QKV tensor.  O defaults to a new tensor laid out like Q."""
        import torch
        n_text, gridH, gridW, head_dim, r = self.shape
        B, H, N, d = Q.shape
        if N != n_text + gridH * gridW or d != head_dim or _dtype_code(Q) != self.dtype:
            raise ClearAttnError(CLEAR_ERR_MISMATCH, "tensor shape or dtype differs from the context's")
        if O is None:
            O = torch.empty_strided(Q.shape, Q.stride(), dtype=Q.dtype, device=Q.device)
        for t in (Q, K, V, O):
            if not (t.is_cuda and t.shape == Q.shape and t.dtype == Q.dtype and t.stride(3) == 1):
                raise ClearAttnError(CLEAR_ERR_INVALID_ARG, "Q, K, V, O must be device tensors of one shape and dtype with contiguous channels")
        strides = (ctypes.c_longlong * 12)(*[t.stride(k) for t in (Q, K, V, O) for k in (0, 1, 2)])
        s = torch.cuda.current_stream(Q.device).cuda_stream if stream is None else stream
        prologue = any(x is not None for x in (q_gain, k_gain, rope_y, rope_x, logit_scale))
        if prologue:
            _check_prologue_tables(Q.device, head_dim, gridH, gridW, (q_gain, k_gain), rope_y, rope_x)
            ptr = lambda t: None if t is None else t.data_ptr()
            _check(lib().clear_attn_forward_prologue_strided(self._ctx, Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), strides, B, H,
                                                             n_text, gridH, gridW, head_dim, r, ptr(q_gain), ptr(k_gain), norm_eps, ptr(rope_y),
                                                             ptr(rope_x), 1.0 if logit_scale is None else logit_scale, ctypes.c_void_p(s)),
                   self._ctx)
        else:
            _check(lib().clear_attn_forward_strided(self._ctx, Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(),
                                                    None if lse is None else lse.data_ptr(), strides, B, H,
                                                    n_text, gridH, gridW, head_dim, r, ctypes.c_void_p(s)), self._ctx)
        return O

    def backward_strided(self, Q, K, V, O, dO, lse, stream=None):
        """clear_attn_backward_strided: Q, K, V, O, dO are [B, H, N, head_dim] views with any batch / head / token strides
        and contiguous channels; returns (dQ, dK, dV) laid out like Q, K, V."""
        import torch
        n_text, gridH, gridW, head_dim, r = self.shape
        B, H, N, d = Q.shape
        outs = [torch.empty_strided(t.shape, t.stride(), dtype=t.dtype, device=t.device) if min(t.stride()[:3]) > 0 else torch.empty_like(t)
                for t in (Q, K, V)]
        for t in (Q, K, V, O, dO, *outs):
            if not (t.is_cuda and t.shape == Q.shape and t.dtype == Q.dtype and t.stride(3) == 1):
                raise ClearAttnError(CLEAR_ERR_INVALID_ARG, "tensors must be device tensors of one shape and dtype with contiguous channels")
        strides = (ctypes.c_longlong * 24)(*[t.stride(k) for t in (Q, K, V, O, dO, *outs) for k in (0, 1, 2)])
        s = torch.cuda.current_stream(Q.device).cuda_stream if stream is None else stream
        _check(lib().clear_attn_backward_strided(self._ctx, Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), dO.data_ptr(), lse.data_ptr(),
                                                 outs[0].data_ptr(), outs[1].data_ptr(), outs[2].data_ptr(), strides, B, H, n_text, gridH, gridW,
                                                 head_dim, r, ctypes.c_void_p(s)), self._ctx)
        return tuple(outs)

    def forward_lse(self, Q, K, V, O=None, lse=None, stream=None):
        """clear_attn_forward_lse: returns (O, lse) with lse fp32 [B, H, N]."""
        import torch
        n_text, gridH, gridW, head_dim, r = self.shape
        B, H, N, d = self._check_call(Q, {"Q": Q, "K": K, "V": V, "O": O}, "forward_lse")
        _check_f32(Q, "lse", lse, (B, H, N))
        if O is None:
            O = torch.empty_like(Q)
        if lse is None:
            lse = torch.empty((B, H, N), dtype=torch.float32, device=Q.device)
        s = torch.cuda.current_stream(Q.device).cuda_stream if stream is None else stream
        _check(lib().clear_attn_forward_lse(self._ctx, Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), lse.data_ptr(), B, H,
                                            n_text, gridH, gridW, head_dim, r, ctypes.c_void_p(s)), self._ctx)
        return O, lse

    def backward(self, Q, K, V, O, dO, lse, stream=None):
        """clear_attn_backward: returns (dQ, dK, dV)."""
        import torch
        n_text, gridH, gridW, head_dim, r = self.shape
        B, H, N, d = self._check_call(Q, {"Q": Q, "K": K, "V": V, "O": O, "dO": dO}, "backward")
        if lse is None:
            raise ClearAttnError(CLEAR_ERR_INVALID_ARG, "backward: lse (from forward_lse) is required")
        _check_f32(Q, "lse", lse, (B, H, N))
        dQ, dK, dV = torch.empty_like(Q), torch.empty_like(Q), torch.empty_like(Q)
        s = torch.cuda.current_stream(Q.device).cuda_stream if stream is None else stream
        _check(lib().clear_attn_backward(self._ctx, Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), dO.data_ptr(), lse.data_ptr(),
                                         dQ.data_ptr(), dK.data_ptr(), dV.data_ptr(), B, H, n_text, gridH, gridW, head_dim, r,
                                         ctypes.c_void_p(s)), self._ctx)
        return dQ, dK, dV

    def forward_band(self, Q, K, V, O, own_y0, own_y1, text_keys, text_o=None, text_lse=None, stream=None):
        """clear_attn_forward_band on the context's (local) grid.  Returns (O, text_o, text_lse)."""
        import torch
        n_text, gridH, gridW, head_dim, r = self.shape
        B, H, N, d = self._check_call(Q, {"Q": Q, "K": K, "V": V, "O": O}, "forward_band")
        if O is None:
            raise ClearAttnError(CLEAR_ERR_INVALID_ARG, "forward_band: O is required (rows outside the band are left as they are)")
        _check_f32(Q, "text_o", text_o, (B, H, n_text, d))
        _check_f32(Q, "text_lse", text_lse, (B, H, n_text))
        if n_text > 0:
            if text_o is None:
                text_o = torch.empty((B, H, n_text, d), dtype=torch.float32, device=Q.device)
            if text_lse is None:
                text_lse = torch.empty((B, H, n_text), dtype=torch.float32, device=Q.device)
        s = torch.cuda.current_stream(Q.device).cuda_stream if stream is None else stream
        _check(lib().clear_attn_forward_band(
            self._ctx, Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), B, H, n_text, gridH, gridW, head_dim, r,
            own_y0, own_y1, int(bool(text_keys)), ctypes.c_void_p(text_o.data_ptr() if text_o is not None else None),
            ctypes.c_void_p(text_lse.data_ptr() if text_lse is not None else None), ctypes.c_void_p(s)), self._ctx)
        return O, text_o, text_lse

    def forward_profile(self, Q, K, V, O, reps=5, stream=None):
        """Average milliseconds per launch of (image-query, text-query, merge) kernels; synchronises."""
        import torch
        n_text, gridH, gridW, head_dim, r = self.shape
        B, H, N, d = self._check_call(Q, {"Q": Q, "K": K, "V": V, "O": O}, "forward_profile")
        if O is None:
            raise ClearAttnError(CLEAR_ERR_INVALID_ARG, "forward_profile: O is required")
        s = torch.cuda.current_stream(Q.device).cuda_stream if stream is None else stream
        ms = (ctypes.c_float * 3)()
        _check(lib().clear_attn_forward_profile(self._ctx, Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), B, H,
                                                n_text, gridH, gridW, head_dim, r, ctypes.c_void_p(s), reps, ms), self._ctx)
        return tuple(float(x) for x in ms)

    def schedule_size(self):
        v = [ctypes.c_int(0) for _ in range(5)]
        npairs = ctypes.c_longlong(0)
        _check(lib().clear_attn_schedule_size(self._ctx, *[ctypes.byref(x) for x in v], ctypes.byref(npairs)), self._ctx)
        return tuple(int(x.value) for x in v) + (int(npairs.value),)

    def schedule_copy(self):
        *_, nq, npairs = self.schedule_size()
        row_ptr = np.zeros(nq + 1, dtype=np.int32)
        col_idx = np.zeros(max(1, npairs), dtype=np.int32)
        flags = np.zeros(max(1, npairs), dtype=np.uint8)
        _check(lib().clear_attn_schedule_copy(self._ctx, row_ptr.ctypes.data, col_idx.ctypes.data, flags.ctypes.data), self._ctx)
        return row_ptr, col_idx[:npairs], flags[:npairs]

    def executed_pairs(self):
        out = ctypes.c_ulonglong(0)
        _check(lib().clear_attn_executed_pairs(self._ctx, ctypes.byref(out)), self._ctx)
        return int(out.value)

    def destroy(self):
        if self._ctx:
            lib().clear_attn_destroy(self._ctx)
            self._ctx = ctypes.c_void_p(None)

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def _check_prologue_tables(device, head_dim, gridH, gridW, gains, rope_y, rope_x):
    import torch
    for g in gains:
        if g is not None and not (g.is_cuda and g.device == device and g.dtype == torch.float32 and g.is_contiguous() and g.shape == (head_dim,)):
            raise ClearAttnError(CLEAR_ERR_INVALID_ARG, "gains must be contiguous fp32 device tensors [head_dim]")
    for t, n in ((rope_y, gridH), (rope_x, gridW)):
        if t is not None and not (t.is_cuda and t.device == device and t.dtype == torch.float32 and t.is_contiguous()
                                  and t.shape == (n, head_dim // 2, 2)):
            raise ClearAttnError(CLEAR_ERR_INVALID_ARG, "rotary tables must be contiguous fp32 device tensors [grid, head_dim/2, 2]")


def clear_attn_qk_prologue(X, n_text, gridH, gridW, gain=None, norm_eps=1e-6, rope_y=None, rope_x=None, out=None, stream=None):
    """clear_attn_qk_prologue on a bf16 device tensor [B, H, N, head_dim]; out may be X itself."""
    import torch
    B, H, N, d = X.shape
    if not (X.is_cuda and X.is_contiguous() and X.dtype == torch.bfloat16 and N == n_text + gridH * gridW):
        raise ClearAttnError(CLEAR_ERR_INVALID_ARG, "X must be a contiguous bf16 device tensor [B, H, n_text + gridH*gridW, head_dim]")
    _check_prologue_tables(X.device, d, gridH, gridW, (gain,), rope_y, rope_x)
    if out is None:
        out = torch.empty_like(X)
    s = torch.cuda.current_stream(X.device).cuda_stream if stream is None else stream
    ptr = lambda t: None if t is None else t.data_ptr()
    _check(lib().clear_attn_qk_prologue(X.data_ptr(), out.data_ptr(), B, H, n_text, gridH, gridW, d, ptr(gain), norm_eps, ptr(rope_y),
                                        ptr(rope_x), ctypes.c_void_p(s)))
    return out


def clear_attn_band_layout(gridH_total, r, n_bands, band):
    """(y0, y1, halo_top, halo_bottom) of one band."""
    v = [ctypes.c_int(0) for _ in range(4)]
    _check(lib().clear_attn_band_layout(gridH_total, r, n_bands, band, *[ctypes.byref(x) for x in v]))
    return tuple(int(x.value) for x in v)


def clear_attn_merge_text(text_o, text_lse, O, n_text, mode, stream=None):
    """Combines per-band text results (lists of device tensors) into the text rows of O [B, H, N, d]."""
    import torch
    n = len(text_o)
    B, H, N, d = O.shape
    po = (ctypes.c_void_p * n)(*[t.data_ptr() for t in text_o])
    pl = (ctypes.c_void_p * n)(*[t.data_ptr() for t in text_lse])
    s = torch.cuda.current_stream(O.device).cuda_stream if stream is None else stream
    _check(lib().clear_attn_merge_text(n, po, pl, B, H, n_text, ctypes.c_longlong(N), d, mode, ctypes.c_void_p(O.data_ptr()),
                                       _dtype_code(O), ctypes.c_void_p(s)))
    return O


def clear_attn_forward_once(Q, K, V, n_text, gridH, gridW, r):
    """create + forward + destroy for one call (tests, smoke)."""
    ctx = ClearAttn(n_text, gridH, gridW, Q.shape[-1], r, _dtype_code(Q))
    try:
        import torch
        O = ctx.forward(Q, K, V)
        torch.cuda.synchronize(Q.device)
        return O
    finally:
        ctx.destroy()
