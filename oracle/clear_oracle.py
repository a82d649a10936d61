"""ctypes front end of the CPU oracle (oracle/clear_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the bench's cpu_baseline leg.
Nothing here is shared with the HIP path, and nothing here imports it.  All arithmetic lives in
the C file; this module only marshals numpy arrays (widening bf16 / fp32 inputs to fp64, which
is exact) and derives the CSR form of the brute-force tile schedule from the pair counts.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "clear_oracle.c")
_LIB = os.path.join(_HERE, "libclear_oracle.so")
_lib = None


def build(force=False):
    """Compile the oracle with gcc (-O2, OpenMP).  Returns the path of the shared library."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i64, i32, u64 = ctypes.c_int64, ctypes.c_int, ctypes.c_uint64
        vp = ctypes.c_void_p
        lib.oracle_mask.restype = i32
        lib.oracle_mask.argtypes = [i64, i64, i32, i32, i32, i32]
        lib.oracle_row_count.restype = i64
        lib.oracle_row_count.argtypes = [i64, i32, i32, i32, i32]
        lib.oracle_backward_dq_rows.restype = i32
        lib.oracle_backward_dq_rows.argtypes = [vp, vp, vp, vp, vp, i64, i32, i32, i32, i32, i32, vp]
        lib.oracle_backward_dkv_cols.restype = i32
        lib.oracle_backward_dkv_cols.argtypes = [vp, vp, vp, vp, vp, i64, i32, i32, i32, i32, i32, vp, vp]
        lib.oracle_set_mask.restype = None
        lib.oracle_set_mask.argtypes = [i32, i32]
        lib.oracle_mask_count.restype = u64
        lib.oracle_mask_count.argtypes = [i32, i32, i32, i32]
        lib.oracle_mask_dense.restype = None
        lib.oracle_mask_dense.argtypes = [i32, i32, i32, i32, vp]
        lib.oracle_attention_rows.restype = i32
        lib.oracle_attention_rows.argtypes = [vp, vp, vp, vp, i64, i32, i32, i32, i32, i32, vp, vp, vp, vp]
        lib.oracle_tile_pair_counts.restype = None
        lib.oracle_tile_pair_counts.argtypes = [i32] * 7 + [vp]
        lib.oracle_num_threads.restype = i32
        _lib = lib
    return _lib


MASK_DISC, MASK_SQUARE, MASK_SWIN, MASK_STRIDED = 0, 1, 2, 3


class mask_kind:
    """Context manager: `with mask_kind(MASK_SQUARE): ...` makes every oracle call inside use that local mask
    for the image-image pairs (process-wide setting of the C library; the disc of Eq. 3 outside)."""

    def __init__(self, kind, shift=0):
        self.kind, self.shift = kind, shift

    def __enter__(self):
        _load().oracle_set_mask(self.kind, self.shift)

    def __exit__(self, *exc):
        _load().oracle_set_mask(MASK_DISC, 0)


def num_threads():
    return int(_load().oracle_num_threads())


def mask(i, j, n_text, gridH, gridW, r):
    """Eq. 3 for one (query row, key column), 0-based."""
    return int(_load().oracle_mask(i, j, n_text, gridH, gridW, r))


def row_count(i, n_text, gridH, gridW, r):
    return int(_load().oracle_row_count(i, n_text, gridH, gridW, r))


def mask_count(n_text, gridH, gridW, r):
    """sum(M) by visiting every (i, j) of the N x N mask."""
    return int(_load().oracle_mask_count(n_text, gridH, gridW, r))


def mask_dense(n_text, gridH, gridW, r):
    N = n_text + gridH * gridW
    M = np.zeros((N, N), dtype=np.uint8)
    _load().oracle_mask_dense(n_text, gridH, gridW, r, M.ctypes.data)
    return M


def _f64(a):
    """Exact widening to a contiguous fp64 numpy array (accepts numpy arrays or torch CPU tensors)."""
    if hasattr(a, "detach"):  # torch tensor, without importing torch here
        a = a.detach().cpu()
        a = a.double().numpy() if str(a.dtype) != "torch.float64" else a.numpy()
    return np.ascontiguousarray(a, dtype=np.float64)


def attention_rows(Q, K, V, rows, n_text, gridH, gridW, r, return_stats=False):
    """Dense masked softmax attention for the given rows of one [N, d] (batch, head) slice."""
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    N, d = Q.shape
    assert N == n_text + gridH * gridW and K.shape == (N, d) and V.shape == (N, d)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    assert rows.ndim == 1 and (rows.size == 0 or (rows.min() >= 0 and rows.max() < N))
    O = np.empty((rows.size, d), dtype=np.float64)
    m = np.empty(rows.size, dtype=np.float64)
    l = np.empty(rows.size, dtype=np.float64)
    cnt = np.empty(rows.size, dtype=np.int64)
    if rows.size:
        rc = _load().oracle_attention_rows(Q.ctypes.data, K.ctypes.data, V.ctypes.data, rows.ctypes.data,
                                           rows.size, n_text, gridH, gridW, d, r, O.ctypes.data,
                                           m.ctypes.data, l.ctypes.data, cnt.ctypes.data)
        if rc != 0:
            raise RuntimeError("oracle_attention_rows failed")
    return (O, m, l, cnt) if return_stats else O


def backward_dq_rows(Q, K, V, dO, rows, n_text, gridH, gridW, r):
    """dQ of the given query rows of one [N, d] slice, for upstream gradient dO [N, d].  fp64 [len(rows), d]."""
    lib = _load()
    Q, K, V, dO = _f64(Q), _f64(K), _f64(V), _f64(dO)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    d = Q.shape[1]
    out = np.zeros((len(rows), d), dtype=np.float64)
    rc = lib.oracle_backward_dq_rows(Q.ctypes.data, K.ctypes.data, V.ctypes.data, dO.ctypes.data, rows.ctypes.data, len(rows),
                                     n_text, gridH, gridW, d, r, out.ctypes.data)
    if rc != 0:
        raise RuntimeError("oracle_backward_dq_rows failed")
    return out


def backward_dkv_cols(Q, K, V, dO, cols, n_text, gridH, gridW, r):
    """(dK, dV) of the given key columns of one [N, d] slice.  fp64 [len(cols), d] each."""
    lib = _load()
    Q, K, V, dO = _f64(Q), _f64(K), _f64(V), _f64(dO)
    cols = np.ascontiguousarray(cols, dtype=np.int64)
    d = Q.shape[1]
    dK = np.zeros((len(cols), d), dtype=np.float64)
    dV = np.zeros((len(cols), d), dtype=np.float64)
    rc = lib.oracle_backward_dkv_cols(Q.ctypes.data, K.ctypes.data, V.ctypes.data, dO.ctypes.data, cols.ctypes.data, len(cols),
                                      n_text, gridH, gridW, d, r, dK.ctypes.data, dV.ctypes.data)
    if rc != 0:
        raise RuntimeError("oracle_backward_dkv_cols failed")
    return dK, dV


def backward(Q, K, V, dO, n_text, gridH, gridW, r):
    """(dQ, dK, dV) for every token of one [N, d] slice."""
    N = Q.shape[0]
    idx = np.arange(N, dtype=np.int64)
    dK, dV = backward_dkv_cols(Q, K, V, dO, idx, n_text, gridH, gridW, r)
    return backward_dq_rows(Q, K, V, dO, idx, n_text, gridH, gridW, r), dK, dV


def attention(Q, K, V, n_text, gridH, gridW, r):
    """All rows, all heads.  Q, K, V: [B, H, N, d].  Returns fp64 [B, H, N, d]."""
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    B, H, N, d = Q.shape
    rows = np.arange(N, dtype=np.int64)
    O = np.empty((B, H, N, d), dtype=np.float64)
    for b in range(B):
        for h in range(H):
            O[b, h] = attention_rows(Q[b, h], K[b, h], V[b, h], rows, n_text, gridH, gridW, r)
    return O


def tile_pair_counts(gridH, gridW, r, qth, qtw, kth, ktw):
    nq = -(-gridH // qth) * -(-gridW // qtw)
    nk = -(-gridH // kth) * -(-gridW // ktw)
    cnt = np.zeros((nq, nk), dtype=np.int32)
    _load().oracle_tile_pair_counts(gridH, gridW, r, qth, qtw, kth, ktw, cnt.ctypes.data)
    return cnt


def tile_schedule(gridH, gridW, r, qth, qtw, kth, ktw):
    """Brute-force schedule in CSR form: (row_ptr[int32], col_idx[int32], flags[uint8]).

    Key tile kt is listed for query tile qt iff some in-grid element pair is unmasked; its flag is 1
    (FULL) iff every one of the qth*qtw*kth*ktw slot pairs is in-grid and unmasked, else 0 (PARTIAL).
    Key tiles ascend within a row."""
    cnt = tile_pair_counts(gridH, gridW, r, qth, qtw, kth, ktw)
    listed = cnt > 0
    row_ptr = np.zeros(cnt.shape[0] + 1, dtype=np.int32)
    row_ptr[1:] = np.cumsum(listed.sum(axis=1))
    qt, kt = np.nonzero(listed)  # row-major: ascending kt within each qt
    flags = (cnt[qt, kt] == qth * qtw * kth * ktw).astype(np.uint8)
    return row_ptr, kt.astype(np.int32), flags
