"""CPU oracle for padded, strided 2-D convolution and its sparse matrix T = C P.

TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the test-suite, the smoke check and
the benchmark's CPU-baseline leg may import this package.  It shares nothing
with the GPU library and never imports it.

The arithmetic lives in ``conv_oracle.c`` (plain C, double accumulation); this
module only compiles it with gcc and marshals numpy arrays through ctypes.
``paper_matrices`` holds the paper's dense P and C (Section 2 / Section 3) for
tiny shapes, used to pin the C code to the paper's own construction.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "conv_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lock = threading.Lock()
_lib = None


def build(force: bool = False) -> str:
    """Compile conv_oracle.c into liboracle.so (OpenMP, -O2).  Returns its path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
               "-o", tmp, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    with _lock:
        if _lib is None:
            # CONV_ORACLE_LIB: a library to load instead (tests/test_oracle_planted_mistakes.py compiles
            # copies of conv_oracle.c with one mistake each and checks that the pins catch it)
            lib = ctypes.CDLL(os.environ.get("CONV_ORACLE_LIB") or build())
            i, i64, vp = ctypes.c_int, ctypes.c_int64, ctypes.c_void_p
            lib.oracle_out_shape.argtypes = [i] * 5 + [ctypes.POINTER(i64)] * 2
            lib.oracle_out_shape.restype = i
            lib.oracle_nnz_closed.argtypes = [i] * 5
            lib.oracle_nnz_closed.restype = i64
            lib.oracle_nnz_brute.argtypes = [i] * 5
            lib.oracle_nnz_brute.restype = i64
            lib.oracle_csr_row.argtypes = [i] * 5 + [vp, i64, vp, vp]
            lib.oracle_csr_row.restype = i64
            lib.oracle_csr.argtypes = [i] * 5 + [vp, vp, vp, vp, i64]
            lib.oracle_csr.restype = i64
            lib.oracle_conv.argtypes = [i] * 6 + [vp, vp, vp, vp]
            lib.oracle_conv.restype = i
            lib.oracle_csc.argtypes = [i] * 5 + [vp, vp, vp, vp, i64]
            lib.oracle_csc.restype = i64
            lib.oracle_conv_t.argtypes = [i] * 6 + [vp, vp, vp, vp]
            lib.oracle_conv_t.restype = i
            lib.oracle_compact_rows.argtypes = [i] * 5 + [vp]
            lib.oracle_compact_rows.restype = i64
            lib.oracle_compact_decode.argtypes = [i, i, i64, vp, vp, vp, vp, vp, i64]
            lib.oracle_compact_decode.restype = i64
            lib.oracle_conv_channels.argtypes = [i] * 7 + [vp, vp, vp, vp]
            lib.oracle_conv_channels.restype = i
            _lib = lib
    return _lib


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def out_shape(m, n, k, s, p):
    """(m_out, n_out) of Theorem 2.1; ValueError if k > m + 2p or k > n + 2p."""
    mo, no = ctypes.c_int64(), ctypes.c_int64()
    if _load().oracle_out_shape(m, n, k, s, p, ctypes.byref(mo), ctypes.byref(no)) != 0:
        raise ValueError("invalid convolution shape %r" % ((m, n, k, s, p),))
    return int(mo.value), int(no.value)


def nnz_closed(m, n, k, s, p) -> int:
    """Theorem 2.1 evaluated as the printed double sum."""
    v = int(_load().oracle_nnz_closed(m, n, k, s, p))
    if v < 0:
        raise ValueError("invalid convolution shape")
    return v


def nnz_brute(m, n, k, s, p) -> int:
    """Taps that land on an entry of A, counted one window at a time on a 0/1 plane."""
    v = int(_load().oracle_nnz_brute(m, n, k, s, p))
    if v < 0:
        raise ValueError("invalid convolution shape")
    return v


def csr_row(m, n, k, s, p, K, row):
    """(cols int64[c], vals float32[c]) of one row of T, ascending columns."""
    K = _f32(K).reshape(k * k)
    cols = np.empty(k * k, dtype=np.int64)
    vals = np.empty(k * k, dtype=np.float32)
    c = int(_load().oracle_csr_row(m, n, k, s, p, K.ctypes.data, int(row),
                                   cols.ctypes.data, vals.ctypes.data))
    if c < 0:
        raise ValueError("invalid shape or row")
    return cols[:c].copy(), vals[:c].copy()


def csr(m, n, k, s, p, K):
    """(row_ptr int64[rows+1], col_idx int64[nnz], vals float32[nnz]) of T."""
    K = _f32(K).reshape(k * k)
    mo, no = out_shape(m, n, k, s, p)
    cap = mo * no * k * k
    row_ptr = np.empty(mo * no + 1, dtype=np.int64)
    col_idx = np.empty(cap, dtype=np.int64)
    vals = np.empty(cap, dtype=np.float32)
    nnz = int(_load().oracle_csr(m, n, k, s, p, K.ctypes.data, row_ptr.ctypes.data,
                                 col_idx.ctypes.data, vals.ctypes.data, cap))
    if nnz < 0:
        raise ValueError("oracle_csr failed (%d)" % nnz)
    return row_ptr, col_idx[:nnz].copy(), vals[:nnz].copy()


def conv(m, n, k, s, p, A, K, batch: int = 1, want_scale: bool = False):
    """Zero-pad then slide.  A: (m*n*batch,) batch-minor float32.  Returns out
    (m_out*n_out*batch,) float32, and the per-output sum of |K||A| (float64)
    when want_scale is set."""
    A = _f32(A).reshape(-1)
    K = _f32(K).reshape(k * k)
    if A.size != m * n * batch:
        raise ValueError("A has %d elements, expected %d" % (A.size, m * n * batch))
    mo, no = out_shape(m, n, k, s, p)
    out = np.empty(mo * no * batch, dtype=np.float32)
    scale = np.empty(mo * no * batch, dtype=np.float64) if want_scale else None
    rc = _load().oracle_conv(m, n, k, s, p, batch, A.ctypes.data, K.ctypes.data,
                             out.ctypes.data, scale.ctypes.data if want_scale else None)
    if rc != 0:
        raise ValueError("oracle_conv failed (%d)" % rc)
    return (out, scale) if want_scale else out


def csc(m, n, k, s, p, K):
    """(col_ptr int64[cols+1], row_idx int64[nnz], vals float32[nnz]): T column-compressed,
    rows ascending inside a column; equally the CSR arrays of T^T."""
    K = _f32(K).reshape(k * k)
    mo, no = out_shape(m, n, k, s, p)
    cap = mo * no * k * k
    col_ptr = np.empty(m * n + 1, dtype=np.int64)
    row_idx = np.empty(cap, dtype=np.int64)
    vals = np.empty(cap, dtype=np.float32)
    nnz = int(_load().oracle_csc(m, n, k, s, p, K.ctypes.data, col_ptr.ctypes.data,
                                 row_idx.ctypes.data, vals.ctypes.data, cap))
    if nnz < 0:
        raise ValueError("oracle_csc failed (%d)" % nnz)
    return col_ptr, row_idx[:nnz].copy(), vals[:nnz].copy()


def conv_t(m, n, k, s, p, U, K, batch: int = 1, want_scale: bool = False):
    """z = T^T u (the adjoint of the padded, strided convolution).  U: (m_out*n_out*batch,)
    batch-minor float32.  Returns z (m*n*batch,) float32 and optionally the sums of |K||u|."""
    U = _f32(U).reshape(-1)
    K = _f32(K).reshape(k * k)
    mo, no = out_shape(m, n, k, s, p)
    if U.size != mo * no * batch:
        raise ValueError("U has %d elements, expected %d" % (U.size, mo * no * batch))
    out = np.empty(m * n * batch, dtype=np.float32)
    scale = np.empty(m * n * batch, dtype=np.float64) if want_scale else None
    rc = _load().oracle_conv_t(m, n, k, s, p, batch, U.ctypes.data, K.ctypes.data,
                               out.ctypes.data, scale.ctypes.data if want_scale else None)
    if rc != 0:
        raise ValueError("oracle_conv_t failed (%d)" % rc)
    return (out, scale) if want_scale else out


def compact_rows(m, n, k, s, p):
    """Per-row descriptors of the structure-aware storage of T: int32 (rows, 2), column 0 the
    column index of the row's first entry, column 1 the packed tap ranges
    a_lo | r1 << 8 | b_lo << 16 | r2 << 24 (bit pattern); both 0 for a row without entries."""
    mo, no = out_shape(m, n, k, s, p)
    desc = np.empty((mo * no, 2), dtype=np.int32)
    rc = int(_load().oracle_compact_rows(m, n, k, s, p, desc.ctypes.data))
    if rc < 0:
        raise ValueError("oracle_compact_rows failed (%d)" % rc)
    return desc


def compact_decode(n, k, desc, ktab):
    """CSR (row_ptr, col_idx int64, vals float32) of the matrix that descriptors + value table
    stand for; the descriptors are taken as they are."""
    desc = np.ascontiguousarray(desc, dtype=np.int32).reshape(-1, 2)
    ktab = _f32(ktab).reshape(k * k)
    rows = desc.shape[0]
    cap = max(rows * k * k, 1)
    row_ptr = np.empty(rows + 1, dtype=np.int64)
    col_idx = np.empty(cap, dtype=np.int64)
    vals = np.empty(cap, dtype=np.float32)
    nnz = int(_load().oracle_compact_decode(n, k, rows, desc.ctypes.data, ktab.ctypes.data,
                                            row_ptr.ctypes.data, col_idx.ctypes.data,
                                            vals.ctypes.data, cap))
    if nnz < 0:
        raise ValueError("oracle_compact_decode failed (%d)" % nnz)
    return row_ptr, col_idx[:nnz].copy(), vals[:nnz].copy()


def conv_channels(m, n, k, s, p, A, K, channels, batch: int = 1, want_scale: bool = False):
    """Sum over `channels` input planes of the padded, strided convolution of plane ch with
    kernel ch.  A: (channels*m*n*batch,) planes one after the other, each batch-minor; K:
    (channels*k*k,).  Returns out (m_out*n_out*batch,) float32 (and the sums of |K||A|)."""
    A = _f32(A).reshape(-1)
    K = _f32(K).reshape(-1)
    if A.size != channels * m * n * batch or K.size != channels * k * k:
        raise ValueError("operand sizes do not match %d channels" % channels)
    mo, no = out_shape(m, n, k, s, p)
    out = np.empty(mo * no * batch, dtype=np.float32)
    scale = np.empty(mo * no * batch, dtype=np.float64) if want_scale else None
    rc = _load().oracle_conv_channels(m, n, k, s, p, batch, channels, A.ctypes.data, K.ctypes.data,
                                      out.ctypes.data, scale.ctypes.data if want_scale else None)
    if rc != 0:
        raise ValueError("oracle_conv_channels failed (%d)" % rc)
    return (out, scale) if want_scale else out
