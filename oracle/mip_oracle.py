"""ctypes front end of the plain-C oracle in ``mip_gemm_oracle.c``.

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
CPU-baseline leg of the benchmark.  The GPU library never imports this module
and this module never imports the GPU library.

The arithmetic lives entirely in the C file (three plain loops, paper Section 3
``C += A * B`` with INT8 operands and an INT32 accumulator as stated in
Section 5); this file only builds it with the host compiler and marshals numpy
buffers.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading

import numpy as np

ROW_MAJOR, COL_MAJOR = 0, 1
OVERWRITE, ACCUMULATE = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mip_gemm_oracle.c")
_LIB = os.path.join(_HERE, "libmip_oracle.so")
_lock = threading.Lock()
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with the host C compiler (-O2, OpenMP over rows only)."""
    stale = (not os.path.exists(_LIB)
             or os.path.getmtime(_LIB) < os.path.getmtime(_SRC))
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99",
             "-Wall", "-Wextra", "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    with _lock:
        if _lib is None:
            lib = ctypes.CDLL(build())
            i64, vp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
            lib.oracle_mip_gemm.restype = ci
            lib.oracle_mip_gemm.argtypes = [ci, ci, i64, i64, i64,
                                            vp, i64, ci, vp, i64, ci,
                                            vp, i64, ci, ci]
            lib.oracle_mip_gemm_dequant.restype = ci
            lib.oracle_mip_gemm_dequant.argtypes = [ci, ci, i64, i64, i64, vp, i64, ci, vp, i64, ci,
                                                    ctypes.c_float, vp, i64, ci, ci, vp]
            lib.oracle_num_threads.restype = ci
            _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _min_len(rows, cols, ld, order):
    if rows == 0 or cols == 0:
        return 0
    return (rows - 1) * ld + cols if order == ROW_MAJOR else (cols - 1) * ld + rows


def gemm(a_unsigned, b_unsigned, m, n, k, A, lda, orderA, B, ldb, orderB,
         C, ldc, orderC, mode):
    """C (m x n, int32) = [C +] A (m x k) * B (k x n), in place on the flat buffer ``C``.

    ``A``, ``B``, ``C`` are flat, contiguous numpy buffers (int8 or uint8 for
    the operands as the flags say, int32 for ``C``) that hold the matrices in
    the given order with the given leading dimension, counted in elements.
    """
    A = np.asarray(A)
    B = np.asarray(B)
    want_a = np.uint8 if a_unsigned else np.int8
    want_b = np.uint8 if b_unsigned else np.int8
    if A.dtype != want_a or B.dtype != want_b or C.dtype != np.int32:
        raise TypeError("operand dtypes do not match the entry point")
    for X in (A, B, C):
        if X.ndim != 1 or not X.flags.c_contiguous:
            raise ValueError("operands must be flat contiguous buffers")
    if not C.flags.writeable:
        raise ValueError("C must be writeable")
    if A.size < _min_len(m, k, lda, orderA) or B.size < _min_len(k, n, ldb, orderB) \
            or C.size < _min_len(m, n, ldc, orderC):
        raise ValueError("buffer shorter than the matrix it is said to hold")
    rc = _load().oracle_mip_gemm(
        int(bool(a_unsigned)), int(bool(b_unsigned)), m, n, k,
        A.ctypes.data, lda, orderA, B.ctypes.data, ldb, orderB,
        C.ctypes.data, ldc, orderC, mode)
    if rc != 0:
        raise ValueError("oracle rejected the arguments (rc=%d)" % rc)
    return C


def gemm_s8s8s32(m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC, mode):
    return gemm(False, False, m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC, mode)


def gemm_u8s8s32(m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC, mode):
    return gemm(True, False, m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC, mode)


def gemm_s8u8s32(m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC, mode):
    return gemm(False, True, m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC, mode)


def gemm_dequant(a_unsigned, b_unsigned, m, n, k, A, lda, orderA, B, ldb, orderB, scale,
                 C0, ldc, orderC, mode):
    """scale * (A * B) [+ C0] in fp64 (paper Section 7.3, C^r = s_A s_B C^q), dense (m, n) array.

    ``scale`` is rounded to float32 first, as the GPU entry points take a float.
    ``C0`` is the flat float32 buffer to be updated (only read, only in accumulate mode).
    """
    A = np.asarray(A)
    B = np.asarray(B)
    want_a = np.uint8 if a_unsigned else np.int8
    want_b = np.uint8 if b_unsigned else np.int8
    if A.dtype != want_a or B.dtype != want_b:
        raise TypeError("operand dtypes do not match the entry point")
    if A.size < _min_len(m, k, lda, orderA) or B.size < _min_len(k, n, ldb, orderB):
        raise ValueError("buffer shorter than the matrix it is said to hold")
    c_ptr = None
    if C0 is not None:
        C0 = np.asarray(C0)
        if C0.dtype != np.float32 or C0.size < _min_len(m, n, ldc, orderC):
            raise ValueError("C0 must be a float32 buffer that holds the m x n matrix")
        c_ptr = C0.ctypes.data
    out = np.empty((m, n), dtype=np.float64)
    rc = _load().oracle_mip_gemm_dequant(
        int(bool(a_unsigned)), int(bool(b_unsigned)), m, n, k, A.ctypes.data, lda, orderA,
        B.ctypes.data, ldb, orderB, float(np.float32(scale)), c_ptr, ldc, orderC, mode,
        out.ctypes.data)
    if rc != 0:
        raise ValueError("oracle rejected the arguments (rc=%d)" % rc)
    return out
