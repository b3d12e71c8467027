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
_SRC_CONV = os.path.join(_HERE, "mip_conv_oracle.c")
_LIB = os.path.join(_HERE, "libmip_oracle.so")
_lock = threading.Lock()
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with the host C compiler (-O2, OpenMP over rows only)."""
    stale = (not os.path.exists(_LIB)
             or os.path.getmtime(_LIB) < max(os.path.getmtime(_SRC), os.path.getmtime(_SRC_CONV)))
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99",
             "-Wall", "-Wextra", "-o", tmp, _SRC, _SRC_CONV, "-lm"])
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
            lib.oracle_mip_gemm_s16.restype = ci
            lib.oracle_mip_gemm_s16.argtypes = [i64, i64, i64, vp, i64, ci, vp, i64, ci, vp, i64, ci, ci]
            lib.oracle_mip_gemm_dequant.restype = ci
            lib.oracle_mip_gemm_dequant.argtypes = [ci, ci, i64, i64, i64, vp, i64, ci, vp, i64, ci,
                                                    ctypes.c_float, vp, i64, ci, ci, vp]
            lib.oracle_mip_gemm_requant.restype = ci
            lib.oracle_mip_gemm_requant.argtypes = [ci, ci, i64, i64, i64, vp, i64, ci, vp, i64, ci,
                                                    ctypes.c_float, vp, i64, ci]
            lib.oracle_num_threads.restype = ci
            lib.oracle_conv_out_extent.restype = i64
            lib.oracle_conv_out_extent.argtypes = [i64, i64, i64, i64]
            lib.oracle_conv_direct.restype = ci
            lib.oracle_conv_direct.argtypes = [i64] * 9 + [vp, vp, vp, ci]
            lib.oracle_pack_b.restype = ci
            lib.oracle_pack_b.argtypes = [i64, i64, vp, i64, ci, vp, i64]
            lib.oracle_column_sums_s8.restype = ci
            lib.oracle_column_sums_s8.argtypes = [i64, i64, vp, i64, ci, vp]
            lib.oracle_im2col_u8.restype = ci
            lib.oracle_im2col_u8.argtypes = [i64] * 8 + [vp, vp, i64]
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


def gemm_s16(m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC, mode):
    """C (m x n, int32) = [C +] A (m x k) * B (k x n) with int16 operands, in place on the flat
    buffer ``C`` (the (i32, i16, i16) instruction forms of the paper's ISA table); sums wrap."""
    A = np.asarray(A)
    B = np.asarray(B)
    if A.dtype != np.int16 or B.dtype != np.int16 or C.dtype != np.int32:
        raise TypeError("operand dtypes do not match the entry point")
    for X in (A, B, C):
        if X.ndim != 1 or not X.flags.c_contiguous:
            raise ValueError("operands must be flat contiguous buffers")
    if not C.flags.writeable:
        raise ValueError("C must be writeable")
    if A.size < _min_len(m, k, lda, orderA) or B.size < _min_len(k, n, ldb, orderB) \
            or C.size < _min_len(m, n, ldc, orderC):
        raise ValueError("buffer shorter than the matrix it is said to hold")
    rc = _load().oracle_mip_gemm_s16(m, n, k, A.ctypes.data, lda, orderA, B.ctypes.data, ldb, orderB,
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


def gemm_requant(a_unsigned, b_unsigned, m, n, k, A, lda, orderA, B, ldb, orderB, scale,
                 Q, ldq, orderQ):
    """Q (m x n, int8) = clip(rint(scale * (A * B))), in place on the flat int8 buffer ``Q``
    (the quantization scheme of the paper's Section 7.3 applied to the output; the rounding
    decision is taken in float32).  ``scale`` is rounded to float32 first."""
    A = np.asarray(A)
    B = np.asarray(B)
    want_a = np.uint8 if a_unsigned else np.int8
    want_b = np.uint8 if b_unsigned else np.int8
    if A.dtype != want_a or B.dtype != want_b or Q.dtype != np.int8:
        raise TypeError("operand dtypes do not match the entry point")
    if not Q.flags.writeable or Q.ndim != 1 or not Q.flags.c_contiguous:
        raise ValueError("Q must be a flat, contiguous, writeable buffer")
    if A.size < _min_len(m, k, lda, orderA) or B.size < _min_len(k, n, ldb, orderB) \
            or Q.size < _min_len(m, n, ldq, orderQ):
        raise ValueError("buffer shorter than the matrix it is said to hold")
    rc = _load().oracle_mip_gemm_requant(
        int(bool(a_unsigned)), int(bool(b_unsigned)), m, n, k, A.ctypes.data, lda, orderA,
        B.ctypes.data, ldb, orderB, float(np.float32(scale)), Q.ctypes.data, ldq, orderQ)
    if rc != 0:
        raise ValueError("oracle rejected the arguments (rc=%d)" % rc)
    return Q


# ---------------------------------------------------------------------------
# convolution lowering (mip_conv_oracle.c; paper Section 7.2)
# ---------------------------------------------------------------------------

def conv_out_extent(extent, f, stride, pad):
    """h_o (or w_o) for an input extent, filter extent, stride and padding; -1 if the filter does not fit."""
    return int(_load().oracle_conv_out_extent(extent, f, stride, pad))


def conv_direct(I, F, stride, pad, O=None, mode=OVERWRITE):
    """O = CONV(F, I) from the definition.  I: uint8 (b, hi, wi, ci); F: int8 (co, hf, wf, ci);
    returns int32 (b, ho, wo, co); with mode ACCUMULATE adds into the given O."""
    I = np.ascontiguousarray(I)
    F = np.ascontiguousarray(F)
    if I.dtype != np.uint8 or F.dtype != np.int8 or I.ndim != 4 or F.ndim != 4:
        raise TypeError("I must be uint8 (b, hi, wi, ci) and F int8 (co, hf, wf, ci)")
    b, hi, wi, ci = I.shape
    co, hf, wf, ci2 = F.shape
    if ci2 != ci:
        raise ValueError("channel counts differ")
    ho, wo = conv_out_extent(hi, hf, stride, pad), conv_out_extent(wi, wf, stride, pad)
    if ho < 1 or wo < 1:
        raise ValueError("the filter does not fit the padded image")
    if O is None:
        if mode == ACCUMULATE:
            raise ValueError("accumulate needs an O to add into")
        O = np.empty((b, ho, wo, co), dtype=np.int32)
    if O.dtype != np.int32 or O.shape != (b, ho, wo, co) or not O.flags.c_contiguous:
        raise ValueError("O must be a contiguous int32 (b, ho, wo, co) array")
    rc = _load().oracle_conv_direct(b, hi, wi, ci, co, hf, wf, stride, pad,
                                    F.ctypes.data, I.ctypes.data, O.ctypes.data, mode)
    if rc != 0:
        raise ValueError("oracle rejected the arguments (rc=%d)" % rc)
    return O


def im2col_u8(I, hf, wf, stride, pad, ldm=None, fill=0x5A):
    """The augmented matrix of I for an hf x wf filter: uint8 (n, ldm) array whose first
    k = hf*wf*ci columns are the matrix (n = b*ho*wo rows); columns beyond k keep ``fill``."""
    I = np.ascontiguousarray(I)
    if I.dtype != np.uint8 or I.ndim != 4:
        raise TypeError("I must be uint8 (b, hi, wi, ci)")
    b, hi, wi, ci = I.shape
    ho, wo = conv_out_extent(hi, hf, stride, pad), conv_out_extent(wi, wf, stride, pad)
    if ho < 1 or wo < 1:
        raise ValueError("the filter does not fit the padded image")
    k = hf * wf * ci
    ldm = k if ldm is None else ldm
    M = np.full((b * ho * wo, ldm), fill, dtype=np.uint8)
    rc = _load().oracle_im2col_u8(b, hi, wi, ci, hf, wf, stride, pad, I.ctypes.data,
                                  M.ctypes.data, ldm)
    if rc != 0:
        raise ValueError("oracle rejected the arguments (rc=%d)" % rc)
    return M


def pack_b(k, n, B, ldb, orderB, ldp=None, fill=0x5A):
    """The k x n 8-bit matrix in the flat buffer ``B`` rewritten with k contiguous: uint8 (n, ldp)
    array whose row j holds column j of B in its first k bytes; bytes beyond keep ``fill``."""
    B = np.ascontiguousarray(B).view(np.uint8).reshape(-1)
    ldp = k if ldp is None else ldp
    if B.size < _min_len(k, n, ldb, orderB):
        raise ValueError("buffer shorter than the matrix it is said to hold")
    P = np.full((n, ldp), fill, dtype=np.uint8)
    rc = _load().oracle_pack_b(k, n, B.ctypes.data, ldb, orderB, P.ctypes.data, ldp)
    if rc != 0:
        raise ValueError("oracle rejected the arguments (rc=%d)" % rc)
    return P


def column_sums(k, n, B, ldb, orderB):
    """int32 array of n: the sum over k of every column of the signed k x n matrix in ``B``."""
    B = np.ascontiguousarray(B).view(np.int8).reshape(-1)
    if B.size < _min_len(k, n, ldb, orderB):
        raise ValueError("buffer shorter than the matrix it is said to hold")
    s = np.zeros(n, dtype=np.int32)
    rc = _load().oracle_column_sums_s8(k, n, B.ctypes.data, ldb, orderB, s.ctypes.data)
    if rc != 0:
        raise ValueError("oracle rejected the arguments (rc=%d)" % rc)
    return s


def packed_weights_layout(k, n):
    """(pitch of a column, columns held, byte offset of the k-sums, total bytes) of the packed
    form of a k x n weight matrix: columns k-contiguous, each padded with zeros to a whole
    number of k blocks (128 bytes from k = 1024 on, 64 below), the column count padded with
    zero columns to a multiple of 256, then one int32 k-sum per (real) column."""
    block = 128 if k >= 1024 else 64
    kp = max(block, -(-k // block) * block)
    cols = max(256, -(-n // 256) * 256)
    return kp, cols, kp * cols, kp * cols + 4 * n


def pack_weights(k, n, B, ldb, orderB):
    """The packed form of the signed k x n matrix in ``B`` as a flat uint8 array: oracle_pack_b
    into a zeroed buffer with the pitch above, followed by oracle_column_sums_s8."""
    kp, cols, at, total = packed_weights_layout(k, n)
    out = np.zeros(total, dtype=np.uint8)
    out[:n * kp] = pack_b(k, n, B, ldb, orderB, ldp=kp, fill=0).reshape(-1)
    out[at:] = column_sums(k, n, B, ldb, orderB).view(np.uint8)
    return out
