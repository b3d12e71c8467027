"""Thin ctypes binding of the C ABI declared in ``include/mipgemm.h``.

Argument marshalling only: every step of the GEMM runs in the HIP kernels of
``libmipgemm.so``.  Operands are device pointers: pass torch CUDA tensors (their
``data_ptr()`` is taken) or plain integer addresses.  PyTorch appears here only
as the owner of device memory and streams.

There is no fallback: if the shared library has not been built
(``python -m paper_2506_11728_amd.build``) loading raises.
"""
from __future__ import annotations

import ctypes
import os
import threading

ROW_MAJOR, COL_MAJOR = 0, 1
OVERWRITE, ACCUMULATE = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libmipgemm.so")
_lock = threading.Lock()
_lib = None

_GEMM_ARGTYPES = [ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                  ctypes.c_void_p, ctypes.c_int64, ctypes.c_int,
                  ctypes.c_void_p, ctypes.c_int64, ctypes.c_int,
                  ctypes.c_void_p, ctypes.c_int64, ctypes.c_int,
                  ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]


class MipGemmError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__("mipgemm error %d: %s" % (code, text))
        self.code = code


def library_path() -> str:
    return _LIB_PATH


def exported_symbols():
    """Names include/mipgemm.h declares; the library must export every one."""
    return ["mipgemm_s8s8s32", "mipgemm_u8s8s32", "mipgemm_s8u8s32",
            "mipgemm_s8s8f32", "mipgemm_u8s8f32", "mipgemm_s8u8f32",
            "mipgemm_workspace_size", "mipgemm_strerror", "mipgemm_variant_name",
            "mipgemm_mfma_ceiling", "mipgemm_conv_s8u8s32", "mipgemm_conv_workspace_size",
            "mipgemm_conv_variant_name", "mipgemm_im2col_u8", "mipgemm_conv_s8u8f32",
            "mipgemm_pack_b", "mipgemm_s8s8s32_batched", "mipgemm_u8s8s32_batched",
            "mipgemm_s8u8s32_batched", "mipgemm_variant_name_with_workspace",
            "mipgemm_variant_name_for_mode", "mipgemm_set_tuning",
            "mipgemm_conv_workspace_size_unaligned", "mipgemm_mfma_ceiling_clocked",
            "mipgemm_s8s8s32_clocked", "mipgemm_s8s8s32_noalloc", "mipgemm_static_scratch_bytes",
            "mipgemm_workspace_size_f32", "mipgemm_s8s8s8", "mipgemm_u8s8s8", "mipgemm_s8u8s8",
            "mipgemm_packed_weights_bytes", "mipgemm_pack_weights", "mipgemm_s8s8s32_packed",
            "mipgemm_u8s8s32_packed", "mipgemm_conv_filter_sums",
            "mipgemm_conv_s8u8s32_with_sums", "mipgemm_conv_s8u8f32_with_sums", "mipgemm_conv_s8u8s8",
            "mipgemm_s16s16s32", "mipgemm_workspace_size_s16"]


def load_library() -> ctypes.CDLL:
    global _lib
    with _lock:
        if _lib is None:
            if not os.path.exists(_LIB_PATH):
                raise ImportError(
                    "libmipgemm.so is not built (%s); run `python -m paper_2506_11728_amd.build`. "
                    "There is no CPU fallback." % _LIB_PATH)
            # PyTorch owns device memory and streams here and ships its own HIP runtime: it
            # must be the one in the process before the library binds to it (loaded the other
            # way round, the two runtimes disagree and launches fail with "no device")
            import torch  # noqa: F401
            lib = ctypes.CDLL(_LIB_PATH)
            for name in ("mipgemm_s8s8s32", "mipgemm_u8s8s32", "mipgemm_s8u8s32"):
                fn = getattr(lib, name)
                fn.restype = ctypes.c_int
                fn.argtypes = _GEMM_ARGTYPES
            for name in ("mipgemm_s8s8f32", "mipgemm_u8s8f32", "mipgemm_s8u8f32",
                         "mipgemm_s8s8s8", "mipgemm_u8s8s8", "mipgemm_s8u8s8"):
                fn = getattr(lib, name)
                fn.restype = ctypes.c_int
                fn.argtypes = _GEMM_ARGTYPES + [ctypes.c_float]
            lib.mipgemm_workspace_size.restype = ctypes.c_size_t
            lib.mipgemm_workspace_size.argtypes = [ctypes.c_int64] * 3 + [ctypes.c_int] * 3
            lib.mipgemm_workspace_size_f32.restype = ctypes.c_size_t
            lib.mipgemm_workspace_size_f32.argtypes = [ctypes.c_int64] * 3 + [ctypes.c_int] * 3
            lib.mipgemm_strerror.restype = ctypes.c_char_p
            lib.mipgemm_strerror.argtypes = [ctypes.c_int]
            for fn in (lib.mipgemm_variant_name, lib.mipgemm_variant_name_with_workspace):
                fn.restype = ctypes.c_char_p
                fn.argtypes = ([ctypes.c_int64] * 3 + [ctypes.c_int64, ctypes.c_int] * 3
                               + [ctypes.c_int] * 3)
            i64, vp = ctypes.c_int64, ctypes.c_void_p
            lib.mipgemm_conv_s8u8s32.restype = ctypes.c_int
            lib.mipgemm_conv_s8u8s32.argtypes = [i64] * 9 + [vp, vp, vp, ctypes.c_int, vp,
                                                             ctypes.c_size_t, vp]
            lib.mipgemm_conv_s8u8f32.restype = ctypes.c_int
            lib.mipgemm_conv_s8u8f32.argtypes = [i64] * 9 + [vp, vp, vp, ctypes.c_int, vp,
                                                             ctypes.c_size_t, vp, ctypes.c_float]
            lib.mipgemm_conv_filter_sums.restype = ctypes.c_int
            lib.mipgemm_conv_filter_sums.argtypes = [i64, i64, vp, vp, vp]
            lib.mipgemm_conv_s8u8s32_with_sums.restype = ctypes.c_int
            lib.mipgemm_conv_s8u8s32_with_sums.argtypes = [i64] * 9 + [vp, vp, vp, ctypes.c_int, vp,
                                                                       ctypes.c_size_t, vp, vp]
            lib.mipgemm_conv_s8u8f32_with_sums.restype = ctypes.c_int
            lib.mipgemm_conv_s8u8f32_with_sums.argtypes = [i64] * 9 + [vp, vp, vp, ctypes.c_int, vp,
                                                                       ctypes.c_size_t, vp, ctypes.c_float, vp]
            lib.mipgemm_conv_s8u8s8.restype = ctypes.c_int
            lib.mipgemm_conv_s8u8s8.argtypes = [i64] * 9 + [vp, vp, vp, ctypes.c_int, vp,
                                                            ctypes.c_size_t, vp, ctypes.c_float, vp]
            lib.mipgemm_conv_workspace_size.restype = ctypes.c_size_t
            lib.mipgemm_conv_workspace_size.argtypes = [i64] * 9
            lib.mipgemm_conv_workspace_size_unaligned.restype = ctypes.c_size_t
            lib.mipgemm_conv_workspace_size_unaligned.argtypes = [i64] * 9
            lib.mipgemm_variant_name_for_mode.restype = ctypes.c_char_p
            lib.mipgemm_variant_name_for_mode.argtypes = (
                [ctypes.c_int64] * 3 + [ctypes.c_int64, ctypes.c_int] * 3 + [ctypes.c_int] * 4)
            lib.mipgemm_set_tuning.restype = ctypes.c_int
            lib.mipgemm_set_tuning.argtypes = [ctypes.c_char_p, ctypes.c_char_p]
            lib.mipgemm_conv_variant_name.restype = ctypes.c_char_p
            lib.mipgemm_conv_variant_name.argtypes = [i64] * 9
            for fn in (lib.mipgemm_s8s8s32_batched, lib.mipgemm_u8s8s32_batched,
                       lib.mipgemm_s8u8s32_batched):
                fn.restype = ctypes.c_int
                fn.argtypes = ([i64] * 3 + [vp, i64, ctypes.c_int, i64] * 3
                               + [i64, ctypes.c_int, vp, ctypes.c_size_t, vp])
            lib.mipgemm_pack_b.restype = ctypes.c_int
            lib.mipgemm_pack_b.argtypes = [i64, i64, vp, i64, ctypes.c_int, vp, i64, vp]
            lib.mipgemm_s16s16s32.restype = ctypes.c_int
            lib.mipgemm_s16s16s32.argtypes = _GEMM_ARGTYPES
            lib.mipgemm_workspace_size_s16.restype = ctypes.c_size_t
            lib.mipgemm_workspace_size_s16.argtypes = [i64] * 3
            lib.mipgemm_packed_weights_bytes.restype = ctypes.c_size_t
            lib.mipgemm_packed_weights_bytes.argtypes = [i64, i64]
            lib.mipgemm_pack_weights.restype = ctypes.c_int
            lib.mipgemm_pack_weights.argtypes = [i64, i64, vp, i64, ctypes.c_int, vp, ctypes.c_size_t, vp]
            for fn in (lib.mipgemm_s8s8s32_packed, lib.mipgemm_u8s8s32_packed):
                fn.restype = ctypes.c_int
                fn.argtypes = ([i64] * 3 + [vp, i64, ctypes.c_int, vp, vp, i64, ctypes.c_int,
                                            ctypes.c_int, vp, ctypes.c_size_t, vp])
            lib.mipgemm_im2col_u8.restype = ctypes.c_int
            lib.mipgemm_im2col_u8.argtypes = [i64] * 8 + [vp, vp, i64, vp]
            lib.mipgemm_mfma_ceiling.restype = ctypes.c_int
            lib.mipgemm_mfma_ceiling.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_void_p,
                                                 ctypes.POINTER(ctypes.c_double)]
            lib.mipgemm_mfma_ceiling_clocked.restype = ctypes.c_int
            lib.mipgemm_mfma_ceiling_clocked.argtypes = [
                ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.POINTER(ctypes.c_double),
                ctypes.POINTER(ctypes.c_double)]
            lib.mipgemm_s8s8s32_clocked.restype = ctypes.c_int
            lib.mipgemm_s8s8s32_clocked.argtypes = _GEMM_ARGTYPES[:13] + [vp, vp, ctypes.c_size_t]
            lib.mipgemm_s8s8s32_noalloc.restype = ctypes.c_int
            lib.mipgemm_s8s8s32_noalloc.argtypes = _GEMM_ARGTYPES[:13] + [vp]
            lib.mipgemm_static_scratch_bytes.restype = ctypes.c_size_t
            lib.mipgemm_static_scratch_bytes.argtypes = []
            _lib = lib
    return _lib


def _ptr(x):
    if x is None:
        return None
    if isinstance(x, int):
        return x or None
    return x.data_ptr() or None          # torch tensor (device memory)


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None    # torch.cuda.Stream


def _call(name, m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC, mode,
          workspace, workspace_bytes, stream, check, *extra):
    rc = getattr(load_library(), name)(
        m, n, k, _ptr(A), lda, orderA, _ptr(B), ldb, orderB, _ptr(C), ldc, orderC, mode,
        _ptr(workspace), workspace_bytes, _stream(stream), *extra)
    if check and rc != 0:
        raise MipGemmError(rc, mipgemm_strerror(rc))
    return rc


def mipgemm_s8s8s32(m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC, mode,
                    workspace=None, workspace_bytes=0, stream=None, check=True):
    """C = [C +] A * B, int8 x int8 -> int32 (see include/mipgemm.h)."""
    return _call("mipgemm_s8s8s32", m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC,
                 mode, workspace, workspace_bytes, stream, check)


def mipgemm_u8s8s32(m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC, mode,
                    workspace=None, workspace_bytes=0, stream=None, check=True):
    """Same with an unsigned A."""
    return _call("mipgemm_u8s8s32", m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC,
                 mode, workspace, workspace_bytes, stream, check)


def mipgemm_s8u8s32(m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC, mode,
                    workspace=None, workspace_bytes=0, stream=None, check=True):
    """Same with an unsigned B."""
    return _call("mipgemm_s8u8s32", m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC,
                 mode, workspace, workspace_bytes, stream, check)


def mipgemm_s8s8f32(m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC, mode,
                    workspace=None, workspace_bytes=0, stream=None, scale=1.0, check=True):
    """C (float) = [C +] scale * (A * B): the integer GEMM with the dequantising scale fused in."""
    return _call("mipgemm_s8s8f32", m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC,
                 mode, workspace, workspace_bytes, stream, check, scale)


def mipgemm_u8s8f32(m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC, mode,
                    workspace=None, workspace_bytes=0, stream=None, scale=1.0, check=True):
    """Same with an unsigned A."""
    return _call("mipgemm_u8s8f32", m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC,
                 mode, workspace, workspace_bytes, stream, check, scale)


def mipgemm_s8u8f32(m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC, mode,
                    workspace=None, workspace_bytes=0, stream=None, scale=1.0, check=True):
    """Same with an unsigned B."""
    return _call("mipgemm_s8u8f32", m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC,
                 mode, workspace, workspace_bytes, stream, check, scale)


def mipgemm_s8s8s8(m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC, mode,
                   workspace=None, workspace_bytes=0, stream=None, scale=1.0, check=True):
    """C (int8) = clip(rint(scale * (A * B))): the integer GEMM with the requantising scale fused in."""
    return _call("mipgemm_s8s8s8", m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC,
                 mode, workspace, workspace_bytes, stream, check, scale)


def mipgemm_u8s8s8(m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC, mode,
                   workspace=None, workspace_bytes=0, stream=None, scale=1.0, check=True):
    """Same with an unsigned A."""
    return _call("mipgemm_u8s8s8", m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC,
                 mode, workspace, workspace_bytes, stream, check, scale)


def mipgemm_s8u8s8(m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC, mode,
                   workspace=None, workspace_bytes=0, stream=None, scale=1.0, check=True):
    """Same with an unsigned B."""
    return _call("mipgemm_s8u8s8", m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC,
                 mode, workspace, workspace_bytes, stream, check, scale)


def mipgemm_conv_s8u8s32(b, hi, wi, ci, co, hf, wf, stride, pad, F, I, O, mode,
                         workspace=None, workspace_bytes=0, stream=None, check=True):
    """O = [O +] CONV(F, I) by lowering to the integer GEMM (see include/mipgemm.h)."""
    rc = load_library().mipgemm_conv_s8u8s32(
        b, hi, wi, ci, co, hf, wf, stride, pad, _ptr(F), _ptr(I), _ptr(O), mode,
        _ptr(workspace), workspace_bytes, _stream(stream))
    if check and rc != 0:
        raise MipGemmError(rc, mipgemm_strerror(rc))
    return rc


def mipgemm_conv_s8u8f32(b, hi, wi, ci, co, hf, wf, stride, pad, F, I, O, mode,
                         workspace=None, workspace_bytes=0, stream=None, scale=1.0, check=True):
    """O (float) = [O +] scale * CONV(F, I): the lowered convolution with the scale fused in."""
    rc = load_library().mipgemm_conv_s8u8f32(
        b, hi, wi, ci, co, hf, wf, stride, pad, _ptr(F), _ptr(I), _ptr(O), mode,
        _ptr(workspace), workspace_bytes, _stream(stream), scale)
    if check and rc != 0:
        raise MipGemmError(rc, mipgemm_strerror(rc))
    return rc


def mipgemm_conv_filter_sums(co, k, F, sums, stream=None, check=True):
    """sums[o] = the sum over k of filter o (F: c_o filters of k = h_f w_f c_i signed bytes each)."""
    rc = load_library().mipgemm_conv_filter_sums(co, k, _ptr(F), _ptr(sums), _stream(stream))
    if check and rc != 0:
        raise MipGemmError(rc, mipgemm_strerror(rc))
    return rc


def mipgemm_conv_s8u8s32_with_sums(b, hi, wi, ci, co, hf, wf, stride, pad, F, I, O, mode, filter_sums,
                                   workspace=None, workspace_bytes=0, stream=None, check=True):
    """mipgemm_conv_s8u8s32 with the filters' k-sums (mipgemm_conv_filter_sums) supplied."""
    rc = load_library().mipgemm_conv_s8u8s32_with_sums(
        b, hi, wi, ci, co, hf, wf, stride, pad, _ptr(F), _ptr(I), _ptr(O), mode,
        _ptr(workspace), workspace_bytes, _stream(stream), _ptr(filter_sums))
    if check and rc != 0:
        raise MipGemmError(rc, mipgemm_strerror(rc))
    return rc


def mipgemm_conv_s8u8f32_with_sums(b, hi, wi, ci, co, hf, wf, stride, pad, F, I, O, mode, filter_sums,
                                   workspace=None, workspace_bytes=0, stream=None, scale=1.0, check=True):
    """mipgemm_conv_s8u8f32 with the filters' k-sums supplied."""
    rc = load_library().mipgemm_conv_s8u8f32_with_sums(
        b, hi, wi, ci, co, hf, wf, stride, pad, _ptr(F), _ptr(I), _ptr(O), mode,
        _ptr(workspace), workspace_bytes, _stream(stream), scale, _ptr(filter_sums))
    if check and rc != 0:
        raise MipGemmError(rc, mipgemm_strerror(rc))
    return rc


def mipgemm_conv_s8u8s8(b, hi, wi, ci, co, hf, wf, stride, pad, F, I, O, mode, filter_sums=None,
                        workspace=None, workspace_bytes=0, stream=None, scale=1.0, check=True):
    """O (int8) = clip(rint(scale * CONV(F, I))): the lowered convolution requantised for the next layer."""
    rc = load_library().mipgemm_conv_s8u8s8(
        b, hi, wi, ci, co, hf, wf, stride, pad, _ptr(F), _ptr(I), _ptr(O), mode,
        _ptr(workspace), workspace_bytes, _stream(stream), scale, _ptr(filter_sums))
    if check and rc != 0:
        raise MipGemmError(rc, mipgemm_strerror(rc))
    return rc


def mipgemm_conv_workspace_size(b, hi, wi, ci, co, hf, wf, stride, pad) -> int:
    return int(load_library().mipgemm_conv_workspace_size(b, hi, wi, ci, co, hf, wf, stride, pad))


def mipgemm_conv_workspace_size_unaligned(b, hi, wi, ci, co, hf, wf, stride, pad) -> int:
    return int(load_library().mipgemm_conv_workspace_size_unaligned(b, hi, wi, ci, co, hf, wf,
                                                                    stride, pad))


def mipgemm_conv_variant_name(b, hi, wi, ci, co, hf, wf, stride, pad) -> str:
    return load_library().mipgemm_conv_variant_name(b, hi, wi, ci, co, hf, wf, stride,
                                                    pad).decode()


def mipgemm_im2col_u8(b, hi, wi, ci, hf, wf, stride, pad, I, M, ldm, stream=None, check=True):
    """The augmented matrix of the lowering alone: one row of hf*wf*ci bytes per output position."""
    rc = load_library().mipgemm_im2col_u8(b, hi, wi, ci, hf, wf, stride, pad, _ptr(I), _ptr(M),
                                          ldm, _stream(stream))
    if check and rc != 0:
        raise MipGemmError(rc, mipgemm_strerror(rc))
    return rc


def _batched(entry, m, n, k, A, lda, orderA, strideA, B, ldb, orderB, strideB,
             C, ldc, orderC, strideC, batch, mode, workspace, workspace_bytes, stream, check):
    rc = getattr(load_library(), entry)(
        m, n, k, _ptr(A), lda, orderA, strideA, _ptr(B), ldb, orderB, strideB,
        _ptr(C), ldc, orderC, strideC, batch, mode, _ptr(workspace), workspace_bytes,
        _stream(stream))
    if check and rc != 0:
        raise MipGemmError(rc, mipgemm_strerror(rc))
    return rc


def mipgemm_s8s8s32_batched(m, n, k, A, lda, orderA, strideA, B, ldb, orderB, strideB,
                            C, ldc, orderC, strideC, batch, mode,
                            workspace=None, workspace_bytes=0, stream=None, check=True):
    """`batch` independent GEMMs of one shape, problem z at A + z*strideA, B + z*strideB, C + z*strideC."""
    return _batched("mipgemm_s8s8s32_batched", m, n, k, A, lda, orderA, strideA, B, ldb, orderB,
                    strideB, C, ldc, orderC, strideC, batch, mode, workspace, workspace_bytes,
                    stream, check)


def mipgemm_u8s8s32_batched(m, n, k, A, lda, orderA, strideA, B, ldb, orderB, strideB,
                            C, ldc, orderC, strideC, batch, mode,
                            workspace=None, workspace_bytes=0, stream=None, check=True):
    """The strided batch with A unsigned."""
    return _batched("mipgemm_u8s8s32_batched", m, n, k, A, lda, orderA, strideA, B, ldb, orderB,
                    strideB, C, ldc, orderC, strideC, batch, mode, workspace, workspace_bytes,
                    stream, check)


def mipgemm_s8u8s32_batched(m, n, k, A, lda, orderA, strideA, B, ldb, orderB, strideB,
                            C, ldc, orderC, strideC, batch, mode,
                            workspace=None, workspace_bytes=0, stream=None, check=True):
    """The strided batch with B unsigned."""
    return _batched("mipgemm_s8u8s32_batched", m, n, k, A, lda, orderA, strideA, B, ldb, orderB,
                    strideB, C, ldc, orderC, strideC, batch, mode, workspace, workspace_bytes,
                    stream, check)


def mipgemm_pack_b(k, n, B, ldb, orderB, P, ldp, stream=None, check=True):
    """The k x n matrix B rewritten with k contiguous (pass P as B with COL_MAJOR, ldb = ldp)."""
    rc = load_library().mipgemm_pack_b(k, n, _ptr(B), ldb, orderB, _ptr(P), ldp, _stream(stream))
    if check and rc != 0:
        raise MipGemmError(rc, mipgemm_strerror(rc))
    return rc


def mipgemm_workspace_size_s16(m, n, k) -> int:
    return int(load_library().mipgemm_workspace_size_s16(m, n, k))


def mipgemm_s16s16s32(m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC, mode,
                      workspace=None, workspace_bytes=0, stream=None, check=True):
    """C = [C +] A * B with int16 operands, through byte planes on the 8-bit kernels; needs a
    workspace of mipgemm_workspace_size_s16(m, n, k) bytes."""
    return _call("mipgemm_s16s16s32", m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC,
                 mode, workspace, workspace_bytes, stream, check)


def mipgemm_packed_weights_bytes(k, n) -> int:
    return int(load_library().mipgemm_packed_weights_bytes(k, n))


def mipgemm_pack_weights(k, n, B, ldb, orderB, packed, packed_bytes=None, stream=None, check=True):
    """The signed k x n matrix B as a packed-weights object in ``packed`` (a device buffer of
    mipgemm_packed_weights_bytes(k, n) bytes): columns k-contiguous and zero-padded, then the k-sums."""
    if packed_bytes is None:
        packed_bytes = packed.numel() * packed.element_size()
    rc = load_library().mipgemm_pack_weights(k, n, _ptr(B), ldb, orderB, _ptr(packed), packed_bytes,
                                             _stream(stream))
    if check and rc != 0:
        raise MipGemmError(rc, mipgemm_strerror(rc))
    return rc


def _call_packed(name, m, n, k, A, lda, orderA, packed, C, ldc, orderC, mode, workspace,
                 workspace_bytes, stream, check):
    rc = getattr(load_library(), name)(m, n, k, _ptr(A), lda, orderA, _ptr(packed), _ptr(C), ldc,
                                       orderC, mode, _ptr(workspace), workspace_bytes, _stream(stream))
    if check and rc != 0:
        raise MipGemmError(rc, mipgemm_strerror(rc))
    return rc


def mipgemm_s8s8s32_packed(m, n, k, A, lda, orderA, packed, C, ldc, orderC, mode,
                           workspace=None, workspace_bytes=0, stream=None, check=True):
    """mipgemm_s8s8s32 with B given as packed weights."""
    return _call_packed("mipgemm_s8s8s32_packed", m, n, k, A, lda, orderA, packed, C, ldc, orderC,
                        mode, workspace, workspace_bytes, stream, check)


def mipgemm_u8s8s32_packed(m, n, k, A, lda, orderA, packed, C, ldc, orderC, mode,
                           workspace=None, workspace_bytes=0, stream=None, check=True):
    """mipgemm_u8s8s32 with B given as packed weights, which bring their k-sums."""
    return _call_packed("mipgemm_u8s8s32_packed", m, n, k, A, lda, orderA, packed, C, ldc, orderC,
                        mode, workspace, workspace_bytes, stream, check)


def mipgemm_workspace_size(m, n, k, orderA, orderB, orderC) -> int:
    return int(load_library().mipgemm_workspace_size(m, n, k, orderA, orderB, orderC))


def mipgemm_workspace_size_f32(m, n, k, orderA, orderB, orderC) -> int:
    return int(load_library().mipgemm_workspace_size_f32(m, n, k, orderA, orderB, orderC))


def mipgemm_strerror(code: int) -> str:
    return load_library().mipgemm_strerror(code).decode()


def mipgemm_variant_name(m, n, k, lda, orderA, ldb, orderB, ldc, orderC,
                         a_unsigned=False, b_unsigned=False, aligned16=True) -> str:
    return load_library().mipgemm_variant_name(
        m, n, k, lda, orderA, ldb, orderB, ldc, orderC,
        int(a_unsigned), int(b_unsigned), int(aligned16)).decode()


def mipgemm_variant_name_for_mode(m, n, k, lda, orderA, ldb, orderB, ldc, orderC,
                                  a_unsigned=False, b_unsigned=False, aligned16=True,
                                  mode=OVERWRITE) -> str:
    return load_library().mipgemm_variant_name_for_mode(
        m, n, k, lda, orderA, ldb, orderB, ldc, orderC,
        int(a_unsigned), int(b_unsigned), int(aligned16), int(mode)).decode()


def mipgemm_set_tuning(name: str, value) -> None:
    """Sets one of the dispatcher's tuning values (MIPGEMM_VARIANT, MIPGEMM_SPLITK, MIPGEMM_PACK,
    MIPGEMM_CONV, MIPGEMM_STAGGER) for the whole process; None or "" clears it."""
    rc = load_library().mipgemm_set_tuning(name.encode(), None if value is None else str(value).encode())
    if rc != 0:
        raise ValueError("mipgemm_set_tuning(%r, %r) rejected" % (name, value))


class tuning:
    """Context manager: the given tuning values inside, cleared again afterwards.

    tuning(MIPGEMM_VARIANT="dma64", MIPGEMM_SPLITK=4); None leaves a value cleared."""

    def __init__(self, **values):
        self.values = values

    def __enter__(self):
        for k, v in self.values.items():
            mipgemm_set_tuning(k, v)
        return self

    def __exit__(self, *exc):
        for k in self.values:
            mipgemm_set_tuning(k, None)
        return False


def mipgemm_variant_name_with_workspace(m, n, k, lda, orderA, ldb, orderB, ldc, orderC,
                                        a_unsigned=False, b_unsigned=False, aligned16=True) -> str:
    return load_library().mipgemm_variant_name_with_workspace(
        m, n, k, lda, orderA, ldb, orderB, ldc, orderC,
        int(a_unsigned), int(b_unsigned), int(aligned16)).decode()


def mipgemm_mfma_ceiling(pattern: int, iterations: int = 20000, stream=None) -> float:
    """TOPS of the register-resident int8 MFMA loop (0: near-zero operands, 1: random operands)."""
    out = ctypes.c_double(0.0)
    rc = load_library().mipgemm_mfma_ceiling(pattern, iterations, _stream(stream), ctypes.byref(out))
    if rc != 0:
        raise MipGemmError(rc, mipgemm_strerror(rc) if rc > 0 else "invalid argument %d" % -rc)
    return out.value


def mipgemm_mfma_ceiling_clocked(pattern: int, iterations: int = 20000, stream=None):
    """(TOPS, shader MHz) of the register-resident int8 MFMA loop; patterns 0..5 as in the header."""
    tops, mhz = ctypes.c_double(0.0), ctypes.c_double(0.0)
    rc = load_library().mipgemm_mfma_ceiling_clocked(pattern, iterations, _stream(stream),
                                                     ctypes.byref(tops), ctypes.byref(mhz))
    if rc != 0:
        raise MipGemmError(rc, mipgemm_strerror(rc) if rc > 0 else "invalid argument %d" % -rc)
    return tops.value, mhz.value


def mipgemm_s8s8s32_clocked(m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC, mode,
                            clocks, clocks_bytes, stream=None, check=True):
    """mipgemm_s8s8s32 on the large-problem kernel with per-workgroup clock counters (benchmarks)."""
    rc = load_library().mipgemm_s8s8s32_clocked(
        m, n, k, _ptr(A), lda, orderA, _ptr(B), ldb, orderB, _ptr(C), ldc, orderC, mode,
        _stream(stream), _ptr(clocks), clocks_bytes)
    if check and rc != 0:
        raise MipGemmError(rc, mipgemm_strerror(rc))
    return rc


ERR_STATIC_SCRATCH = -100


def mipgemm_s8s8s32_noalloc(m, n, k, A, lda, orderA, B, ldb, orderB, C, ldc, orderC, mode,
                            stream=None, check=True):
    """mipgemm_s8s8s32 with the packed route's buffers in the library's static device array."""
    rc = load_library().mipgemm_s8s8s32_noalloc(
        m, n, k, _ptr(A), lda, orderA, _ptr(B), ldb, orderB, _ptr(C), ldc, orderC, mode,
        _stream(stream))
    if check and rc != 0:
        raise MipGemmError(rc, mipgemm_strerror(rc))
    return rc


def mipgemm_static_scratch_bytes() -> int:
    return int(load_library().mipgemm_static_scratch_bytes())
