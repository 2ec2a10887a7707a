"""ctypes binding of libfsrgemm.so: the same entry points as include/fsrgemm.h.

Only argument marshalling happens here.  Pointers may be given as integers
(device addresses) or as objects with a ``data_ptr()`` method (torch tensors);
``stream`` is a hipStream_t handle as an integer (0 = default stream).
There is no fallback: if the library has not been built, every call raises.
"""
from __future__ import annotations

import ctypes
import os

__all__ = [
    "load", "library_path", "gemm_f32", "gemm_f32_ex", "gemm_bf16", "fsrgemm_kernel_for_f32",
    "fsrgemm_kernel_for_f32_ex", "fsrgemm_kernel_for_bf16", "gemm_bf16_ex", "fsrgemm_kernel_for_bf16_ex",
    "gemm_f32_ws", "gemm_f32_noalloc", "gemm_f32_workspace_bytes", "gemm_bf16_ws", "gemm_bf16_workspace_bytes", "transpose_f32",
    "fsrgemm_kernel_for_transpose_f32", "gemm_f32_cfg", "gemm_bf16_cfg", "fsrgemm_tile_count_f32",
    "fsrgemm_tile_count_bf16", "fsrgemm_plan_f32", "fsrgemm_plan_bf16", "fsrgemm_bands_f32", "fsrgemm_bands_bf16", "fsrgemm_kernel_for_f32_cfg",
    "fsrgemm_kernel_for_bf16_cfg", "fsrgemm_mfma_ceiling", "fsrgemm_kernel_for_mfma_ceiling",
    "fsrgemm_status_string", "fsrgemm_version", "check", "FsrGemmError", "EXPORTS",
    "FSRGEMM_PLAN_WORKSPACE", "FSRGEMM_PLAN_RULES_ONLY", "FSRGEMM_OK", "FSRGEMM_ERR_INVALID_ARG", "FSRGEMM_ERR_LAUNCH", "FSRGEMM_ERR_UNSUPPORTED_DEVICE",
    "FSRGEMM_ERR_SCRATCH_LIMIT", "FSRGEMM_NOALLOC_SCRATCH_BYTES",
]

FSRGEMM_OK = 0
FSRGEMM_ERR_INVALID_ARG = -1
FSRGEMM_ERR_LAUNCH = -2
FSRGEMM_ERR_UNSUPPORTED_DEVICE = -3
FSRGEMM_ERR_SCRATCH_LIMIT = -4
FSRGEMM_NOALLOC_SCRATCH_BYTES = 16 * 1024 * 1024
FSRGEMM_PLAN_WORKSPACE = 1
FSRGEMM_PLAN_RULES_ONLY = 2

_i64, _vp = ctypes.c_int64, ctypes.c_void_p
_GEMM = [_i64, _i64, _i64, _vp, _i64, _vp, _i64, _vp, _i64, _vp]
_QUERY = [_i64, _i64, _i64, _vp, _i64, _vp, _i64, _vp, _i64]
# every symbol include/fsrgemm.h declares: name -> (restype, argtypes)
EXPORTS = {
    "gemm_f32": (ctypes.c_int, _GEMM),
    "gemm_f32_ex": (ctypes.c_int, [ctypes.c_int, ctypes.c_int] + _GEMM),
    "gemm_f32_noalloc": (ctypes.c_int, [ctypes.c_int, ctypes.c_int] + _GEMM),
    "gemm_f32_workspace_bytes": (_i64, [ctypes.c_int, ctypes.c_int, _i64, _i64, _i64]),
    "gemm_f32_ws": (ctypes.c_int, [ctypes.c_int, ctypes.c_int] + _GEMM[:-1] + [_vp, _i64, _vp]),
    "gemm_bf16_workspace_bytes": (_i64, [ctypes.c_int, ctypes.c_int, _i64, _i64, _i64]),
    "gemm_bf16_ws": (ctypes.c_int, [ctypes.c_int, ctypes.c_int] + _GEMM[:-1] + [_vp, _i64, _vp]),
    "gemm_bf16": (ctypes.c_int, _GEMM),
    "gemm_bf16_ex": (ctypes.c_int, [ctypes.c_int, ctypes.c_int] + _GEMM),
    "fsrgemm_kernel_for_f32": (ctypes.c_char_p, _QUERY),
    "fsrgemm_kernel_for_f32_ex": (ctypes.c_char_p, [ctypes.c_int, ctypes.c_int] + _QUERY),
    "fsrgemm_kernel_for_bf16": (ctypes.c_char_p, _QUERY),
    "fsrgemm_kernel_for_bf16_ex": (ctypes.c_char_p, [ctypes.c_int, ctypes.c_int] + _QUERY),
    "transpose_f32": (ctypes.c_int, [_i64, _i64, _vp, _i64, _vp, _i64, _vp]),
    "fsrgemm_kernel_for_transpose_f32": (ctypes.c_char_p, [_i64, _i64, _vp, _i64, _vp, _i64]),
    "gemm_f32_cfg": (ctypes.c_int, [ctypes.c_int] * 4 + _GEMM[:-1] + [_vp, _i64, _vp]),
    "gemm_bf16_cfg": (ctypes.c_int, [ctypes.c_int] * 4 + _GEMM[:-1] + [_vp, _i64, _vp]),
    "fsrgemm_kernel_for_f32_cfg": (ctypes.c_char_p, [ctypes.c_int] * 3 + _QUERY),
    "fsrgemm_kernel_for_bf16_cfg": (ctypes.c_char_p, [ctypes.c_int] * 3 + _QUERY),
    "fsrgemm_tile_count_f32": (ctypes.c_int, []),
    "fsrgemm_tile_count_bf16": (ctypes.c_int, []),
    "fsrgemm_plan_f32": (ctypes.c_int, [ctypes.c_int, ctypes.c_int, _i64, _i64, _i64, _vp, _i64, _vp, _i64, ctypes.c_int,
                                        ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int)]),
    "fsrgemm_plan_bf16": (ctypes.c_int, [ctypes.c_int, ctypes.c_int, _i64, _i64, _i64, _vp, _i64, _vp, _i64, ctypes.c_int,
                                         ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int)]),
    "fsrgemm_bands_f32": (ctypes.c_int, [ctypes.c_int, ctypes.c_int, _i64, _i64, _i64, _vp, _i64, _vp, _i64, ctypes.c_int,
                                         ctypes.POINTER(ctypes.c_int), ctypes.POINTER(_i64), ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int)]),
    "fsrgemm_bands_bf16": (ctypes.c_int, [ctypes.c_int, ctypes.c_int, _i64, _i64, _i64, _vp, _i64, _vp, _i64, ctypes.c_int,
                                          ctypes.POINTER(ctypes.c_int), ctypes.POINTER(_i64), ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int)]),
    "fsrgemm_mfma_ceiling": (ctypes.c_int, [ctypes.c_int, ctypes.c_int, _vp, _vp, ctypes.c_int, ctypes.POINTER(ctypes.c_double), _vp]),
    "fsrgemm_kernel_for_mfma_ceiling": (ctypes.c_char_p, [ctypes.c_int]),
    "fsrgemm_status_string": (ctypes.c_char_p, [ctypes.c_int]),
    "fsrgemm_version": (ctypes.c_int, []),
}

_lib = None


class FsrGemmError(RuntimeError):
    pass


def library_path() -> str:
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "libfsrgemm.so")


def load():
    """Load libfsrgemm.so (once).  Raises FsrGemmError if it has not been built."""
    global _lib
    if _lib is None:
        path = library_path()
        if not os.path.exists(path):
            raise FsrGemmError(
                "%s is missing: build it first (python -m paper_2506_09092_amd.build); there is no fallback path" % path)
        try:
            # torch carries its own HIP runtime; import it first so that the library binds to the
            # runtime that owns the caller's tensors and streams instead of loading a second one
            import torch  # noqa: F401
        except ImportError:
            pass
        lib = ctypes.CDLL(path)
        for name, (res, args) in EXPORTS.items():
            fn = getattr(lib, name)
            fn.restype, fn.argtypes = res, args
        _lib = lib
    return _lib


def _ptr(x):
    if x is None:
        return None
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    return int(x)


def gemm_f32(M, N, K, A, lda, B, ldb, C, ldc, stream=0) -> int:
    return load().gemm_f32(M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(C), ldc, _ptr(stream) or None)


def gemm_f32_ex(transA, transB, M, N, K, A, lda, B, ldb, C, ldc, stream=0) -> int:
    return load().gemm_f32_ex(int(transA), int(transB), M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(C), ldc,
                              _ptr(stream) or None)


def gemm_f32_noalloc(transA, transB, M, N, K, A, lda, B, ldb, C, ldc, stream=0) -> int:
    return load().gemm_f32_noalloc(int(transA), int(transB), M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(C), ldc,
                                   _ptr(stream) or None)


def gemm_f32_workspace_bytes(transA, transB, M, N, K) -> int:
    return int(load().gemm_f32_workspace_bytes(int(transA), int(transB), M, N, K))


def gemm_f32_ws(transA, transB, M, N, K, A, lda, B, ldb, C, ldc, workspace, workspace_bytes, stream=0) -> int:
    return load().gemm_f32_ws(int(transA), int(transB), M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(C), ldc,
                              _ptr(workspace), int(workspace_bytes), _ptr(stream) or None)


def gemm_bf16_workspace_bytes(transA, transB, M, N, K) -> int:
    return int(load().gemm_bf16_workspace_bytes(int(transA), int(transB), M, N, K))


def gemm_bf16_ws(transA, transB, M, N, K, A, lda, B, ldb, C, ldc, workspace, workspace_bytes, stream=0) -> int:
    return load().gemm_bf16_ws(int(transA), int(transB), M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(C), ldc,
                               _ptr(workspace), int(workspace_bytes), _ptr(stream) or None)


def gemm_bf16(M, N, K, A, lda, B, ldb, C, ldc, stream=0) -> int:
    return load().gemm_bf16(M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(C), ldc, _ptr(stream) or None)


def gemm_bf16_ex(transA, transB, M, N, K, A, lda, B, ldb, C, ldc, stream=0) -> int:
    return load().gemm_bf16_ex(int(transA), int(transB), M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(C), ldc,
                               _ptr(stream) or None)


def gemm_f32_cfg(tile, k_slices, transA, transB, M, N, K, A, lda, B, ldb, C, ldc, workspace=0, workspace_bytes=0, stream=0) -> int:
    return load().gemm_f32_cfg(int(tile), int(k_slices), int(transA), int(transB), M, N, K, _ptr(A), lda, _ptr(B), ldb,
                               _ptr(C), ldc, _ptr(workspace), int(workspace_bytes), _ptr(stream) or None)


def gemm_bf16_cfg(tile, k_slices, transA, transB, M, N, K, A, lda, B, ldb, C, ldc, workspace=0, workspace_bytes=0, stream=0) -> int:
    return load().gemm_bf16_cfg(int(tile), int(k_slices), int(transA), int(transB), M, N, K, _ptr(A), lda, _ptr(B), ldb,
                                _ptr(C), ldc, _ptr(workspace), int(workspace_bytes), _ptr(stream) or None)


def fsrgemm_kernel_for_f32_cfg(tile, transA, transB, M, N, K, A, lda, B, ldb, C, ldc):
    r = load().fsrgemm_kernel_for_f32_cfg(int(tile), int(transA), int(transB), M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(C), ldc)
    return None if r is None else r.decode()


def fsrgemm_kernel_for_bf16_cfg(tile, transA, transB, M, N, K, A, lda, B, ldb, C, ldc):
    r = load().fsrgemm_kernel_for_bf16_cfg(int(tile), int(transA), int(transB), M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(C), ldc)
    return None if r is None else r.decode()


def fsrgemm_tile_count_f32() -> int:
    return int(load().fsrgemm_tile_count_f32())


def fsrgemm_tile_count_bf16() -> int:
    return int(load().fsrgemm_tile_count_bf16())


def _plan(fn, transA, transB, M, N, K, A, lda, B, ldb, with_workspace, rules_only):
    tile, slices = ctypes.c_int(-1), ctypes.c_int(-1)
    flags = (FSRGEMM_PLAN_WORKSPACE if with_workspace else 0) | (FSRGEMM_PLAN_RULES_ONLY if rules_only else 0)
    rc = fn(int(transA), int(transB), M, N, K, _ptr(A), lda, _ptr(B), ldb, flags, ctypes.byref(tile), ctypes.byref(slices))
    return None if rc != FSRGEMM_OK else (tile.value, slices.value)


def fsrgemm_plan_f32(transA, transB, M, N, K, A, lda, B, ldb, with_workspace=False, rules_only=False):
    """(tile, k_slices) the dispatcher would take, or None for invalid arguments."""
    return _plan(load().fsrgemm_plan_f32, transA, transB, M, N, K, A, lda, B, ldb, with_workspace, rules_only)


def fsrgemm_plan_bf16(transA, transB, M, N, K, A, lda, B, ldb, with_workspace=False, rules_only=False):
    return _plan(load().fsrgemm_plan_bf16, transA, transB, M, N, K, A, lda, B, ldb, with_workspace, rules_only)


def _bands(fn, transA, transB, M, N, K, A, lda, B, ldb, with_workspace, rules_only):
    dim, at, first, second = ctypes.c_int(-1), _i64(-1), ctypes.c_int(-1), ctypes.c_int(-1)
    flags = (FSRGEMM_PLAN_WORKSPACE if with_workspace else 0) | (FSRGEMM_PLAN_RULES_ONLY if rules_only else 0)
    rc = fn(int(transA), int(transB), M, N, K, _ptr(A), lda, _ptr(B), ldb, flags, ctypes.byref(dim), ctypes.byref(at),
            ctypes.byref(first), ctypes.byref(second))
    return None if rc != FSRGEMM_OK else (dim.value, at.value, first.value, second.value)


def fsrgemm_bands_f32(transA, transB, M, N, K, A, lda, B, ldb, with_workspace=False, rules_only=False):
    """(dim, at, tile_first, tile_second): dim 0 = one launch, 1 = cut along the rows of C at `at`, 2 = along its columns."""
    return _bands(load().fsrgemm_bands_f32, transA, transB, M, N, K, A, lda, B, ldb, with_workspace, rules_only)


def fsrgemm_bands_bf16(transA, transB, M, N, K, A, lda, B, ldb, with_workspace=False, rules_only=False):
    return _bands(load().fsrgemm_bands_bf16, transA, transB, M, N, K, A, lda, B, ldb, with_workspace, rules_only)


def fsrgemm_kernel_for_f32(M, N, K, A, lda, B, ldb, C, ldc):
    r = load().fsrgemm_kernel_for_f32(M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(C), ldc)
    return None if r is None else r.decode()


def fsrgemm_kernel_for_f32_ex(transA, transB, M, N, K, A, lda, B, ldb, C, ldc):
    r = load().fsrgemm_kernel_for_f32_ex(int(transA), int(transB), M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(C), ldc)
    return None if r is None else r.decode()


def fsrgemm_kernel_for_bf16(M, N, K, A, lda, B, ldb, C, ldc):
    r = load().fsrgemm_kernel_for_bf16(M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(C), ldc)
    return None if r is None else r.decode()


def fsrgemm_kernel_for_bf16_ex(transA, transB, M, N, K, A, lda, B, ldb, C, ldc):
    r = load().fsrgemm_kernel_for_bf16_ex(int(transA), int(transB), M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(C), ldc)
    return None if r is None else r.decode()


def transpose_f32(rows, cols, A, lda, T, ldt, stream=0) -> int:
    return load().transpose_f32(rows, cols, _ptr(A), lda, _ptr(T), ldt, _ptr(stream) or None)


def fsrgemm_kernel_for_transpose_f32(rows, cols, A, lda, T, ldt):
    r = load().fsrgemm_kernel_for_transpose_f32(rows, cols, _ptr(A), lda, _ptr(T), ldt)
    return None if r is None else r.decode()


def fsrgemm_mfma_ceiling(kind, passes, operands, sink, workgroups, stream=0):
    """(status, flop of the launch)."""
    flop = ctypes.c_double(0.0)
    rc = load().fsrgemm_mfma_ceiling(int(kind), int(passes), _ptr(operands), _ptr(sink), int(workgroups), ctypes.byref(flop),
                                     _ptr(stream) or None)
    return rc, flop.value


def fsrgemm_kernel_for_mfma_ceiling(kind):
    r = load().fsrgemm_kernel_for_mfma_ceiling(int(kind))
    return None if r is None else r.decode()


def fsrgemm_status_string(status: int) -> str:
    return load().fsrgemm_status_string(int(status)).decode()


def fsrgemm_version() -> int:
    return int(load().fsrgemm_version())


def check(status: int) -> None:
    """Raise FsrGemmError unless status is FSRGEMM_OK."""
    if status != FSRGEMM_OK:
        raise FsrGemmError("fsrgemm: %s (%d)" % (fsrgemm_status_string(status), status))
