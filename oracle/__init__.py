"""CPU oracle for C = A x B (the paper's Task 2, task-prompt table) and for
matrix transposition (Task 8).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
bench's cpu_baseline leg.  The GPU library never imports or calls it, and the
two share no code.

The arithmetic lives in ``gemm_oracle.c`` (a plain fp64 triple loop) and
``transpose_oracle.c`` (an element-by-element move); this module compiles them
with gcc, loads them with ctypes and adds the error metrics that the parity
tests gate on.  Matrices are numpy arrays; their strides are
passed through unchanged, so any row/column-major or padded view works.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gemm_oracle.c")
_SRC_T = os.path.join(_HERE, "transpose_oracle.c")
_LIB = os.path.join(_HERE, "libgemm_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle's C sources into libgemm_oracle.so beside them (gcc, OpenMP)."""
    newest = max(os.path.getmtime(_SRC), os.path.getmtime(_SRC_T))
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < newest:
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-o", tmp, _SRC, _SRC_T, "-lm"]
        )
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i64, vp = ctypes.c_int64, ctypes.c_void_p
        full = [i64, i64, i64, vp, i64, i64, vp, i64, i64, vp, i64, vp, i64]
        ent = [i64, vp, i64, i64, vp, i64, i64, i64, vp, vp, vp, vp]
        for name, sig in (
            ("oracle_gemm_f32", full),
            ("oracle_gemm_bf16", full),
            ("oracle_gemm_f32_entries", ent),
            ("oracle_gemm_bf16_entries", ent),
        ):
            fn = getattr(lib, name)
            fn.argtypes = sig
            fn.restype = ctypes.c_int
        lib.oracle_transpose_f32.argtypes = [i64, i64, vp, i64, i64, vp, i64, i64]
        lib.oracle_transpose_f32.restype = ctypes.c_int
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_set_num_threads.argtypes = [ctypes.c_int]
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def set_num_threads(n: int) -> None:
    _load().oracle_set_num_threads(int(n))


def _strides(x: np.ndarray):
    assert x.ndim == 2
    it = x.dtype.itemsize
    assert x.strides[0] % it == 0 and x.strides[1] % it == 0
    return x.strides[0] // it, x.strides[1] // it


def _kind(A: np.ndarray, B: np.ndarray) -> str:
    if A.dtype == np.float32 and B.dtype == np.float32:
        return "f32"
    if A.dtype == np.uint16 and B.dtype == np.uint16:
        return "bf16"
    raise TypeError("oracle takes float32 x float32 or uint16(bf16 bits) x uint16")


def gemm(A: np.ndarray, B: np.ndarray, want_scale: bool = True):
    """Return (C, S): C = A @ B in fp64, S = |A| @ |B| in fp64 (or None).

    A is (M, K), B is (K, N); float32, or uint16 holding bf16 bit patterns.
    Any strides are accepted (pass ``Bt.T`` for a column-major B).
    """
    kind = _kind(A, B)
    M, K = A.shape
    K2, N = B.shape
    if K != K2:
        raise ValueError("inner dimensions differ")
    C = np.empty((M, N), dtype=np.float64)
    S = np.empty((M, N), dtype=np.float64) if want_scale else None
    if M == 0 or N == 0:
        return C, S
    a_rs, a_cs = _strides(A)
    b_rs, b_cs = _strides(B)
    fn = getattr(_load(), "oracle_gemm_" + kind)
    rc = fn(M, N, K, A.ctypes.data, a_rs, a_cs, B.ctypes.data, b_rs, b_cs,
            C.ctypes.data, N, S.ctypes.data if want_scale else None, N)
    assert rc == 0
    return C, S


def transpose(A: np.ndarray) -> np.ndarray:
    """T with T[j][i] = A[i][j]: a new C-contiguous (cols, rows) float32 array.  Any strides are accepted."""
    if A.dtype != np.float32 or A.ndim != 2:
        raise TypeError("oracle.transpose takes a 2-D float32 array")
    rows, cols = A.shape
    T = np.empty((cols, rows), dtype=np.float32)
    if rows and cols:
        a_rs, a_cs = _strides(A)
        rc = _load().oracle_transpose_f32(rows, cols, A.ctypes.data, a_rs, a_cs, T.ctypes.data, rows, 1)
        assert rc == 0
    return T


def gemm_entries(A: np.ndarray, B: np.ndarray, ii, jj):
    """(c, s) for the listed entries only: c[t] = sum_k A[ii[t],k] B[k,jj[t]]."""
    kind = _kind(A, B)
    K = A.shape[1]
    if B.shape[0] != K:
        raise ValueError("inner dimensions differ")
    ii = np.ascontiguousarray(ii, dtype=np.int64)
    jj = np.ascontiguousarray(jj, dtype=np.int64)
    assert ii.shape == jj.shape and ii.ndim == 1
    if ii.size:
        assert 0 <= ii.min() and ii.max() < A.shape[0]
        assert 0 <= jj.min() and jj.max() < B.shape[1]
    c = np.empty(ii.size, dtype=np.float64)
    s = np.empty(ii.size, dtype=np.float64)
    a_rs, a_cs = _strides(A)
    b_rs, b_cs = _strides(B)
    fn = getattr(_load(), "oracle_gemm_%s_entries" % kind)
    rc = fn(K, A.ctypes.data, a_rs, a_cs, B.ctypes.data, b_rs, b_cs,
            ii.size, ii.ctypes.data, jj.ctypes.data, c.ctypes.data, s.ctypes.data)
    assert rc == 0
    return c, s


def bf16_bits_to_f64(x: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns (uint16) to fp64."""
    assert x.dtype == np.uint16
    return (x.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def componentwise_error(got: np.ndarray, ref: np.ndarray, scale: np.ndarray) -> float:
    """max_ij |got - ref| / S_ij with 0/0 := 0 and x/0 := inf (x != 0).

    This is the gated error metric: S_ij = sum_k |a_ik||b_kj| is the natural
    scale of a length-K dot product, so the bound is attainable even where
    C_ij cancels to almost zero.  NaN anywhere in ``got`` gives inf.
    """
    got = np.asarray(got, dtype=np.float64)
    if got.size == 0:
        return 0.0
    if not np.all(np.isfinite(got)):
        return float("inf")
    d = np.abs(got - ref)
    with np.errstate(divide="ignore", invalid="ignore"):
        r = np.where(scale > 0, d / scale, np.where(d > 0, np.inf, 0.0))
    return float(r.max())


def freivalds_residual(A: np.ndarray, B: np.ndarray, got: np.ndarray, n_vec: int = 3, seed: int = 0) -> float:
    """Randomised whole-matrix check in O(MN + MK + KN) fp64 work.

    For random +-1 vectors x returns max_i |(got x)_i - (A (B x))_i| / (|A| (|B| 1))_i.
    A wrong entry of ``got`` of relative size e (against S) shows up as a
    residual of about e / sqrt(N) or more, so this catches gross errors
    anywhere in a matrix too large to verify entry by entry.
    """
    if A.dtype == np.uint16:
        Af, Bf = bf16_bits_to_f64(A), bf16_bits_to_f64(B)
    else:
        Af, Bf = A.astype(np.float64), B.astype(np.float64)
    G = np.asarray(got, dtype=np.float64)
    if not np.all(np.isfinite(G)):
        return float("inf")
    rng = np.random.default_rng(seed)
    scale = np.abs(Af) @ (np.abs(Bf) @ np.ones(Bf.shape[1]))
    worst = 0.0
    for _ in range(n_vec):
        x = rng.integers(0, 2, size=Bf.shape[1]).astype(np.float64) * 2.0 - 1.0
        r = np.abs(G @ x - Af @ (Bf @ x))
        with np.errstate(divide="ignore", invalid="ignore"):
            q = np.where(scale > 0, r / scale, np.where(r > 0, np.inf, 0.0))
        worst = max(worst, float(q.max()) if q.size else 0.0)
    return worst
