"""Validator-side plumbing shared by the bench and the GPU tests: moves seeded
operands to the device with canary padding, calls the C ABI, brings C back and
checks the canaries.  No arithmetic of the product happens here."""
from __future__ import annotations

import numpy as np
import torch

from . import inputs

SENTINEL = np.float32(-7.25e30)      # pre-fill of C and its padding
_NAN = {np.dtype(np.float32): np.float32(np.nan), np.dtype(np.uint16): np.uint16(0x7FC0)}


def _dev(buf: np.ndarray) -> torch.Tensor:
    if buf.dtype == np.uint16:
        return torch.from_numpy(buf.view(np.int16)).cuda()
    return torch.from_numpy(buf).cuda()


def _unpack(flat: np.ndarray, M: int, N: int, ldc: int, offset: int) -> np.ndarray:
    """Checks that everything outside the M x N block still holds the sentinel; returns the block."""
    assert np.all(flat[:offset] == SENTINEL), "wrote before C"
    assert np.all(flat[offset + M * ldc:] == SENTINEL), "wrote past C"
    body = flat[offset:offset + M * ldc].reshape(M, ldc)
    assert np.all(body[:, N:] == SENTINEL), "wrote into C's row padding"
    return body[:, :N].copy()


def _run(call, stored, out_shape, lds, ldc, offset, repeat, workspace_bytes=None):
    """The one run loop: `stored` are the operands as they lie in memory (numpy, 2-D), embedded at leading dimensions
    `lds` with NaN padding and `offset` leading elements; the result block of `out_shape` sits at leading dimension
    `ldc` in a sentinel-filled buffer, and so does a workspace of `workspace_bytes` (None: the call takes none).
    `call(operand pointers..., result pointer, workspace pointer or None, stream)` makes the library call and
    returns its status.  Every repeat starts from fresh result and workspace buffers; all repeats must agree bit for
    bit.  Returns the result block."""
    dev = [_dev(inputs.embed(x, ld, _NAN[x.dtype], offset)) for x, ld in zip(stored, lds)]
    ptrs = [d.data_ptr() + x.dtype.itemsize * offset for d, x in zip(dev, stored)]
    rows, cols = out_shape
    c_host = np.full(offset + rows * ldc + 3, SENTINEL, dtype=np.float32)
    guard = 64
    ws_host = None if workspace_bytes is None else np.full(workspace_bytes // 4 + guard, SENTINEL, dtype=np.float32)
    outs = []
    for _ in range(repeat):
        c = _dev(c_host)
        ws = None if ws_host is None else _dev(ws_host)
        st = call(*ptrs, c.data_ptr() + 4 * offset, ws.data_ptr() if workspace_bytes else None, torch.cuda.current_stream().cuda_stream)
        lib_check(st)
        torch.cuda.synchronize()
        if ws is not None:
            assert np.all(ws.cpu().numpy()[workspace_bytes // 4:] == SENTINEL), "wrote past the workspace"
        outs.append(_unpack(c.cpu().numpy(), rows, cols, ldc, offset))
    for o in outs[1:]:
        assert np.array_equal(o.view(np.uint32), outs[0].view(np.uint32)), "run-to-run results differ"
    return outs[0]


def lib_check(status):
    from . import fsrgemm

    fsrgemm.check(status)


def _stored(transA, transB, A, B):
    """Operands in the storage the flags describe: an operand flagged transposed is handed over as K x M / N x K."""
    return (np.ascontiguousarray(A.T) if transA else A), (np.ascontiguousarray(B.T) if transB else B)


def _lds(sa, sb, N, lda, ldb, ldc):
    return lda or max(sa.shape[1], 1), ldb or max(sb.shape[1], 1), ldc or max(N, 1)


def run_f32(lib, A: np.ndarray, B: np.ndarray, lda=None, ldb=None, ldc=None, offset=0, repeat=1):
    """C = A.B through gemm_f32 with padded, canaried buffers.  Returns the M x N result (numpy)."""
    (M, K), N = A.shape, B.shape[1]
    lda, ldb, ldc = _lds(A, B, N, lda, ldb, ldc)
    return _run(lambda a, b, c, ws, st: lib.gemm_f32(M, N, K, a, lda, b, ldb, c, ldc, st), (A, B), (M, N), (lda, ldb), ldc, offset, repeat)


def run_f32_ex(lib, transA: bool, transB: bool, A: np.ndarray, B: np.ndarray, lda=None, ldb=None, ldc=None, offset=0,
               repeat=1):
    """C = A.B through gemm_f32_ex.  A (M x K) and B (K x N) are the logical operands; an operand flagged
    transposed is handed to the library in transposed storage (K x M, N x K)."""
    (M, K), N = A.shape, B.shape[1]
    sa, sb = _stored(transA, transB, A, B)
    lda, ldb, ldc = _lds(sa, sb, N, lda, ldb, ldc)
    return _run(lambda a, b, c, ws, st: lib.gemm_f32_ex(transA, transB, M, N, K, a, lda, b, ldb, c, ldc, st), (sa, sb), (M, N), (lda, ldb),
                ldc, offset, repeat)


def _run_ws(lib, kind: str, transA, transB, A, B, workspace_bytes, lda, ldb, ldc, offset, repeat, forced=None):
    (M, K), N = A.shape, B.shape[1]
    sa, sb = _stored(transA, transB, A, B)
    lda, ldb, ldc = _lds(sa, sb, N, lda, ldb, ldc)
    gemm, query = (lib.gemm_f32_ws, lib.gemm_f32_workspace_bytes) if kind == "f32" else (lib.gemm_bf16_ws, lib.gemm_bf16_workspace_bytes)
    if forced is not None:          # (tile, k_slices): the *_cfg entry point with exactly the workspace its split needs
        gemm_cfg = lib.gemm_f32_cfg if kind == "f32" else lib.gemm_bf16_cfg
        gemm = lambda *args: gemm_cfg(forced[0], forced[1], *args)
        workspace_bytes = forced[1] * M * N * 4 if forced[1] > 1 or (kind == "f32" and forced[0] == 4) else 0
    if workspace_bytes is None:
        workspace_bytes = query(transA, transB, M, N, K)
    return _run(lambda a, b, c, ws, st: gemm(transA, transB, M, N, K, a, lda, b, ldb, c, ldc, ws, workspace_bytes, st), (sa, sb), (M, N),
                (lda, ldb), ldc, offset, repeat, workspace_bytes=workspace_bytes)


def run_f32_ws(lib, transA: bool, transB: bool, A: np.ndarray, B: np.ndarray, workspace_bytes=None, lda=None, ldb=None,
               ldc=None, offset=0, repeat=1):
    """C = A.B through gemm_f32_ws with a canaried workspace of `workspace_bytes` (default: what the library asks
    for).  A (M x K), B (K x N) are the logical operands.  Checks that nothing behind the stated workspace size
    was written; returns the M x N result."""
    return _run_ws(lib, "f32", transA, transB, A, B, workspace_bytes, lda, ldb, ldc, offset, repeat)


def run_bf16_ws(lib, transA: bool, transB: bool, A: np.ndarray, B: np.ndarray, workspace_bytes=None, lda=None, ldb=None,
                ldc=None, offset=0, repeat=1):
    """The same through gemm_bf16_ws; operands are bf16 bit patterns."""
    return _run_ws(lib, "bf16", transA, transB, A, B, workspace_bytes, lda, ldb, ldc, offset, repeat)


def run_cfg(lib, kind: str, tile: int, k_slices: int, transA: bool, transB: bool, A: np.ndarray, B: np.ndarray, lda=None,
            ldb=None, ldc=None, offset=0, repeat=1):
    """C = A.B through gemm_f32_cfg / gemm_bf16_cfg (kind "f32" / "bf16") with the given tile and K slices, and a
    canaried workspace of exactly the size the split needs.  Raises FsrGemmError when the library rejects the
    candidate."""
    return _run_ws(lib, kind, transA, transB, A, B, None, lda, ldb, ldc, offset, repeat, forced=(tile, k_slices))


def run_bf16(lib, A: np.ndarray, Bt: np.ndarray, lda=None, ldb=None, ldc=None, offset=0, repeat=1):
    """C = A.B through gemm_bf16; A is (M, K) bf16 bits, Bt is (N, K) bf16 bits (column-major B)."""
    (M, K), N = A.shape, Bt.shape[0]
    assert Bt.shape[1] == K
    lda, ldb, ldc = lda or max(K, 1), ldb or max(K, 1), ldc or max(N, 1)
    return _run(lambda a, b, c, ws, st: lib.gemm_bf16(M, N, K, a, lda, b, ldb, c, ldc, st), (A, Bt), (M, N), (lda, ldb), ldc, offset, repeat)


def run_bf16_ex(lib, transA: bool, transB: bool, A: np.ndarray, B: np.ndarray, lda=None, ldb=None, ldc=None, offset=0,
                repeat=1):
    """C = A.B through gemm_bf16_ex.  A (M x K) and B (K x N) are the logical operands as bf16 bits; an operand
    flagged transposed is handed to the library in transposed storage (K x M, N x K)."""
    (M, K), N = A.shape, B.shape[1]
    sa, sb = _stored(transA, transB, A, B)
    lda, ldb, ldc = _lds(sa, sb, N, lda, ldb, ldc)
    return _run(lambda a, b, c, ws, st: lib.gemm_bf16_ex(transA, transB, M, N, K, a, lda, b, ldb, c, ldc, st), (sa, sb), (M, N), (lda, ldb),
                ldc, offset, repeat)


def run_noalloc(lib, transA: bool, transB: bool, A: np.ndarray, B: np.ndarray, lda=None, ldb=None, ldc=None, offset=0, repeat=1):
    """C = A.B through gemm_f32_noalloc (the library's own scratch array instead of a workspace)."""
    (M, K), N = A.shape, B.shape[1]
    sa, sb = _stored(transA, transB, A, B)
    lda, ldb, ldc = _lds(sa, sb, N, lda, ldb, ldc)
    return _run(lambda a, b, c, ws, st: lib.gemm_f32_noalloc(transA, transB, M, N, K, a, lda, b, ldb, c, ldc, st), (sa, sb), (M, N), (lda, ldb),
                ldc, offset, repeat)


def run_transpose(lib, A: np.ndarray, lda=None, ldt=None, offset=0, repeat=1):
    """T = transpose of A (rows x cols float32) through transpose_f32 with padded, canaried buffers.
    Returns the cols x rows result; checks that nothing outside it was written."""
    rows, cols = A.shape
    lda, ldt = lda or max(cols, 1), ldt or max(rows, 1)
    return _run(lambda a, t, ws, st: lib.transpose_f32(rows, cols, a, lda, t, ldt, st), (A,), (cols, rows), (lda,), ldt, offset, repeat)
