"""Host-side checks that need no GPU: the library loads, exports what the header
declares, and rejects malformed problems before touching the device."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2506_09092_amd as lib

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "fsrgemm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b([a-z_0-9]+)\s*\(", text)) - {"defined"})


def test_library_loads_and_exports_every_declared_symbol():
    names = _declared_functions()
    assert {"gemm_f32", "gemm_bf16", "fsrgemm_status_string", "fsrgemm_version"} <= set(names)
    assert set(names) == set(lib.EXPORTS)
    handle = ctypes.CDLL(lib.library_path())
    for n in names:
        assert hasattr(handle, n), n
    assert lib.fsrgemm_version() >= 100


def test_status_strings():
    seen = {lib.fsrgemm_status_string(s) for s in (0, -1, -2, -3)}
    assert len(seen) == 4 and "ok" in seen
    assert "unknown" in lib.fsrgemm_status_string(-99)


P = 0x1000      # a non-null, 16-byte aligned fake address: never dereferenced by the checks


@pytest.mark.parametrize("fn", ["gemm_f32", "gemm_bf16"])
def test_invalid_arguments_are_rejected_without_a_device(fn):
    f = getattr(lib, fn)
    ldb_min = 8 if fn == "gemm_f32" else 16          # N for row-major B, K for column-major B
    ok = dict(M=4, N=8, K=16, A=P, lda=16, B=P, ldb=ldb_min, C=P, ldc=8)

    def call(**kw):
        a = dict(ok, **kw)
        return f(a["M"], a["N"], a["K"], a["A"], a["lda"], a["B"], a["ldb"], a["C"], a["ldc"], 0)

    bad = lib.FSRGEMM_ERR_INVALID_ARG
    assert call(M=-1) == bad and call(N=-1) == bad and call(K=-1) == bad
    assert call(lda=15) == bad and call(ldb=ldb_min - 1) == bad and call(ldc=7) == bad
    assert call(A=None) == bad and call(B=None) == bad and call(C=None) == bad
    assert call(M=2 ** 31) == bad and call(K=2 ** 31) == bad
    # empty outputs are fine and launch nothing, whatever the pointers
    assert call(M=0, A=None, C=None) == lib.FSRGEMM_OK
    assert call(N=0, ldb=ldb_min if fn == "gemm_bf16" else 0, ldc=0, B=None, C=None) == lib.FSRGEMM_OK
    with pytest.raises(lib.FsrGemmError):
        lib.check(bad)


def test_dispatch_query_names_variants():
    q = lib.fsrgemm_kernel_for_f32
    fast = q(4096, 4096, 4096, P, 4096, P, 4096, P, 4096)
    ragged = q(4097, 17, 1000, P, 1000, P, 20, P, 17)
    unaligned = q(123, 20, 8, P + 4, 8, P + 4, 20, P, 20)
    # <TM, TN, min waves, load mode, A layout, B layout>: tile (64 TM) x (64 TN); mode 0 unchecked vectors,
    # 1 vectors + predicated edges, 2 scalar; row-major A is contiguous along k (0), row-major B along n (1)
    # the direct-to-LDS kernel <blocks per wavefront, A layout, B layout> where it fits, in the shape that fills whole
    # rounds; a rest of K in whole 16-byte pieces stays (one more K-tile with zero pieces), and no shape takes a K below 32
    assert fast == "gemm_f32_main_kernel<4, 4, 0, 1>"
    assert q(4096, 4096, 4112, P, 4112, P, 4096, P, 4096) == "gemm_f32_main_kernel<4, 4, 0, 1>"
    assert q(4096, 4096, 16, P, 16, P, 4096, P, 4096) == "gemm_f32_kernel<4, 2, 2, 0, 0, 1>"
    assert ragged == "gemm_f32_kernel<1, 1, 4, 1, 0, 1>" and unaligned == "gemm_f32_kernel<1, 1, 4, 2, 0, 1>"
    assert q(4090, 4090, 129, P, 132, P, 4092, P, 4090) == "gemm_f32_kernel<4, 2, 2, 1, 0, 1>"
    # one row and column beyond 4096 would cost the largest tile a whole further round: a smaller one takes it
    assert q(4097, 4097, 129, P, 132, P, 4100, P, 4097) == "gemm_f32_kernel<2, 2, 3, 1, 0, 1>"
    assert q(64, 64, 0, P, 4, P, 64, P, 64) == "gemm_f32_kernel<1, 1, 4, 1, 0, 1>"                    # K = 0 never takes the unchecked mode
    assert q(4, 4, 4, P, 3, P, 4, P, 4) is None
    qb = lib.fsrgemm_kernel_for_bf16
    assert qb(8192, 8192, 8192, P, 8192, P, 8192, P, 8192) == "gemm_bf16_main_kernel<8, 8, 0, 0>"
    # general kernel <T, min waves, load mode>: tile (64 T) x (64 T)
    # <blocks of 16 rows per wavefront, of 16 columns, A layout, B layout>: tile (32 IM) x (32 JN), in the shape that fills
    # whole rounds; a K that is not whole K-tiles of 64 but whole 16-byte pieces stays (one more K-tile with zero pieces)
    assert qb(8192, 8192, 8200, P, 8200, P, 8200, P, 8192) == "gemm_bf16_main_kernel<8, 8, 0, 0>"
    assert qb(8192, 8192, 8196, P, 8200, P, 8200, P, 8192) == "gemm_bf16_kernel<4, 1, 1, 0, 0>"   # K not a multiple of 8
    assert qb(6144, 6144, 6144, P, 6144, P, 6144, P, 6144) == "gemm_bf16_main_kernel<8, 6, 0, 0>"   # 768 tiles of 256 x 192: 3 whole rounds
    assert qb(8192, 8192, 56, P, 56, P, 56, P, 8192) == "gemm_bf16_kernel<4, 1, 1, 0, 0>"           # under one K-tile
    assert qb(2048, 2048, 512, P, 512, P, 512, P, 2048) == "gemm_bf16_main_kernel<4, 4, 0, 0>"      # 256 tiles of 128 x 128, two to a compute unit
    assert qb(2048, 2048, 516, P, 516, P, 516, P, 2048) == "gemm_bf16_kernel<2, 2, 2, 0, 0>"       # rows that are not whole pieces: the general tile
    assert qb(100, 100, 100, P, 100, P, 100, P, 100) == "gemm_bf16_kernel<1, 4, 2, 0, 0>"         # ld not a multiple of 8
    assert qb(100, 100, 100, P, 104, P, 104, P, 100) == "gemm_bf16_kernel<1, 4, 1, 0, 0>"
    # leading dimensions of 2^25 elements and more do not fit the main kernel's 32-bit lane offsets
    assert qb(8192, 8192, 8192, P, 1 << 25, P, 8192, P, 8192) == "gemm_bf16_kernel<4, 1, 0, 0, 0>"
    assert qb(8192, 8192, 8192, P, (1 << 25) - 8, P, 8192, P, 8192) == "gemm_bf16_main_kernel<8, 8, 0, 0>"
    # ragged M and N still take the unchecked kernels (last tiles are shifted back); a ragged K does not
    assert qb(8000, 8000, 8000, P, 8000, P, 8000, P, 8000) == "gemm_bf16_main_kernel<8, 8, 0, 0>"
    assert qb(8000, 8000, 8008, P, 8008, P, 8008, P, 8000) == "gemm_bf16_main_kernel<8, 8, 0, 0>"
    assert qb(8000, 8000, 8004, P, 8008, P, 8008, P, 8000) == "gemm_bf16_kernel<4, 1, 1, 0, 0>"
    assert qb(255, 8192, 8192, P, 8192, P, 8192, P, 8192) == "gemm_bf16_kernel<1, 4, 0, 0, 0>"          # 4 x 128 tiles of 64
    assert q(4000, 4000, 4000, P, 4000, P, 4000, P, 4000) == "gemm_f32_main_kernel<4, 4, 0, 1>"
    assert q(4000, 4000, 4008, P, 4008, P, 4000, P, 4000) == "gemm_f32_main_kernel<4, 4, 0, 1>"          # a rest of K
    assert q(4000, 4000, 4010, P, 4012, P, 4000, P, 4000) == "gemm_f32_kernel<4, 2, 2, 1, 0, 1>"          # K not a multiple of 4
    assert q(63, 4000, 4000, P, 4000, P, 4000, P, 4000) == "gemm_f32_kernel<1, 1, 4, 1, 0, 1>"            # narrower than a tile
    # other storage orders: <.., A layout, B layout> with 0 = contiguous along k, 1 = along m / n
    qx = lib.fsrgemm_kernel_for_bf16_ex
    assert qx(0, 1, 8192, 8192, 8192, P, 8192, P, 8192, P, 8192) == "gemm_bf16_main_kernel<8, 8, 0, 0>"
    assert qx(0, 0, 8192, 8192, 8192, P, 8192, P, 8192, P, 8192) == "gemm_bf16_main_kernel<8, 8, 0, 1>"
    assert qx(1, 1, 8192, 8192, 8192, P, 8192, P, 8192, P, 8192) == "gemm_bf16_main_kernel<8, 8, 1, 0>"
    assert qx(1, 0, 8192, 8192, 8192, P, 8192, P, 8192, P, 8192) == "gemm_bf16_main_kernel<8, 8, 1, 1>"
    # an operand contiguous along m (n) keeps the main kernel only if M (N) is a multiple of 8
    assert qx(1, 0, 8000, 4008, 512, P, 8000, P, 4008, P, 4008) == "gemm_bf16_main_kernel<8, 8, 1, 1>"
    assert qx(1, 1, 8004, 8000, 512, P, 8008, P, 512, P, 8000) == "gemm_bf16_kernel<4, 1, 0, 1, 0>"
    assert qx(0, 0, 8004, 8004, 512, P, 512, P, 8008, P, 8004) == "gemm_bf16_kernel<4, 1, 0, 0, 1>"
    assert qx(0, 1, 8004, 8004, 512, P, 512, P, 512, P, 8004) == "gemm_bf16_main_kernel<6, 6, 0, 0>"
    assert qx(1, 0, 100, 100, 100, P, 104, P, 104, P, 100) == "gemm_bf16_kernel<1, 4, 1, 1, 1>"
    # with such an operand the 128 x 128 tile runs from 4 tiles on (with both operands along k: from 192 tiles on, the
    # general 64 x 64 tile below)
    assert qx(0, 0, 1024, 1024, 1024, P, 1024, P, 1024, P, 1024) == "gemm_bf16_main_kernel<4, 4, 0, 1>"
    assert qx(1, 1, 256, 256, 4096, P, 256, P, 4096, P, 256) == "gemm_bf16_main_kernel<4, 4, 1, 0>"
    assert qx(1, 0, 2048, 2048, 2048, P, 2048, P, 2048, P, 2048) == "gemm_bf16_main_kernel<4, 4, 1, 1>"
    assert qx(1, 0, 128, 256, 512, P, 128, P, 256, P, 256) == "gemm_bf16_kernel<1, 4, 0, 1, 1>"         # 2 tiles
    assert qx(0, 1, 1024, 1024, 1024, P, 1024, P, 1024, P, 1024) == "gemm_bf16_kernel<1, 4, 0, 0, 0>"
    qh = lib.fsrgemm_kernel_for_bf16_cfg
    for tile, (im, jn) in {0: (8, 8), 5: (6, 8), 6: (4, 8), 7: (8, 6), 8: (6, 6), 9: (8, 4), 10: (4, 4)}.items():
        for ta, tb in ((0, 1), (0, 0), (1, 1), (1, 0)):
            assert qh(tile, ta, tb, 512, 512, 512, P, 512, P, 512, P, 512) == "gemm_bf16_main_kernel<%d, %d, %d, %d>" % (im, jn, ta, 1 - tb)
    assert qx(1, 0, 100, 90, 80, P, 99, P, 90, P, 90) is None                                 # lda < M for a transposed A


@pytest.mark.parametrize("ta,tb", [(0, 0), (0, 1), (1, 0), (1, 1)])
def test_transposed_storage_arguments(ta, tb):
    # leading dimensions are checked against the extent that is contiguous in the stated storage order
    M, N, K = 6, 10, 16
    lda_min, ldb_min = (M if ta else K), (K if tb else N)

    def call(lda, ldb, ldc=N):
        return lib.gemm_f32_ex(ta, tb, M, N, K, P, lda, P, ldb, P, ldc, 0)

    bad = lib.FSRGEMM_ERR_INVALID_ARG
    assert call(lda_min - 1, ldb_min) == bad and call(lda_min, ldb_min - 1) == bad and call(lda_min, ldb_min, N - 1) == bad
    assert lib.gemm_f32_ex(ta, tb, 0, N, K, None, lda_min, P, ldb_min, None, N, 0) == lib.FSRGEMM_OK
    q = lib.fsrgemm_kernel_for_f32_ex
    # <TM, TN, min waves, load mode, A layout, B layout>: layout 0 = contiguous along k, 1 = along m / n
    assert q(ta, tb, 4096, 4096, 4096, P, 4096, P, 4096, P, 4096) == "gemm_f32_main_kernel<4, 4, %d, %d>" % (ta, 1 - tb)
    assert q(ta, tb, 4096, 2048, 4096, P, 4096, P, 4096, P, 2048) == "gemm_f32_main_kernel<2, 4, %d, %d>" % (ta, 1 - tb)
    assert q(ta, tb, 4096, 2048, 16, P, 4096, P, 2048, P, 2048) == "gemm_f32_kernel<4, 2, 2, 0, %d, %d>" % (ta, 1 - tb)     # K below a K-tile of 32
    assert q(ta, tb, M, N, K, P, lda_min - 1, P, ldb_min, P, N) is None
    assert lib.fsrgemm_kernel_for_f32(4096, 4096, 4096, P, 4096, P, 4096, P, 4096) == q(0, 0, 4096, 4096, 4096, P, 4096, P, 4096, P, 4096)


def test_workspace_query_and_argument_checks():
    wb = lib.gemm_f32_workspace_bytes
    # (under 64 rows the direct-to-LDS shapes do not fit: the general 64 x 64 tile in slices)
    assert wb(0, 0, 17, 4096, 4096) == 16 * 17 * 4096 * 4           # 64 tiles, 256 K-tiles -> 16 slices of 16 K-tiles
    assert wb(0, 0, 8, 4096, 4096) == 2 * 8 * 4096 * 4              # a row-major B streams through the vector kernels whatever its alignment: 2 slices
    assert wb(0, 0, 17, 16384, 16384) == 4 * 17 * 16384 * 4         # 256 tiles -> 4 slices
    assert wb(0, 0, 8, 16384, 16384) == 0                           # streamed in one piece: 512 workgroups
    assert wb(0, 0, 1, 4096, 4096) == 2 * 4096 * 4                  # a row times a matrix: 128 workgroups of 32 columns -> 2 slices
    assert wb(0, 0, 4096, 1, 4096) == 0                             # a matrix times a column: 1024 workgroups of 4 rows
    assert wb(0, 0, 1280, 1280, 1280) == 0                           # 400 tiles, but only 80 K-tiles
    assert wb(0, 0, 256, 256, 65536) == 64 * 256 * 256 * 4           # 4 tiles of 128 x 128 -> the cap of 64 slices: 16 MiB
    # 16 tiles of 64 x 64 x 16 slices (a workgroup per compute unit) on the direct-to-LDS kernel, 64 slices on the general
    # one, which runs if the operands turn out misaligned: the query names the larger need
    assert wb(0, 0, 256, 256, 16384) == 64 * 256 * 256 * 4 and wb(0, 0, 768, 768, 2048) == 3 * 768 * 768 * 4
    assert wb(1, 1, 256, 256, 65536) == wb(0, 0, 256, 256, 65536)
    assert wb(0, 0, 64, 64, 256) == 0                                 # K too short to cut
    assert wb(0, 0, 4096, 4096, 4096) == 0 and wb(0, 0, 0, 5, 4096) == 0 and wb(0, 0, -1, 5, 4096) == 0
    wh = lib.gemm_bf16_workspace_bytes
    assert wh(0, 1, 8, 4096, 4096) == 16 * 8 * 4096 * 4 and wh(0, 1, 64, 64, 256) == 0 and wh(0, 1, 8192, 8192, 8192) == 0
    assert wh(0, 1, 8, 16384, 16384) == 4 * 8 * 16384 * 4
    # a vector on one side: the streaming kernels; one wavefront per matrix row needs no split, 64 columns per workgroup do
    assert wh(0, 1, 1, 4096, 4096) == 0 and wh(0, 0, 1, 4096, 4096) == 4 * 4096 * 4
    pb = lib.fsrgemm_plan_bf16
    assert pb(0, 1, 1, 8192, 8192, P, 8192, P, 8192) == (4, 1) and pb(0, 0, 1, 8192, 8192, P, 8192, P, 8192, True) == (4, 8) and pb(0, 0, 1, 4096, 4096, P, 4096, P, 4096, True) == (4, 4)
    qb = lib.fsrgemm_kernel_for_bf16_ex
    assert qb(0, 1, 1, 8192, 8192, P, 8192, P, 8192, P, 8192) == "gemv_rows_bf16_kernel<true>"
    assert qb(0, 0, 1, 8192, 8192, P, 8192, P, 8192, P, 8192) == "gemv_cols_bf16_kernel<true>"
    assert qb(0, 1, 1, 8192, 8196, P, 8196, P, 8196, P, 8192) == "gemv_rows_bf16_kernel<false>"         # rows not 16-byte aligned
    assert lib.fsrgemm_kernel_for_bf16_cfg(4, 0, 1, 8192, 1, 8192, P, 8192, P, 8192, P, 1) == "gemv_rows_bf16_kernel<true>"
    # up to 16 vectors contiguous along k against a matrix contiguous along k, K whole 16-byte pieces: the matrix-core kernel
    assert lib.fsrgemm_kernel_for_bf16_cfg(4, 0, 1, 8192, 2, 8192, P, 8192, P, 8192, P, 2) == "gemv_rows_bf16_mfma_direct_kernel"       # up to 8: the form without LDS
    assert lib.fsrgemm_kernel_for_bf16_cfg(4, 0, 1, 8192, 9, 8192, P, 8192, P, 8192, P, 9) == "gemv_rows_bf16_mfma_kernel"
    assert lib.fsrgemm_kernel_for_bf16_cfg(4, 0, 1, 8192, 16, 8192, P, 8192, P, 8192, P, 16) == "gemv_rows_bf16_mfma_kernel"
    assert lib.fsrgemm_kernel_for_bf16_cfg(4, 0, 1, 8192, 2, 8188, P, 8192, P, 8192, P, 2) == "gemv_rows_bf16_few_kernel<2>"      # K not whole pieces
    assert lib.fsrgemm_kernel_for_bf16_cfg(4, 1, 1, 8192, 2, 8192, P, 8192, P, 8192, P, 2) == "gemv_cols_bf16_few_kernel<2>"
    assert lib.fsrgemm_kernel_for_bf16_cfg(4, 0, 1, 8192, 17, 8192, P, 8192, P, 8192, P, 17) is None            # 17 columns: no vector side
    assert lib.fsrgemm_kernel_for_bf16_cfg(4, 1, 1, 8192, 9, 8192, P, 8192, P, 8192, P, 9) is None              # nine, and not the matrix-core kernel's storage
    assert lib.fsrgemm_kernel_for_bf16_cfg(4, 0, 1, 8192, 2, 8192, P + 2, 8192, P, 8192, P, 2) == "gemv_rows_bf16_few_kernel<2>"       # the streamed operand misaligned: lane arithmetic
    assert lib.fsrgemm_kernel_for_bf16_cfg(4, 0, 1, 8192, 9, 8192, P + 2, 8192, P, 8192, P, 9) is None          # nine vectors need the matrix-core kernel, which needs aligned pieces
    # without a workspace the streaming kernels take such calls; with one, the 64 x 64 tiles where they split K and there are
    # more than 8 vectors on a long matrix (matrix-core kernel) or more than 4 (the others)
    pbx = lambda M, N, K, ws: lib.fsrgemm_plan_bf16(0, 1, M, N, K, P, K, P, K, ws, True)
    assert pbx(8, 8192, 8192, False) == (4, 1) and pbx(8, 8192, 8192, True) == (4, 1) and pbx(16, 8192, 8192, False) == (4, 1)
    assert pbx(16, 8192, 8192, True) == (3, 8) and pbx(16, 2048, 8192, True) == (4, 4) and pbx(12, 1024, 16384, True) == (4, 8)
    assert pbx(17, 8192, 8192, False) == (3, 1) and pbx(8, 8192, 128, True) == (4, 1)
    pbn = lambda M, N, K, ws: lib.fsrgemm_plan_bf16(0, 0, M, N, K, P, K, P, N, ws, True)
    assert pbn(4, 8192, 8192, True) == (4, 4) and pbn(8, 8192, 8192, True) == (3, 8) and pbn(8, 8192, 8192, False) == (4, 1) and pbn(16, 8192, 8192, False) == (3, 1)
    assert lib.fsrgemm_kernel_for_bf16_ex(0, 0, 3, 8192, 8192, P, 8192, P, 8192, P, 8192) == "gemv_cols_bf16_few_kernel<4>"
    bad = lib.FSRGEMM_ERR_INVALID_ARG
    assert lib.gemm_bf16_ws(0, 1, 1, 8, 4096, P, 4096, P, 4096, P, 8, None, 64, 0) == bad
    assert lib.gemm_bf16_ws(0, 1, 1, 8, 4096, P, 4096, P, 4095, P, 8, P, 1 << 20, 0) == bad   # ldb < K
    assert lib.gemm_f32_ws(0, 0, 1, 8, 4096, P, 4096, P, 8, P, 8, None, 64, 0) == bad      # bytes without a pointer
    assert lib.gemm_f32_ws(0, 0, 1, 8, 4096, P, 4096, P, 8, P, 8, P, -1, 0) == bad
    assert lib.gemm_f32_ws(0, 0, 1, 8, 4096, P, 4095, P, 8, P, 8, P, 1 << 20, 0) == bad    # lda < K
    assert lib.gemm_f32_ws(0, 0, 0, 8, 4096, None, 4096, P, 8, None, 8, None, 0, 0) == lib.FSRGEMM_OK


def test_f32_tile_rule_follows_the_round_model():
    # fewest rounds of 256 tiles, weighted by the tile's time; sizes where the configurations win in turn.  The
    # direct-to-LDS kernel (5..16: tiles with sides of 256, 192, 128 and 64) enters where it fits
    # (aligned operands, whole K-tiles of 32) with the shape whose tiles fill whole rounds
    pf = lambda n, a=P, K=None: lib.fsrgemm_plan_f32(0, 0, n, n, K or n, a, K or n, P, n)[0]
    assert [pf(n) for n in (1024, 2048, 3072, 4096, 6144, 8192)] == [14, 10, 12, 5, 9, 5]
    assert pf(1024, P + 4) == 2 and pf(2560) == 14 and lib.fsrgemm_plan_f32(0, 0, 1024, 2048, 4096, P, 4096, P, 2048)[0] == 15
    assert [pf(n, P + 4) for n in (4096, 8192)] == [0, 0] and pf(4096, K=4112) == 5      # misaligned A: the general kernel; a rest of K: the same tile
    assert lib.fsrgemm_plan_f32(0, 0, 4096, 4096, 4110, P, 4112, P, 4096)[0] == 0 and pf(4096, K=16) == 0     # K not a multiple of 4, K below a K-tile
    assert lib.fsrgemm_plan_f32(0, 0, 17, 100000, 64, P, 64, P, 100000)[0] == 2          # a sliver: small tiles waste least
    assert lib.fsrgemm_plan_f32(0, 0, 262144, 2048, 4096, P, 4096, P, 2048)[0] == 5        # the paper's largest Task-2 size


def test_splits_take_the_larger_tile_where_it_still_fills_the_compute_units():
    # with a workspace, on the general kernels (fp32: operands the direct-to-LDS kernel cannot take, here a misaligned A): the
    # slices from the shape, then 128 x 128 tiles if tiles x slices reaches 240 workgroups (fp32: and a slice keeps 1024 k),
    # else 64 x 64 tiles.  fp32 tiles: 1 = 128 x 128, 2 = 64 x 64; bf16: 2 = 128 x 128, 3 = 64 x 64
    pf = lambda M, N, K: lib.fsrgemm_plan_f32(0, 0, M, N, K, P + 4, K, P, N, True, True)
    pb = lambda M, N, K: lib.fsrgemm_plan_bf16(0, 1, M, N, K, P, K, P, K, True, True)
    assert pf(512, 512, 65536) == (1, 16) and pf(384, 384, 65536) == (1, 28) and pf(1024, 1024, 4096) == (1, 4)
    assert pf(768, 768, 4096) == (2, 4)             # 36 tiles x 4 slices: too few workgroups
    assert pf(256, 256, 16384) == (2, 64)           # slices of 256 k: too short
    # bf16 from 128 rows and columns on: 64 x 64 tiles of the general kernel or 128 x 128 direct-to-LDS tiles (candidate 10) in
    # the slice count with the least modelled time, about a workgroup per compute unit; no split where K is short
    assert pb(512, 512, 65536) == (10, 16) and pb(256, 256, 16384) == (3, 16) and pb(768, 768, 4096) == (10, 5) and pb(512, 512, 8192) == (10, 10)
    assert pb(128, 2048, 4096) == (3, 4) and pb(1024, 1024, 2048) == (3, 1) and pb(512, 512, 512) == (3, 1)
    assert lib.fsrgemm_plan_bf16(0, 1, 512, 512, 65536, P + 2, 65536, P, 65536, True, True) == (3, 16)       # misaligned A: the general kernel only
    assert lib.gemm_f32_workspace_bytes(0, 0, 512, 512, 65536) == 16 * 512 * 512 * 4
    # a problem under 128 rows or columns keeps 64 x 64 tiles: most of a 128-wide tile would be padding
    assert pf(17, 8192, 8192) == (2, 8) and lib.fsrgemm_plan_f32(0, 0, 17, 8192, 8192, P, 8192, P, 8192, True, True) == (2, 8) and pb(32, 28672, 8192) == (3, 2) and pb(96, 8192, 8192) == (3, 4) and pb(128, 8192, 8192) == (10, 4)
    # fp32 with up to 16 rows (or columns) streams the other operand through the vector kernels (candidate 3), whatever that
    # operand's alignment: K slices only up to 256 workgroups.  With 9 .. 16
    # vectors against a matrix contiguous along k, and a workspace, the tiles in K slices stay
    assert pf(8, 8192, 8192) == (3, 1) and pf(8, 2048, 8192) == (3, 4) and lib.fsrgemm_plan_f32(0, 1, 8, 2048, 8192, P, 8192, P, 8192, True, True) == (3, 4)
    # (the streamed matrix may have any alignment)
    assert lib.fsrgemm_plan_f32(0, 0, 8, 8192, 8192, P, 8192, P + 4, 8192, True, True) == (3, 1) and lib.fsrgemm_plan_f32(0, 0, 8, 8192, 8192, P, 8192, P, 8193, True, True) == (3, 1)
    assert lib.fsrgemm_plan_f32(0, 1, 8, 8192, 8192, P, 8192, P + 4, 8192, True, True) == (3, 1) and lib.fsrgemm_plan_f32(0, 1, 8, 8192, 8192, P, 8192, P, 8193, True, True) == (3, 1)
    assert lib.fsrgemm_plan_f32(0, 0, 9, 8192, 8192, P, 8192, P, 8192, True, True) == (3, 1) and lib.fsrgemm_plan_f32(0, 0, 8, 2048, 8192, P, 8192, P, 2048, False, True) == (3, 1)
    assert lib.fsrgemm_plan_f32(0, 1, 16, 8192, 8192, P, 8192, P, 8192, True, True) == (2, 8) and lib.fsrgemm_plan_f32(0, 1, 16, 8192, 8192, P, 8192, P, 8192, False, True) == (3, 1)
    assert lib.fsrgemm_plan_f32(0, 1, 8, 8192, 8192, P, 8192, P, 8192, True, True) == (3, 1)
    assert lib.fsrgemm_kernel_for_f32_ex(0, 0, 12, 8192, 8192, P, 8192, P, 8192, P, 8192) == "gemv_cols_f32_few_kernel<16>"
    assert lib.fsrgemm_kernel_for_f32_ex(0, 0, 8, 2048, 8192, P, 8192, P, 2048, P, 2048) == "gemv_cols_f32_few_kernel<8>"
    assert lib.fsrgemm_kernel_for_f32_ex(0, 1, 3, 2048, 8192, P, 8192, P, 8192, P, 2048) == "gemv_rows_f32_few_kernel<4>"
    assert lib.fsrgemm_kernel_for_f32_ex(1, 0, 2048, 2, 8192, P, 2048, P, 2, P, 2) == "gemv_cols_f32_few_kernel<2>"
    assert lib.fsrgemm_kernel_for_f32_ex(1, 0, 3, 2, 8192, P, 4, P, 2, P, 2).startswith("gemm_f32_kernel<")     # three columns to walk: no whole piece
    assert lib.gemm_f32_workspace_bytes(0, 0, 8, 2048, 8192) == 4 * 8 * 2048 * 4 and lib.gemm_f32_workspace_bytes(0, 1, 8, 2048, 8192) == 4 * 8 * 2048 * 4


def test_f32_slices_on_the_direct_to_lds_shapes():
    # fp32 with a workspace and operands the direct-to-LDS kernel takes: the shape and slice count with the least modelled
    # time -- about a workgroup per compute unit, slices of 256 k and more, whole K-tiles; unsplit where that is as good
    pf = lambda M, N, K: lib.fsrgemm_plan_f32(0, 0, M, N, K, P, K, P, N, True, True)
    assert pf(256, 256, 16384) == (14, 16) and pf(64, 64, 4096) == (14, 16) and pf(256, 256, 1024) == (14, 4)       # 64 x 64 tiles
    assert pf(512, 512, 2048) == (14, 4) and pf(128, 2048, 4096) == (14, 4) and pf(768, 768, 2048) == (15, 3)       # .., 128 x 64
    assert pf(512, 512, 65536) == (10, 16) and pf(768, 768, 8192) == (10, 7) and pf(256, 256, 65536) == (10, 64)    # 128 x 128
    assert pf(1024, 1024, 4096) == (14, 1) and pf(64, 64, 256) == (14, 1) and pf(2048, 2048, 4096) == (10, 1)       # as without a workspace
    assert lib.gemm_f32_workspace_bytes(0, 0, 768, 768, 8192) == 7 * 768 * 768 * 4 and lib.gemm_f32_workspace_bytes(0, 0, 1024, 1024, 4096) == 4 * 1024 * 1024 * 4
    assert lib.fsrgemm_kernel_for_f32_cfg(14, 0, 0, 256, 256, 16384, P, 16384, P, 256, P, 256) == "gemm_f32_main_kernel<1, 1, 0, 1>"


def test_forced_configurations_and_plan_queries():
    bad, ok = lib.FSRGEMM_ERR_INVALID_ARG, lib.FSRGEMM_OK
    assert lib.fsrgemm_tile_count_f32() == 17 and lib.fsrgemm_tile_count_bf16() == 11
    f = lambda tile, s, ws=None, wsb=0, M=64, N=64, K=4096: lib.gemm_f32_cfg(tile, s, 0, 0, M, N, K, P, K, P, N, P, N, ws, wsb, 0)
    assert f(-1, 1) == bad and f(17, 1) == bad and f(0, 0) == bad and f(0, 65) == bad
    assert f(3, 1) == bad and f(3, 1, K=0, M=1) == bad                          # the vector kernels need M or N = 1 and K > 0
    assert f(2, 4) == bad and f(2, 4, P, 4 * 64 * 64 * 4 - 1) == bad            # a split without / with too small a workspace
    assert f(2, 4, P + 2, 1 << 20) == bad                                      # misaligned workspace
    assert f(2, 2, P, 1 << 30, M=2048, N=2048) == bad                          # partial products beyond 16 MiB
    assert f(2, 8, P, 1 << 24, K=100) == bad                                   # more slices than K-tiles (7)
    assert f(2, 1, None, 8) == bad and f(2, 1, P, -1) == bad
    assert lib.gemm_f32_cfg(1, 1, 0, 0, 0, 64, 64, None, 64, P, 64, None, 64, None, 0, 0) == ok      # empty: nothing to launch
    assert lib.gemm_f32_cfg(1, 1, 0, 0, 8, 8, 8, P, 7, P, 8, P, 8, None, 0, 0) == bad                # the usual argument checks
    g = lambda tile, s, M, N, K, a=P, lda=None, ws=None, wsb=0: lib.gemm_bf16_cfg(tile, s, 0, 1, M, N, K, a, lda or K, P, K, P, N, ws, wsb, 0)
    # the direct-to-LDS candidate is rejected where its kernel's conditions fail, never replaced
    assert g(0, 1, 255, 512, 512) == bad and g(0, 1, 512, 512, 100) == bad and g(0, 1, 512, 512, 56) == bad and g(0, 1, 512, 512, 512, a=P + 2) == bad
    assert g(0, 1, 512, 512, 512, lda=516) == bad and g(0, 2, 512, 512, 512) == bad and g(0, 2, 512, 512, 64, ws=P, wsb=1 << 24) == bad
    assert g(0, 4, 512, 512, 320, ws=P, wsb=1 << 24) == bad            # 5 K-tiles of 64 in slices of 2: the fourth slice would be empty
    assert g(4, 1, 512, 512, 512) == bad and g(5, 1, 1, 512, 512) == bad and g(1, 1, 0, 512, 512) == ok     # candidate 4: vector shapes only
    # names of forced candidates; None where the forced call would reject the candidate
    qc, qh = lib.fsrgemm_kernel_for_f32_cfg, lib.fsrgemm_kernel_for_bf16_cfg
    assert qc(0, 0, 0, 10, 10, 10, P, 10, P, 10, P, 10) == "gemm_f32_kernel<4, 2, 2, 2, 0, 1>"        # the largest tile on a tiny unaligned problem
    assert qc(3, 0, 0, 17, 17, 10, P, 10, P, 17, P, 17) is None and qc(14, 0, 0, 1, 10, 10, P, 10, P, 10, P, 10) is None
    assert qc(3, 0, 0, 1, 16, 16, P, 16, P, 16, P, 16) == "gemv_cols_f32_kernel<true>"
    assert qh(0, 0, 1, 520, 392, 128, P, 128, P, 128, P, 392) == "gemm_bf16_main_kernel<8, 8, 0, 0>"
    assert qh(0, 0, 1, 520, 392, 100, P, 104, P, 104, P, 392) is None and qh(4, 0, 1, 520, 392, 128, P, 128, P, 128, P, 392) is None
    assert qh(1, 1, 0, 8, 8, 8, P, 8, P, 8, P, 8) == "gemm_bf16_kernel<4, 1, 1, 1, 1>"
    # candidate 4: small results of long sums; its slices are workgroups, each with a partial result in the workspace
    sk = lambda M, N, K, s, ws=P, wsb=1 << 20: lib.gemm_f32_cfg(4, s, 1, 0, M, N, K, P, M, P, N, P, N, ws, wsb, 0)
    assert sk(17, 4, 4096, 4) == bad and sk(12, 16, 4096, 4) == bad and sk(64, 64, 4096, 4) == bad      # no register block that large
    assert sk(10, 10, 4096, 0) == bad and sk(10, 10, 4096, 257) == bad and sk(10, 10, 8, 9) == bad       # parts: 1..256, at most K
    assert sk(10, 10, 4096, 1, None, 0) == bad and sk(10, 10, 4096, 4, P, 4 * 100 * 4 - 1) == bad        # always needs its workspace
    assert sk(0, 10, 4096, 4) == ok
    assert qc(4, 1, 0, 10, 10, 1 << 20, P, 10, P, 10, P, 10) == "gemm_f32_skinny_kernel<12, 12, true, true>"
    assert qc(4, 1, 0, 10, 1, 1 << 20, P, 10, P, 1, P, 1) == "gemm_f32_skinny_kernel<12, 4, true, false>"
    assert qc(4, 1, 0, 16, 8, 64, P, 16, P, 8, P, 8) == "gemm_f32_skinny_kernel<16, 8, true, false>" and qc(4, 1, 0, 16, 9, 64, P, 16, P, 9, P, 9) is None
    assert qc(4, 1, 0, 10, 10, 1 << 20, P, 10, P + 64, 10, P, 10) == "gemm_f32_skinny_kernel<12, 12, true, false>"      # two different matrices
    assert qc(4, 1, 0, 9, 8, 64, P, 9, P, 8, P, 8) == "gemm_f32_skinny_kernel<12, 8, false, false>"            # odd leading dimension
    # an odd M is read element by element even where rows start 8-byte aligned: its last pair would reach into the padding
    assert qc(4, 1, 0, 9, 8, 64, P, 10, P, 8, P, 8) == "gemm_f32_skinny_kernel<12, 8, false, false>"
    assert qc(4, 1, 0, 10, 8, 64, P, 10, P, 8, P, 8) == "gemm_f32_skinny_kernel<12, 8, true, false>"
    assert qc(4, 0, 0, 1, 8, 64, P, 64, P, 8, P, 8) == "gemm_f32_skinny_kernel<4, 8, false, false>"    # a row vector is tall with leading dimension 1
    assert qc(4, 0, 0, 16, 8, 64, P, 64, P, 8, P, 8) is None                    # only for operands stored with k as the row index
    assert lib.gemm_f32_cfg(4, 4, 0, 0, 10, 10, 4096, P, 4096, P, 10, P, 10, P, 1 << 20, 0) == bad
    assert sk(10, 10, 1 << 30, 1, P, 1 << 20) == bad                            # one piece that long does not fit 32-bit lane offsets
    # the dispatcher takes it for such shapes when the call brings a workspace: the normal equations of least squares
    pfw = lambda M, N, K: lib.fsrgemm_plan_f32(1, 0, M, N, K, P, M, P, N, True)
    assert pfw(10, 10, 1 << 22) == (4, 256) and pfw(10, 1, 1 << 14) == (4, 64) and pfw(10, 10, 4095)[0] != 4
    assert lib.fsrgemm_plan_f32(1, 0, 10, 10, 1 << 22, P, 10, P, 10, False) == (3, 1)             # ten columns of a transposed X: the streaming kernel
    assert lib.gemm_f32_workspace_bytes(1, 0, 10, 10, 1 << 22) == 256 * 100 * 4 and lib.gemm_f32_workspace_bytes(1, 0, 10, 1, 4096) == 16 * 10 * 4
    # candidates 5..13: the direct-to-LDS kernel with tiles 256 x 256, 192 x 256, 128 x 256, 256 x 128, 192 x 128, 128 x 128,
    # 256 x 192, 192 x 192, 128 x 192;
    # rejected where its conditions fail, never replaced; K slices only of whole K-tiles of 32, with a workspace for them
    mk = lambda M, N, K, ta=0, tb=0, a=P, lda=None, s=1, ws=None, wsb=0: lib.gemm_f32_cfg(
        5, s, ta, tb, M, N, K, a, lda or (M if ta else K), P, K if tb else N, P, N, ws, wsb, 0)
    assert mk(255, 512, 512) == bad and mk(512, 255, 512) == bad and mk(512, 512, 50) == bad and mk(512, 512, 28) == bad and mk(512, 512, 0) == bad
    assert mk(512, 512, 512, a=P + 4) == bad and mk(512, 512, 512, lda=514) == bad and mk(512, 512, 512, s=2) == bad
    assert mk(512, 512, 512, s=2, ws=P, wsb=2 * 512 * 512 * 4 - 1) == bad and mk(512, 512, 32, s=2, ws=P, wsb=1 << 24) == bad
    assert mk(512, 512, 160, s=4, ws=P, wsb=1 << 24) == bad         # 5 K-tiles in slices of 2: the fourth slice would be empty
    assert mk(510, 512, 512, ta=1) == bad and mk(512, 510, 512) == bad            # a shifted last tile would start off a 16-byte piece
    assert mk(0, 512, 512) == ok and mk(512, 512, 512, ws=None, wsb=8) == bad
    assert qc(5, 0, 0, 510, 512, 64, P, 64, P, 512, P, 512) == "gemm_f32_main_kernel<4, 4, 0, 1>"
    assert qc(5, 1, 1, 512, 510, 64, P, 512, P, 64, P, 510) == "gemm_f32_main_kernel<4, 4, 1, 0>"
    assert qc(6, 0, 0, 192, 256, 64, P, 64, P, 256, P, 256) == "gemm_f32_main_kernel<3, 4, 0, 1>" and qc(6, 0, 0, 191, 256, 64, P, 64, P, 256, P, 256) is None
    assert qc(6, 1, 0, 192, 256, 64, P, 192, P, 256, P, 256) == "gemm_f32_main_kernel<3, 4, 1, 1>"
    assert qc(12, 0, 0, 192, 192, 64, P, 64, P, 192, P, 192) == "gemm_f32_main_kernel<3, 3, 0, 1>" and qc(13, 0, 0, 128, 191, 64, P, 64, P, 192, P, 191) is None
    assert qc(10, 1, 0, 128, 128, 32, P, 128, P, 128, P, 128) == "gemm_f32_main_kernel<2, 2, 1, 1>" and qc(10, 0, 0, 128, 127, 32, P, 32, P, 128, P, 127) is None
    assert qc(9, 0, 1, 200, 130, 96, P, 96, P, 96, P, 130) == "gemm_f32_main_kernel<3, 2, 0, 0>"
    assert qc(5, 0, 0, 512, 512, 48, P, 48, P, 512, P, 512) == "gemm_f32_main_kernel<4, 4, 0, 1>" and qc(5, 0, 0, 512, 512, 28, P, 28, P, 512, P, 512) is None
    assert lib.fsrgemm_kernel_for_f32(4096, 4096, 4096, P, 4096, P, 4096, P, 4096) == "gemm_f32_main_kernel<4, 4, 0, 1>"
    # plan queries: the rules, in the terms of the forced calls
    pf, pb = lib.fsrgemm_plan_f32, lib.fsrgemm_plan_bf16
    assert pf(0, 0, 4096, 4096, 4096, P, 4096, P, 4096) == (5, 1) and pf(0, 0, 200, 200, 200, P, 200, P, 200) == (14, 1) and pf(0, 0, 200, 200, 202, P, 202, P, 200) == (2, 1)
    assert pf(0, 0, 64, 64, 1 << 20, P, 1 << 20, P, 64, True) == (14, 64)
    assert pf(0, 0, 64, 64, 1 << 20, P, 1 << 20, P, 64, False) == (14, 1)
    assert pb(0, 1, 8192, 8192, 8192, P, 8192, P, 8192) == (0, 1)
    assert pb(0, 1, 8192, 8192, 8200, P, 8200, P, 8200) == (0, 1)              # a rest of K in whole 16-byte pieces: still the direct-to-LDS kernel
    assert pb(0, 1, 8192, 8192, 8196, P, 8200, P, 8200) == (1, 1)              # otherwise the general kernel of that tile
    assert pb(0, 1, 6144, 6144, 6144, P, 6144, P, 6144) == (7, 1) and pb(0, 0, 6144, 6144, 6144, P, 6144, P, 6144) == (7, 1)   # 256 x 192, in every storage order
    # the rules (two bands); a row of the selection table (one launch of 64 x 64 tiles)
    assert lib.fsrgemm_bands_f32(0, 0, 2560, 2560, 2560, P, 2560, P, 2560, False, True)[0] == 1 and lib.fsrgemm_bands_f32(0, 0, 2560, 2560, 2560, P, 2560, P, 2560)[0] == 0
    assert pb(0, 1, 512, 512, 512, P, 512, P, 512, True) == (3, 1) and pb(0, 1, 512, 512, 4096, P, 4096, P, 4096, True) == (3, 4)       # bf16: no split of a short K
    # between 64 and 127 tiles of 256 x 256: a larger shape in one round, or 128 x 128 tiles, by the modelled times
    assert pb(0, 1, 2560, 2560, 2560, P, 2560, P, 2560) == (6, 1) and pb(1, 0, 2048, 2560, 8192, P, 2048, P, 2560) == (6, 1)
    assert pb(0, 1, 2048, 2048, 2048, P, 2048, P, 2048) == (10, 1) and pb(0, 1, 2048, 2048, 512, P, 512, P, 512) == (10, 1)
    for ta, tb in ((0, 1), (0, 0), (1, 1), (1, 0)):      # one round of 256 tiles of 192 x 192 rather than 192 of 192 x 256
        assert pb(ta, tb, 3072, 3072, 3072, P, 3072, P, 3072) == (8, 1)
    assert pb(0, 1, 3072, 4096, 4096, P, 4096, P, 4096) == (5, 1)                    # 256 tiles of 192 x 256 rather than 192 of 256 x 256
    assert pb(0, 1, 300, 300, 300, P, 300, P, 300) == (3, 1)
    assert pf(0, 0, -1, 1, 1, P, 1, P, 1) is None
    # a vector on one side: the streaming kernels (candidate 3), split along K only where the output alone gives few workgroups
    assert pf(0, 0, 1, 4096, 4096, P, 4096, P, 4096) == (3, 1) and pf(0, 0, 4096, 1, 4096, P, 4096, P, 1) == (3, 1)
    assert pf(0, 0, 1, 4096, 4096, P, 4096, P, 4096, True) == (3, 2)            # 128 workgroups of 32 columns -> 2 slices
    assert pf(0, 0, 4096, 1, 4096, P, 4096, P, 1, True) == (3, 1)               # 1024 workgroups of 4 rows already
    assert pf(0, 0, 1, 1024, 1024, P, 1024, P, 1024, True) == (3, 1)            # too short to pay for a second launch
    assert pf(0, 0, 1, 17, 1 << 20, P, 1 << 20, P, 17, True) == (3, 64) and pf(0, 0, 1, 4096, 0, P, 1, P, 4096) == (2, 1)
    # a dot product in any storage order (a vector is tall either way), a row times a tall matrix: the small-result kernel
    assert pf(0, 0, 1, 1, 1 << 20, P, 1 << 20, P, 1, True) == pf(1, 1, 1, 1, 1 << 20, P, 1, P, 1 << 20, True) == (4, 256)
    assert pf(0, 0, 1, 10, 1 << 20, P, 1 << 20, P, 10, True) == (4, 256) and pf(0, 1, 1, 10, 1 << 20, P, 1 << 20, P, 1 << 20, True)[0] == 3
    assert pf(0, 0, 1, 64, (1 << 30) + 16, P, (1 << 30) + 16, P, 64)[0] == 2        # beyond the vector kernels' 32-bit k arithmetic
    qv = lib.fsrgemm_kernel_for_f32_ex
    assert qv(0, 0, 4096, 1, 4096, P, 4096, P, 1, P, 1) == "gemv_rows_f32_kernel<true>"
    assert qv(0, 0, 1, 4096, 4096, P, 4096, P, 4096, P, 4096) == "gemv_cols_f32_kernel<true>"
    assert qv(0, 1, 1, 4096, 4096, P, 4096, P, 4096, P, 4096) == "gemv_rows_f32_kernel<true>"
    assert qv(1, 0, 4096, 1, 4096, P, 4096, P, 1, P, 1) == "gemv_cols_f32_kernel<true>"
    assert qv(0, 0, 4096, 1, 4095, P, 4095, P, 1, P, 1) == "gemv_rows_f32_kernel<false>"        # rows not 16-byte aligned
    assert qv(0, 0, 1, 4096, 4096, P, 4096, P + 4, 4096, P, 4096) == "gemv_cols_f32_kernel<false>"
    # the workspace query and the plan agree
    for M, N, K in ((1, 4096, 4096), (64, 64, 4097), (256, 256, 65536), (4096, 4096, 4096)):
        s = pf(0, 0, M, N, K, P, K, P, N, True)[1]
        assert lib.gemm_f32_workspace_bytes(0, 0, M, N, K) == (s * M * N * 4 if s > 1 else 0)


def test_dispatcher_only_plans_candidates_that_the_forced_calls_accept():
    # a seeded sweep over shapes, storage orders, paddings and alignments: whatever the dispatcher plans must be a
    # candidate its own forced entry point would run, within the documented limits
    import random

    rng = random.Random(20)
    dims = [1, 2, 7, 10, 16, 17, 63, 64, 65, 255, 256, 257, 1000, 4096, 4097, 8192, 1 << 16, 1 << 20, (1 << 22) + 3]
    for case in range(4000):
        kind = rng.choice(("f32", "bf16"))
        ta, tb = rng.randint(0, 1), rng.randint(0, 1)
        M, N, K = rng.choice(dims), rng.choice(dims), rng.choice(dims)
        if M * N > 1 << 28:
            N = 16
        lda, ldb = (M if ta else K) + rng.choice((0, 0, 1, 3, 4, 8)), (K if tb else N) + rng.choice((0, 0, 1, 3, 4, 8))
        esize = 4 if kind == "f32" else 2
        a, b = P + esize * rng.choice((0, 0, 1, 2, 4)), P + esize * rng.choice((0, 0, 1, 2, 4))
        plan, named = ((lib.fsrgemm_plan_f32, lib.fsrgemm_kernel_for_f32_cfg) if kind == "f32" else
                       (lib.fsrgemm_plan_bf16, lib.fsrgemm_kernel_for_bf16_cfg))
        count = lib.fsrgemm_tile_count_f32() if kind == "f32" else lib.fsrgemm_tile_count_bf16()
        query = lib.gemm_f32_workspace_bytes if kind == "f32" else lib.gemm_bf16_workspace_bytes
        for with_ws in (False, True):
            got = plan(ta, tb, M, N, K, a, lda, b, ldb, with_ws)
            assert got is not None, (kind, ta, tb, M, N, K)
            tile, slices = got
            ctx = (kind, ta, tb, M, N, K, lda, ldb, with_ws, tile, slices)
            small_result = kind == "f32" and tile == 4
            assert 0 <= tile < count and 1 <= slices <= (256 if small_result else 64), ctx
            assert named(tile, ta, tb, M, N, K, a, lda, b, ldb, P, N) is not None, ctx
            if not with_ws:
                assert slices == 1 and not small_result, ctx
            elif slices > 1 or small_result:
                assert slices * M * N * 4 <= 16 << 20 and slices <= K, ctx
                assert query(ta, tb, M, N, K) >= slices * M * N * 4, ctx         # (the query covers either alignment's plan)
            else:
                pass            # (a plan for otherwise aligned operands may be split: the query names that need)
            if kind == "bf16" and (tile == 0 or 5 <= tile <= 9):   # of the bf16 direct-to-LDS shapes only 128x128 takes K slices
                assert slices == 1, ctx


def _slices_fit(K, slices, k_tile):
    # whole K-tiles per slice, the last slice takes the rest and must hold at least one whole K-tile
    per = ((K + k_tile - 1) // k_tile + slices - 1) // slices * k_tile
    return (slices - 1) * per + k_tile <= K


def test_slice_plans_for_problems_of_few_tiles():
    # the shapes the slice planners are for (sides of 128 to 3072, K up to 65536, aligned and padded operands in every
    # storage order): a split plan on a direct-to-LDS tile has slices of whole K-tiles with a last slice that is not
    # empty, fits the workspace the query names (at most 16 MiB), and is never slower by the planner's own rule than
    # no split at all would need to be: it is only taken with a workspace
    import random

    rng = random.Random(21)
    sides = [128, 192, 256, 320, 384, 512, 640, 768, 1000, 1024, 1536, 2048, 2560, 3072]
    depths = [64, 256, 512, 1000, 1024, 2048, 3072, 4096, 8192, 16384, 65536]
    seen = {"f32": 0, "bf16": 0}
    for case in range(3000):
        kind = rng.choice(("f32", "bf16"))
        ta, tb = rng.randint(0, 1), rng.randint(0, 1)
        M, N, K = rng.choice(sides), rng.choice(sides), rng.choice(depths)
        pad = 4 if kind == "f32" else 8                      # keeps 16-byte rows
        lda, ldb = (M if ta else K) + rng.choice((0, 0, pad)), (K if tb else N) + rng.choice((0, 0, pad))
        plan, named = ((lib.fsrgemm_plan_f32, lib.fsrgemm_kernel_for_f32_cfg) if kind == "f32" else
                       (lib.fsrgemm_plan_bf16, lib.fsrgemm_kernel_for_bf16_cfg))
        query = lib.gemm_f32_workspace_bytes if kind == "f32" else lib.gemm_bf16_workspace_bytes
        assert plan(ta, tb, M, N, K, P, lda, P, ldb, False)[1] == 1
        tile, slices = plan(ta, tb, M, N, K, P, lda, P, ldb, True)
        ctx = (kind, ta, tb, M, N, K, lda, ldb, tile, slices)
        name = named(tile, ta, tb, M, N, K, P, lda, P, ldb, P, N)
        assert name is not None, ctx
        if slices == 1:
            continue
        assert slices * M * N * 4 <= query(ta, tb, M, N, K) <= 16 << 20, ctx
        if "main" in name:                                   # a direct-to-LDS tile: slices of whole K-tiles
            seen[kind] += 1
            k_tile = 32 if kind == "f32" else 64
            assert _slices_fit(K, slices, k_tile), ctx
            per = ((K + k_tile - 1) // k_tile + slices - 1) // slices * k_tile
            assert per >= (256 if kind == "f32" else 512), ctx              # the planners' shortest slices
    assert seen["f32"] > 50 and seen["bf16"] > 50, seen


def test_tuned_table_rows_are_well_formed():
    # every row of the table names a candidate the forced entry point would accept for its problem
    import os
    import re

    path = os.path.join(os.path.dirname(lib.library_path()), "csrc", "tuned_table.inc")
    rows = [tuple(int(x) for x in m.groups()) for m in re.finditer(r"^\s*\{(\d+), (\d+), (\d+), (\d+), (\d+), (\d+), (\d+), (\d+), (\d+)\},", open(path).read(), re.M)]
    assert len(set(r[:7] for r in rows)) == len(rows)                  # one row per (problem, workspace) pair
    for kind, ta, tb, M, N, K, ws, tile, slices in rows:
        assert kind in (0, 1) and ta in (0, 1) and tb in (0, 1) and ws in (0, 1) and M > 0 and N > 0 and K > 0
        assert 0 <= tile < (lib.fsrgemm_tile_count_bf16() if kind else lib.fsrgemm_tile_count_f32())
        assert 1 <= slices <= 256 and (ws == 1 or slices == 1) and slices * M * N * 4 <= (16 << 20 if slices > 1 else 1 << 62)
        assert ws == 1 or not (kind == 0 and tile == 4)                   # the small-result kernel cannot serve a call without a workspace
        plan = (lib.fsrgemm_plan_bf16 if kind else lib.fsrgemm_plan_f32)(ta, tb, M, N, K, P, M if ta else K, P, K if tb else N, bool(ws))
        assert plan == (tile, slices), (plan, (tile, slices))
        rules = (lib.fsrgemm_plan_bf16 if kind else lib.fsrgemm_plan_f32)(ta, tb, M, N, K, P, M if ta else K, P, K if tb else N, bool(ws), True)
        bands = (lib.fsrgemm_bands_bf16 if kind else lib.fsrgemm_bands_f32)(ta, tb, M, N, K, P, M if ta else K, P, K if tb else N, bool(ws), True)
        assert rules != plan or bands[0] != 0                             # a row that repeats the rules is never written (one launch
                                                                          # of the first band's tile is not the rules' two bands)
        assert (lib.fsrgemm_bands_bf16 if kind else lib.fsrgemm_bands_f32)(ta, tb, M, N, K, P, M if ta else K, P, K if tb else N, bool(ws))[0] == 0    # a row is one launch
        if ws:
            q = lib.gemm_bf16_workspace_bytes if kind else lib.gemm_f32_workspace_bytes
            assert q(ta, tb, M, N, K) == (slices * M * N * 4 if slices > 1 else 0)


def test_header_is_plain_c_and_declares_what_the_binding_loads(tmp_path):
    # the boundary is a C ABI: the header must compile as C99 on its own, and every function it declares must be one
    # the binding knows (and the other way round)
    import os
    import re
    import subprocess

    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    header = os.path.join(root, "include", "fsrgemm.h")
    src = tmp_path / "use.c"
    src.write_text('#include "fsrgemm.h"\nint main(void) { return gemm_f32(0, 0, 0, 0, 1, 0, 1, 0, 1, 0) == FSRGEMM_OK && fsrgemm_version() > 0 ? 0 : 1; }\n')
    subprocess.check_call(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-I", os.path.dirname(header), "-fsyntax-only", str(src)])
    text = re.sub(r"/\*.*?\*/", "", open(header).read(), flags=re.S)
    declared = set(re.findall(r"\b(\w+)\s*\(", text)) - {"defined"}
    assert declared == set(lib.EXPORTS), declared ^ set(lib.EXPORTS)


def test_transpose_argument_checks():
    f, bad = lib.transpose_f32, lib.FSRGEMM_ERR_INVALID_ARG
    assert f(-1, 4, P, 4, P, 4, 0) == bad and f(4, -1, P, 4, P, 4, 0) == bad
    assert f(4, 8, P, 7, P, 4, 0) == bad and f(4, 8, P, 8, P, 3, 0) == bad        # lda < cols, ldt < rows
    assert f(4, 8, None, 8, P, 4, 0) == bad and f(4, 8, P, 8, None, 4, 0) == bad
    assert f(2 ** 31, 1, P, 1, P, 2 ** 31, 0) == bad
    assert f(0, 8, None, 8, None, 0, 0) == lib.FSRGEMM_OK and f(4, 0, None, 0, None, 4, 0) == lib.FSRGEMM_OK
    # <tile rows, tile columns, bounds-checked>: wide tiles from 128 columns on, checks only below 64 rows or columns
    q = lib.fsrgemm_kernel_for_transpose_f32
    assert q(4096, 4096, P, 4096, P, 4096) == "transpose_f32_kernel<64, 128, false>"
    assert q(2048, 2176, P, 2176, P, 2048) == "transpose_f32_kernel<64, 128, false>"
    # up to 512 tiles of 64 x 128 (two to a compute unit): 32 x 64 tiles
    assert q(64, 128, P, 128, P, 64) == q(2048, 2048, P, 2048, P, 2048) == q(5000, 127, P, 127, P, 5000) == "transpose_f32_kernel<32, 64, false>"
    assert q(40000, 127, P, 127, P, 40000) == "transpose_f32_kernel<64, 64, false>"
    assert q(63, 4096, P, 4096, P, 63) == q(4096, 63, P, 63, P, 4096) == "transpose_f32_kernel<64, 64, true>"
    assert q(0, 8, None, 8, None, 0) == "none" and q(4, 8, P, 7, P, 4) is None and q(4, 8, None, 8, P, 4) is None


def test_build_refuses_spills_in_hand_scheduled_kernels():
    # the build parses the compiler's resource-usage remarks for the kernels that issue loads from
    # inline assembly; any spill (or missing remarks) must stop it
    from paper_2506_09092_amd import build

    ok = ("x.hip:1:1: remark: Function Name: k [-Rpass-analysis=kernel-resource-usage]\n"
          "x.hip:1:1: remark:     ScratchSize [bytes/lane]: 0 [-Rpass-analysis=kernel-resource-usage]\n"
          "x.hip:1:1: remark:     SGPRs Spill: 0 [-Rpass-analysis=kernel-resource-usage]\n"
          "x.hip:1:1: remark:     VGPRs Spill: 0 [-Rpass-analysis=kernel-resource-usage]\n")
    assert "no spills" in build.check_no_spills("x.hip", ok)
    for field in ("SGPRs Spill: 0", "VGPRs Spill: 0", "ScratchSize [bytes/lane]: 0"):
        with pytest.raises(RuntimeError):
            build.check_no_spills("x.hip", ok.replace(field, field[:-1] + "4"))
    with pytest.raises(RuntimeError):
        build.check_no_spills("x.hip", "")
    # the other kernels only have to stay out of scratch memory
    assert "no scratch" in build.check_no_spills("x.hip", ok.replace("VGPRs Spill: 0", "VGPRs Spill: 9"), scratch_only=True)
    with pytest.raises(RuntimeError):
        build.check_no_spills("x.hip", ok.replace("ScratchSize [bytes/lane]: 0", "ScratchSize [bytes/lane]: 64"), scratch_only=True)
    assert "gemm_bf16_main.hip" in build.NO_SPILL_SOURCES


def test_f32_direct_to_lds_kernel_is_not_planned_beyond_its_32_bit_lane_offsets():
    # the kernel adds a 32-bit byte offset per lane (up to 7 rows and 28 elements along k, up to 2 k-rows along m / n)
    # to a uniform base: leading dimensions of 2^24 elements and more take the general tiles in their checked mode
    q, qx = lib.fsrgemm_kernel_for_f32, lib.fsrgemm_kernel_for_f32_ex
    n, big = 4096, 1 << 24
    assert q(n, n, n, P, big - 4, P, n, P, n) == "gemm_f32_main_kernel<4, 4, 0, 1>"
    for lda, ldb in ((big, n), (n, big), (160000000, n), (1 << 30, n), (n, 1 << 30)):
        name = q(n, n, n, P, lda, P, ldb, P, n)
        assert name.startswith("gemm_f32_kernel<") and name.split(", ")[3] == "1", (lda, ldb, name)      # load mode 1: checked
    assert qx(1, 0, n, n, n, P, big, P, n, P, n).startswith("gemm_f32_kernel<")
    assert qx(1, 1, n, n, n, P, n, P, big, P, n).startswith("gemm_f32_kernel<")
    # forced: rejected, not replaced
    for tile in range(5, 17):       # (rejected before any launch: the addresses are fake)
        assert lib.gemm_f32_cfg(tile, 1, 0, 0, n, n, n, P, big, P, n, P, n, None, 0, 0) == lib.FSRGEMM_ERR_INVALID_ARG
        assert lib.fsrgemm_kernel_for_f32_cfg(tile, 0, 0, n, n, n, P, n, P, big, P, n) is None
    assert lib.fsrgemm_plan_f32(0, 0, n, n, n, P, big, P, n)[0] < 3


def test_small_result_kernel_is_planned_only_where_its_launcher_accepts_the_pieces():
    # normal equations with a widely padded X: 2^22 rows in 256 pieces are 16384 rows a piece, and 16384 * 40000
    # elements do not fit the kernel's 32-bit lane offsets -- the plan must fall back to another kernel in K slices, and
    # whatever it names must be what the forced entry point accepts for the same arguments
    bad = lib.FSRGEMM_ERR_INVALID_ARG
    K = 1 << 22
    assert lib.fsrgemm_plan_f32(1, 0, 10, 10, K, P, 10, P, 10, True) == (4, 256)
    for lda in (10, 1024, 32766, 32768, 40000, 1 << 20):
        tile, slices = lib.fsrgemm_plan_f32(1, 0, 10, 10, K, P, lda, P, 10, True)
        fits = (K // 256) * lda < 1 << 29
        assert (tile == 4) == fits, (lda, tile, slices)
        assert (lib.fsrgemm_kernel_for_f32_cfg(4, 1, 0, 10, 10, K, P, lda, P, 10, P, 10) is None) == (not fits)
        if not fits:        # (only rejected calls are made here: the addresses are fake)
            assert lib.gemm_f32_cfg(4, 256, 1, 0, 10, 10, K, P, lda, P, 10, P, 10, P, 256 * 100 * 4, 0) == bad
            assert tile == 3 and slices > 1             # (ten columns of a transposed X in aligned pieces: the streaming kernel)
    # the same on B's side, and for a dot product of two strided vectors
    assert lib.fsrgemm_plan_f32(1, 0, 10, 10, K, P, 10, P, 40000, True) == (3, 64)
    assert lib.fsrgemm_plan_f32(1, 1, 1, 1, K, P, 1, P, K, True) == (4, 256)


def test_mfma_ceiling_arguments():
    # the register-only MFMA loop of the profiler leg: argument errors come before any HIP call
    bad = lib.FSRGEMM_ERR_INVALID_ARG
    f = lambda kind=1, passes=10, ops=P, sink=P, groups=256: lib.fsrgemm_mfma_ceiling(kind, passes, ops, sink, groups)[0]
    assert f(kind=2) == bad and f(kind=-1) == bad and f(passes=0) == bad and f(passes=(1 << 24) + 1) == bad
    assert f(groups=0) == bad and f(groups=(1 << 16) + 1) == bad and f(ops=None) == bad and f(sink=None) == bad and f(ops=P + 4) == bad
    assert lib.fsrgemm_kernel_for_mfma_ceiling(0) == "mfma_ceiling_kernel<0>" and lib.fsrgemm_kernel_for_mfma_ceiling(1) == "mfma_ceiling_kernel<1>"
    assert lib.fsrgemm_kernel_for_mfma_ceiling(2) is None


def _band_problems(kind, ta, tb, M, N, K, a, lda, b, ldb, dim, at):
    """The two products a cut at row (dim 1) or column (dim 2) `at` of C leaves: (M, N, A, B) of each band."""
    esize = 4 if kind == "f32" else 2
    if dim == 1:
        a2 = a + esize * (at if ta else at * lda)
        return (at, N, a, b), (M - at, N, a2, b)
    b2 = b + esize * (at * ldb if tb else at)
    return (M, at, a, b), (M, N - at, a, b2)


def test_two_band_plans():
    # where no tile shape fills whole rounds of the 256 compute units the dispatcher cuts C once and gives each band its own
    # shape: 5120^2 as rows 0..1023 in 64 x 64 tiles (1280 = five rounds) + the rest in 128 x 128 tiles (1280 = five rounds of
    # a tile of four times the work) instead of 729 tiles of 192 x 192 (2.85 -> 3 rounds); fp32 candidates: 5 + shape
    bf = lambda M, N, K, a=P, **kw: lib.fsrgemm_bands_f32(0, 0, M, N, K, a, K, P, N, **kw)
    assert bf(5120, 5120, 2048) == (1, 1024, 14, 10)
    assert lib.fsrgemm_plan_f32(0, 0, 5120, 5120, 2048, P, 2048, P, 5120) == (14, 1)            # the first band's tile
    name = lib.fsrgemm_kernel_for_f32(5120, 5120, 2048, P, 2048, P, 5120, P, 5120)
    assert name == "gemm_f32_main_kernel<1, 1, 0, 1> + gemm_f32_main_kernel<2, 2, 0, 1> (rows from 1024)"
    # whole rounds in one launch stay one launch; so do misaligned operands (no direct-to-LDS kernel), table rows and splits
    assert bf(4096, 4096, 4096) == (0, 0, 5, 5) and bf(6144, 6144, 2048) == (0, 0, 9, 9) and bf(1024, 1024, 1024)[0] == 0
    assert bf(5120, 5120, 2048, a=P + 4)[0] == 0
    assert lib.fsrgemm_bands_f32(0, 0, 512, 512, 65536, P, 65536, P, 512, with_workspace=True)[0] == 0
    # bf16: 7168^3 in 256 x 192 tiles is 4.16 rounds
    got = lib.fsrgemm_bands_bf16(0, 1, 7168, 7168, 7168, P, 7168, P, 7168)
    assert got[0] in (1, 2) and got[1] % 64 == 0 and 0 < got[1] < 7168
    assert lib.fsrgemm_bands_bf16(0, 1, 8192, 8192, 8192, P, 8192, P, 8192) == (0, 0, 0, 0)
    # argument errors
    assert lib.fsrgemm_bands_f32(0, 0, -1, 8, 8, P, 8, P, 8) is None and lib.fsrgemm_bands_bf16(0, 1, 8, 8, 1 << 31, P, 8, P, 8) is None


def test_each_band_is_a_problem_the_forced_call_accepts():
    # over a seeded sweep of large problems in every storage order, with padded leading dimensions and ragged extents: a cut is
    # a multiple of 64 strictly inside the matrix, and each band, on its shifted operands, is a problem the forced entry point of
    # its tile accepts (same alignment rules, extents at least one tile)
    import random

    rng = random.Random(21)
    cut = 0
    for case in range(1500):
        kind = rng.choice(("f32", "bf16"))
        ta, tb = rng.randint(0, 1), rng.randint(0, 1)
        M, N = rng.choice((2048, 2560, 3000, 3584, 4000, 4608, 5000, 5120, 7168, 9000, 11111, 12288)), rng.choice((2048, 2304, 3584, 4608, 5120, 6656, 7000, 7168, 10000))
        M, N = M - M % 8, N - N % 8
        K = rng.choice((64, 128, 2048, 4104, 8192))
        pad = 8 * rng.choice((0, 0, 1, 5))
        lda, ldb = (M if ta else K) + pad, (K if tb else N) + pad
        bands, named = ((lib.fsrgemm_bands_f32, lib.fsrgemm_kernel_for_f32_cfg) if kind == "f32" else (lib.fsrgemm_bands_bf16, lib.fsrgemm_kernel_for_bf16_cfg))
        plan = lib.fsrgemm_plan_f32 if kind == "f32" else lib.fsrgemm_plan_bf16
        got = bands(ta, tb, M, N, K, P, lda, P, ldb)
        assert got is not None
        dim, at, first, second = got
        ctx = (kind, ta, tb, M, N, K, lda, ldb, got)
        assert plan(ta, tb, M, N, K, P, lda, P, ldb) == (first, 1), ctx
        if dim == 0:
            assert at == 0 and first == second, ctx
            continue
        cut += 1
        assert dim in (1, 2) and at % 64 == 0 and 0 < at < (M if dim == 1 else N), ctx
        for tile, (m, n, a, b) in zip((first, second), _band_problems(kind, ta, tb, M, N, K, P, lda, P, ldb, dim, at)):
            name = named(tile, ta, tb, m, n, K, a, lda, b, ldb, P, N)
            assert name is not None and "main_kernel" in name, ctx
    assert cut > 100        # the sweep does exercise the two-band path
