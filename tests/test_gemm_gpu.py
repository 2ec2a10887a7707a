"""Parity of the HIP path against the CPU oracle, called through the C ABI.

Gate: e = max_ij |got - ref| / S_ij with S = |A||B| (fp64, from the oracle);
e <= 1e-5 for fp32, e <= 1e-2 for bf16 inputs; bit-exact on small-integer
operands, where every summation order is exact.
"""
import math
import re
import sys

import numpy as np
import pytest

import oracle
from paper_2506_09092_amd import inputs
from tests.validator import one_entry_per_block

from paper_2506_09092_amd.harness import (run_bf16, run_bf16_ex, run_bf16_ws, run_cfg, run_f32, run_f32_ex, run_f32_ws,
                                          run_transpose)

pytestmark = pytest.mark.gpu
TOL_F32 = 1e-5
TOL_BF16 = 1e-2


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def check_f32(lib, A, B, tol=TOL_F32, **kw):
    got = run_f32(lib, A, B, **kw)
    ref, S = oracle.gemm(A, B)
    e = oracle.componentwise_error(got, ref, S)
    assert e <= tol, "componentwise error %.3e > %.1e" % (e, tol)
    return got, ref, e


def check_bf16(lib, A, Bt, tol=TOL_BF16, **kw):
    got = run_bf16(lib, A, Bt, **kw)
    ref, S = oracle.gemm(A, Bt.T)
    e = oracle.componentwise_error(got, ref, S)
    assert e <= tol, "componentwise error %.3e > %.1e" % (e, tol)
    return got, ref, e


def test_f32_256_uniform(gpu):
    say("fp32 256^3 uniform seed 0")
    check_f32(gpu, inputs.uniform_pm1(0, 1, 256, 256), inputs.uniform_pm1(0, 2, 256, 256), repeat=2)


def test_f32_256_integers_bit_exact(gpu):
    say("fp32 256^3 integers seed 0")
    A, B = inputs.small_ints(0, 3, 256, 256), inputs.small_ints(0, 4, 256, 256)
    got = run_f32(gpu, A, B)
    ref, _ = oracle.gemm(A, B)
    assert np.array_equal(got.astype(np.float64), ref)
    assert not np.any(np.signbit(got[got == 0]))


def test_f32_1024_uniform(gpu):
    say("fp32 1024^3 uniform seed 1")
    check_f32(gpu, inputs.uniform_pm1(1, 1, 1024, 1024), inputs.uniform_pm1(1, 2, 1024, 1024))


def test_f32_sweep_64_shapes(gpu):
    cases = inputs.sweep_cases(3, 64)
    failed = []
    for c in cases:
        say("sweep case %(index)d: M=%(M)d N=%(N)d K=%(K)d lda=%(lda)d ldb=%(ldb)d ldc=%(ldc)d off=%(offset)d" % c)
        A = inputs.uniform_pm1(3, 2 * c["index"] + 10, c["M"], c["K"])
        B = inputs.uniform_pm1(3, 2 * c["index"] + 11, c["K"], c["N"])
        got = run_f32(gpu, A, B, lda=c["lda"], ldb=c["ldb"], ldc=c["ldc"], offset=c["offset"], repeat=2)
        ref, S = oracle.gemm(A, B)
        e = oracle.componentwise_error(got, ref, S)
        if not e <= TOL_F32:
            failed.append((c["index"], e))
    assert not failed, failed


LAYOUTS = [(0, 1), (1, 0), (1, 1)]          # (transA, transB) beyond the plain row-major pair


def test_f32_transposed_storage_sweep(gpu):
    # the 64 sweep shapes again with A, B or both stored transposed; one oracle result per shape serves all three
    cases = inputs.sweep_cases(3, 64)
    failed = []
    for c in cases:
        M, N, K = c["M"], c["N"], c["K"]
        say("transposed sweep case %d: M=%d N=%d K=%d" % (c["index"], M, N, K))
        A = inputs.uniform_pm1(3, 2 * c["index"] + 10, M, K)
        B = inputs.uniform_pm1(3, 2 * c["index"] + 11, K, N)
        ref, S = oracle.gemm(A, B)
        pad_a, pad_b = c["lda"] - K, c["ldb"] - N          # the case's padding, applied to whichever extent is contiguous
        for ta, tb in LAYOUTS:
            lda, ldb = (M if ta else K) + pad_a, (K if tb else N) + pad_b
            got = run_f32_ex(gpu, ta, tb, A, B, lda=max(lda, 1), ldb=max(ldb, 1), ldc=c["ldc"], offset=c["offset"], repeat=2)
            e = oracle.componentwise_error(got, ref, S)
            if not e <= TOL_F32:
                failed.append((c["index"], ta, tb, e))
    assert not failed, failed


def test_bf16_sweep_64_shapes_every_storage_order(gpu):
    # the 64 sweep shapes (ragged, padded, offset by an element) with bf16 operands in the four storage orders; one
    # oracle result per shape serves all four.  Products of bf16 values are exact in fp32, so the error is that of fp32
    # accumulation and the fp32 bound holds as well as the bf16 one
    cases = inputs.sweep_cases(3, 64)
    failed = []
    for c in cases:
        M, N, K = c["M"], c["N"], c["K"]
        say("bf16 sweep case %d: M=%d N=%d K=%d" % (c["index"], M, N, K))
        A = inputs.bf16_normal_scaled(3, 2 * c["index"] + 10, M, K, 1 / math.sqrt(max(K, 1)))
        B = inputs.bf16_normal_scaled(3, 2 * c["index"] + 11, K, N, 1 / math.sqrt(max(K, 1)))
        ref, S = oracle.gemm(A, B)
        pad_a, pad_b = c["lda"] - K, c["ldb"] - N
        for ta, tb in [(0, 1)] + BF16_STORAGE:
            lda, ldb = (M if ta else K) + pad_a, (K if tb else N) + pad_b
            got = run_bf16_ex(gpu, ta, tb, A, B, lda=max(lda, 1), ldb=max(ldb, 1), ldc=c["ldc"], offset=c["offset"], repeat=2)
            e = oracle.componentwise_error(got, ref, S)
            if not e <= TOL_F32:
                failed.append((c["index"], ta, tb, e))
    assert not failed, failed


@pytest.mark.parametrize("ta,tb", LAYOUTS)
def test_f32_transposed_storage_tile_configs(gpu, ta, tb):
    # every tile configuration in its unchecked-vector mode, small K included, and integers bit for bit
    # (forced: the dispatcher gives most of these shapes to the direct-to-LDS kernel)
    for (M, N, K), tile, name in (((2048, 2048, 48), 1, "gemm_f32_kernel<2, 2, 3, 0, %d, %d>"),
                                  ((4096, 2048, 16), 0, "gemm_f32_kernel<4, 2, 2, 0, %d, %d>"),
                                  ((4096, 2048, 112), 0, "gemm_f32_kernel<4, 2, 2, 0, %d, %d>"),
                                  ((1024, 1024, 1024), 2, "gemm_f32_kernel<1, 1, 4, 0, %d, %d>")):
        say("transposed %d%d %dx%dx%d" % (ta, tb, M, N, K))
        lda, ldb = (M if ta else K), (K if tb else N)
        assert gpu.fsrgemm_kernel_for_f32_cfg(tile, ta, tb, M, N, K, 0x1000, lda, 0x1000, ldb, 0x1000, N) == name % (ta, 1 - tb)
        A, B = inputs.uniform_pm1(6, 1, M, K), inputs.uniform_pm1(6, 2, K, N)
        got = run_cfg(gpu, "f32", tile, 1, ta, tb, A, B, repeat=2)
        ref, S = oracle.gemm(A, B)
        assert oracle.componentwise_error(got, ref, S) <= TOL_F32
    A, B = inputs.small_ints(0, 3, 256, 256), inputs.small_ints(0, 4, 256, 256)
    ref, _ = oracle.gemm(A, B)
    assert np.array_equal(run_f32_ex(gpu, ta, tb, A, B).astype(np.float64), ref)


def test_f32_ex_plain_is_gemm_f32(gpu):
    A, B = inputs.uniform_pm1(6, 5, 300, 200), inputs.uniform_pm1(6, 6, 200, 260)
    assert np.array_equal(run_f32_ex(gpu, 0, 0, A, B).view(np.uint32), run_f32(gpu, A, B).view(np.uint32))


@pytest.mark.parametrize("shape", [(1, 1, 1), (17, 17, 17), (128, 128, 128), (130, 70, 200), (257, 255, 129),
                                   (33, 65, 31), (512, 384, 1000), (300, 520, 64),
                                   (2048, 2048, 192), (2000, 2100, 100)])          # the last two: 128 x 128 tiles
def test_bf16_shapes(gpu, shape):
    M, N, K = shape
    say("bf16 %dx%dx%d" % shape)
    A = inputs.bf16_normal_scaled(4, 20, M, K, 1 / math.sqrt(K))
    Bt = inputs.bf16_normal_scaled(4, 21, N, K, 1 / math.sqrt(K))
    check_bf16(gpu, A, Bt, repeat=2)
    pad = 8 if (M + N) % 2 == 0 else 3                     # aligned and unaligned leading dimensions
    check_bf16(gpu, A, Bt, lda=K + pad, ldb=K + pad, ldc=N + 5, offset=1 if pad == 3 else 0)


SKINNY = [(1, 4096, 4096), (4096, 1, 4096), (1, 1, 4096), (64, 64, 4097), (16, 1000, 3000), (257, 100, 2049),
          (3, 700, 1031), (300, 5, 8192), (128, 128, 16384), (512, 512, 1024),
          (256, 256, 16384), (768, 768, 2048), (320, 264, 1000)]       # K slices on the direct-to-LDS shapes (64 x 64 x 16, 128 x 64 x 3, ..)


@pytest.mark.parametrize("shape", SKINNY)
def test_f32_workspace_split_k(gpu, shape):
    # few output tiles, long K: with the workspace the product is cut along K and summed in slice order
    M, N, K = shape
    need = gpu.gemm_f32_workspace_bytes(0, 0, M, N, K)
    say("split-K %dx%dx%d workspace %d bytes" % (M, N, K, need))
    vector = min(M, N) <= 16                # the streaming kernels: whether they split depends on the storage order
    assert (need > 0 or vector) and need % (4 * M * N) == 0 and need <= 16 << 20
    A, B = inputs.uniform_pm1(7, 1, M, K), inputs.uniform_pm1(7, 2, K, N)
    ref, S = oracle.gemm(A, B)
    for ta, tb in ((0, 0), (0, 1), (1, 0), (1, 1)):
        assert vector or gpu.gemm_f32_workspace_bytes(ta, tb, M, N, K) == need
        got = run_f32_ws(gpu, ta, tb, A, B, repeat=2)
        assert oracle.componentwise_error(got, ref, S) <= TOL_F32
    pad = 3 if (M + N) % 2 else 4
    got = run_f32_ws(gpu, 0, 0, A, B, lda=K + pad, ldb=N + pad, ldc=N + 1, offset=1 if pad == 3 else 0, repeat=2)
    assert oracle.componentwise_error(got, ref, S) <= TOL_F32
    # a workspace one float short of what the plan for these (aligned) operands uses, or none, must leave the call equal to
    # gemm_f32_ex bit for bit; the query names at least that much (it also covers the plan for misaligned operands)
    plain = run_f32_ex(gpu, 0, 0, A, B)
    tile, slices = gpu.fsrgemm_plan_f32(0, 0, M, N, K, P_FAKE, K, P_FAKE, N, True)
    used = slices * M * N * 4 if slices > 1 or tile == 4 else 0
    assert used <= need
    if used:
        assert np.array_equal(run_f32_ws(gpu, 0, 0, A, B, workspace_bytes=used - 4).view(np.uint32), plain.view(np.uint32))
    assert np.array_equal(run_f32_ws(gpu, 0, 0, A, B, workspace_bytes=0).view(np.uint32), plain.view(np.uint32))


@pytest.mark.parametrize("shape", [(512, 512, 16384), (256, 1024, 16384), (384, 388, 28672)])
def test_splits_on_the_larger_tile(gpu, shape):
    # long-K splits that still fill the compute units with 128 x 128 tiles take those -- fp32: the direct-to-LDS kernel's
    # (candidate 10), or the general kernel's (candidate 1) for operands that are only 4-byte aligned; bf16: candidate 2 --
    # sampled entries against the oracle, and the dispatcher's bits are the forced candidate's
    M, N, K = shape
    rng = np.random.default_rng(23)
    ii, jj = rng.integers(0, M, 4096), rng.integers(0, N, 4096)
    A, B = inputs.uniform_pm1(23, 1, M, K), inputs.uniform_pm1(23, 2, K, N)
    ref, S = oracle.gemm_entries(A, B, ii, jj)
    for offset, want in ((0, 10 if N % 128 == 0 else 14), (1, 1)):       # (a ragged 388 columns: 64 x 64 tiles waste less)
        say("split on 128 x 128 tiles, fp32 %dx%dx%d, operands offset by %d" % (shape + (offset,)))
        tile, slices = gpu.fsrgemm_plan_f32(0, 0, M, N, K, 0x1000 + 4 * offset, K, 0x1000 + 4 * offset, N, True)
        assert tile == want and slices > 1
        got = run_f32_ws(gpu, 0, 0, A, B, offset=offset, repeat=2)
        assert np.all(np.isfinite(got)) and oracle.componentwise_error(got[ii, jj], ref, S) <= TOL_F32
        assert np.array_equal(run_cfg(gpu, "f32", tile, slices, 0, 0, A, B, offset=offset).view(np.uint32), got.view(np.uint32))
    Ah = inputs.bf16_normal_scaled(23, 3, M, K, 1 / math.sqrt(K))
    Bh = np.ascontiguousarray(inputs.bf16_normal_scaled(23, 4, N, K, 1 / math.sqrt(K)).T)
    ref, S = oracle.gemm_entries(Ah, Bh, ii, jj)
    for offset, want in ((0, 10), (1, None)):           # aligned: the direct-to-LDS 128 x 128 tile; otherwise a general tile
        say("split, bf16 %dx%dx%d, operands offset by %d" % (shape + (offset,)))
        tile, slices = gpu.fsrgemm_plan_bf16(0, 1, M, N, K, 0x1000 + 2 * offset, K, 0x1000 + 2 * offset, K, True)
        assert (tile == want if want else tile in (2, 3)) and slices > 1
        got = run_bf16_ws(gpu, 0, 1, Ah, Bh, offset=offset, repeat=2)
        assert np.all(np.isfinite(got)) and oracle.componentwise_error(got[ii, jj], ref, S) <= TOL_BF16
        assert np.array_equal(run_cfg(gpu, "bf16", tile, slices, 0, 1, Ah, Bh, offset=offset).view(np.uint32), got.view(np.uint32))


def test_f32_workspace_integers_bit_exact_and_large_problem_unsplit(gpu):
    A, B = inputs.small_ints(0, 5, 48, 4000), inputs.small_ints(0, 6, 4000, 200)
    assert gpu.gemm_f32_workspace_bytes(0, 0, 48, 200, 4000) > 0
    ref, _ = oracle.gemm(A, B)
    assert np.array_equal(run_f32_ws(gpu, 0, 0, A, B).astype(np.float64), ref)
    # enough tiles already: no workspace wanted, and one that is offered is not touched
    assert gpu.gemm_f32_workspace_bytes(0, 0, 2048, 2048, 4096) == 0
    A, B = inputs.uniform_pm1(7, 3, 1024, 256), inputs.uniform_pm1(7, 4, 256, 1024)
    assert np.array_equal(run_f32_ws(gpu, 0, 0, A, B, workspace_bytes=4096).view(np.uint32), run_f32(gpu, A, B).view(np.uint32))


@pytest.mark.parametrize("shape", [(1, 4096, 4096), (4096, 1, 4096), (8, 1000, 3000), (64, 64, 4100), (130, 70, 3082),
                                   (16, 8192, 2048), (256, 256, 8192),
                                   (512, 512, 8192), (768, 776, 4096)])     # 128 x 128 direct-to-LDS tiles in K slices
def test_bf16_workspace_split_k(gpu, shape):
    M, N, K = shape
    need = gpu.gemm_bf16_workspace_bytes(0, 1, M, N, K)
    say("bf16 split-K %dx%dx%d workspace %d bytes" % (M, N, K, need))
    vector = min(M, N) <= 16                # the streaming kernels: whether they split depends on the storage order
    assert (need > 0 or vector) and need % (4 * M * N) == 0 and need <= 16 << 20
    A = inputs.bf16_normal_scaled(4, 50, M, K, 1 / math.sqrt(K))
    B = inputs.bf16_normal_scaled(4, 51, K, N, 1 / math.sqrt(K))
    ref, S = oracle.gemm(A, B)
    for ta, tb in ((0, 1), (0, 0), (1, 0), (1, 1)):
        got = run_bf16_ws(gpu, ta, tb, A, B, repeat=2)
        assert oracle.componentwise_error(got, ref, S) <= TOL_BF16
    got = run_bf16_ws(gpu, 0, 1, A, B, lda=K + 3, ldb=K + 3, ldc=N + 1, offset=1, repeat=2)
    assert oracle.componentwise_error(got, ref, S) <= TOL_BF16
    plain = run_bf16_ex(gpu, 0, 1, A, B)
    tile, slices = gpu.fsrgemm_plan_bf16(0, 1, M, N, K, P_FAKE, K, P_FAKE, K, True)
    assert slices * M * N * 4 <= need or slices == 1
    if slices > 1:          # one float short of what the plan for these (aligned) operands uses: exactly the plain call
        assert np.array_equal(run_bf16_ws(gpu, 0, 1, A, B, workspace_bytes=slices * M * N * 4 - 4).view(np.uint32), plain.view(np.uint32))
    Ai, Bi = inputs.bf16_small_ints(4, 52, M, K), inputs.bf16_small_ints(4, 53, K, N)
    refi, _ = oracle.gemm(Ai, Bi)
    assert np.array_equal(run_bf16_ws(gpu, 0, 1, Ai, Bi).astype(np.float64), refi)


BF16_STORAGE = [(0, 0), (1, 0), (1, 1)]      # (transA, transB); (0, 1) is what gemm_bf16 takes


@pytest.mark.parametrize("ta,tb", BF16_STORAGE)
@pytest.mark.parametrize("shape", [(1, 1, 1), (17, 17, 17), (130, 70, 200), (257, 255, 129), (33, 65, 31),
                                   (512, 384, 1000), (300, 520, 64),
                                   (2048, 2048, 192), (2000, 2100, 100),             # 128 x 128 tiles
                                   (4096, 2048, 128), (4100, 2052, 72)])             # 256 x 256 tiles
def test_bf16_storage_orders(gpu, shape, ta, tb):
    M, N, K = shape
    say("bf16 storage %d%d %dx%dx%d" % (ta, tb, M, N, K))
    A = inputs.bf16_normal_scaled(4, 40, M, K, 1 / math.sqrt(K))
    B = inputs.bf16_normal_scaled(4, 41, K, N, 1 / math.sqrt(K))
    ref, S = oracle.gemm(A, B)
    got = run_bf16_ex(gpu, ta, tb, A, B, repeat=2)
    assert oracle.componentwise_error(got, ref, S) <= TOL_BF16
    pad = 8 if (M + N) % 2 == 0 else 3                     # aligned and unaligned leading dimensions
    lda, ldb = (M if ta else K) + pad, (K if tb else N) + pad
    got = run_bf16_ex(gpu, ta, tb, A, B, lda=lda, ldb=ldb, ldc=N + 5, offset=1 if pad == 3 else 0)
    assert oracle.componentwise_error(got, ref, S) <= TOL_BF16


@pytest.mark.parametrize("ta,tb", BF16_STORAGE)
@pytest.mark.parametrize("shape", [(4096, 2048, 64), (4096, 2048, 192), (2304, 4096, 448),      # whole tiles, 1 / 3 / 7 K-tiles
                                   (4000, 2104, 256), (2312, 3992, 128), (264, 33000, 64),        # shifted last tiles
                                   (1024, 768, 192), (256, 256, 1024), (264, 520, 328)])          # 128 x 128 tiles: k-rows of 256 bytes
def test_bf16_main_kernel_storage_orders(gpu, shape, ta, tb):
    # operands contiguous along m / n in the direct-to-LDS kernel: k-row tiles and transposing fragment reads
    M, N, K = shape
    say("bf16 main kernel storage %d%d %dx%dx%d" % (ta, tb, M, N, K))
    lda, ldb = (M if ta else K), (K if tb else N)
    is_main = lambda name: re.fullmatch(r"gemm_bf16_main_kernel<[468], [468], %d, %d>" % (ta, 1 - tb), name) is not None     # in whatever tile shape
    assert is_main(gpu.fsrgemm_kernel_for_bf16_ex(ta, tb, M, N, K, 0x1000, lda, 0x1000, ldb, 0x1000, N))
    A = inputs.bf16_normal_scaled(4, 70, M, K, 1 / math.sqrt(K))
    B = inputs.bf16_normal_scaled(4, 71, K, N, 1 / math.sqrt(K))
    ref, S = oracle.gemm(A, B)
    got = run_bf16_ex(gpu, ta, tb, A, B, repeat=2)
    assert oracle.componentwise_error(got, ref, S) <= TOL_BF16
    assert is_main(gpu.fsrgemm_kernel_for_bf16_ex(ta, tb, M, N, K, 0x1000, lda + 8, 0x1000, ldb + 40, 0x1000, N + 3))
    got = run_bf16_ex(gpu, ta, tb, A, B, lda=lda + 8, ldb=ldb + 40, ldc=N + 3, repeat=2)
    assert oracle.componentwise_error(got, ref, S) <= TOL_BF16
    Ai, Bi = inputs.bf16_small_ints(4, 72, M, K), inputs.bf16_small_ints(4, 73, K, N)
    refi, _ = oracle.gemm(Ai, Bi)
    assert np.array_equal(run_bf16_ex(gpu, ta, tb, Ai, Bi).astype(np.float64), refi)


@pytest.mark.parametrize("ta,tb", BF16_STORAGE + [(0, 1)])
def test_bf16_storage_orders_integers_bit_exact(gpu, ta, tb):
    A, B = inputs.bf16_small_ints(4, 42, 384, 512), inputs.bf16_small_ints(4, 43, 512, 320)
    ref, _ = oracle.gemm(A, B)
    assert np.array_equal(run_bf16_ex(gpu, ta, tb, A, B).astype(np.float64), ref)
    if (ta, tb) == (0, 1):          # the plain entry point is this storage pair
        assert np.array_equal(run_bf16(gpu, A, np.ascontiguousarray(B.T)).astype(np.float64), ref)


def test_bf16_512_integers_bit_exact(gpu):
    say("bf16 512^3 integers")
    A, Bt = inputs.bf16_small_ints(4, 30, 512, 512), inputs.bf16_small_ints(4, 31, 512, 512)
    got = run_bf16(gpu, A, Bt)
    ref, _ = oracle.gemm(A, Bt.T)
    assert np.array_equal(got.astype(np.float64), ref)


def test_bf16_big_tile_config_ragged(gpu):
    # large enough for the 256x256 configuration, not a tile multiple
    M, N, K = 2900, 3000, 200
    say("bf16 %dx%dx%d (256-tile, ragged)" % (M, N, K))
    A = inputs.bf16_normal_scaled(4, 40, M, K, 1 / math.sqrt(K))
    Bt = inputs.bf16_normal_scaled(4, 41, N, K, 1 / math.sqrt(K))
    assert gpu.fsrgemm_kernel_for_bf16(M, N, K, 0x1000, K, 0x1000, K, 0x1000, N).startswith("gemm_bf16_main_kernel<")    # with a rest of K
    check_bf16(gpu, A, Bt)
    A2, Bt2 = inputs.bf16_normal_scaled(4, 42, M, K + 4, 1 / math.sqrt(K)), inputs.bf16_normal_scaled(4, 43, N, K + 4, 1 / math.sqrt(K))
    assert gpu.fsrgemm_kernel_for_bf16(M, N, K + 4, 0x1000, K + 8, 0x1000, K + 8, 0x1000, N) == "gemm_bf16_kernel<4, 1, 1, 0, 0>"    # K not whole 16-byte pieces
    check_bf16(gpu, A2, Bt2, lda=K + 8, ldb=K + 8)


@pytest.mark.parametrize("shape,kernel", [((4000, 2100, 256), "gemm_bf16_main_kernel<"),           # the direct-to-LDS kernel in whatever shape, both sides ragged
                                          ((2304, 4090, 64), "gemm_bf16_main_kernel<"),            # one K-tile, ragged N
                                          ((257, 33000, 128), "gemm_bf16_main_kernel<"),           # the last tile row overlaps all but one row
                                          ((8200, 8400, 128), "gemm_bf16_main_kernel<"),           # more than 1024 tiles, both ragged
                                          ((2000, 2100, 128), "gemm_bf16_main_kernel<4, 4, 0, 0>"),  # 128 x 128 tiles of the direct-to-LDS kernel
                                          ((1000, 1100, 128), "gemm_bf16_kernel<1, 4, 0, 0, 0>"),  # too few of those: 64 x 64 tiles, unchecked
                                          ((300, 520, 64), "gemm_bf16_kernel<1, 4, 0, 0, 0>")])    # 64 x 64 tiles, unchecked
def test_bf16_ragged_last_tiles_are_shifted_back(gpu, shape, kernel):
    # aligned problems that are not a whole number of tiles run the unchecked kernels: the last tile row and
    # column start early enough to end with the matrix
    M, N, K = shape
    say("bf16 %dx%dx%d (shifted last tiles)" % shape)
    assert gpu.fsrgemm_kernel_for_bf16(M, N, K, 0x1000, K, 0x1000, K, 0x1000, N).startswith(kernel)
    A = inputs.bf16_normal_scaled(4, 60, M, K, 1 / math.sqrt(K))
    Bt = inputs.bf16_normal_scaled(4, 61, N, K, 1 / math.sqrt(K))
    check_bf16(gpu, A, Bt, repeat=2)
    check_bf16(gpu, A, Bt, lda=K + 8, ldb=K + 24, ldc=N + 3, repeat=2)
    Ai, Bi = inputs.bf16_small_ints(4, 62, M, K), inputs.bf16_small_ints(4, 63, N, K)
    ref, _ = oracle.gemm(Ai, Bi.T)
    assert np.array_equal(run_bf16(gpu, Ai, Bi).astype(np.float64), ref)


@pytest.mark.parametrize("shape,kernel", [((4000, 2040, 64), "gemm_f32_main_kernel<2, 4, 0, 1>"),
                                          ((4000, 2040, 80), "gemm_f32_main_kernel<2, 4, 0, 1>"),          # and a rest of K
                                          ((2040, 2030, 48), "gemm_f32_kernel<2, 2, 3, 0, 0, 1>"),
                                          ((1000, 1000, 1008), "gemm_f32_main_kernel<1, 1, 0, 1>"),
                                          ((1000, 1000, 1010), "gemm_f32_kernel<1, 1, 4, 2, 0, 1>"),          # rows of A that are not whole pieces: the general tile
                                          ((65, 129, 32), "gemm_f32_kernel<1, 1, 4, 0, 0, 1>")])
def test_f32_ragged_last_tiles_are_shifted_back(gpu, shape, kernel):
    M, N, K = shape
    say("fp32 %dx%dx%d (shifted last tiles)" % shape)
    assert gpu.fsrgemm_kernel_for_f32(M, N, K, 0x1000, K, 0x1000, N + (-N) % 4, 0x1000, N) == kernel
    A, B = inputs.uniform_pm1(8, 1, M, K), inputs.uniform_pm1(8, 2, K, N)
    ref, S = oracle.gemm(A, B)
    for ta, tb in ((0, 0), (1, 1)):
        lda, ldb = (M if ta else K), (K if tb else N)
        got = run_f32_ex(gpu, ta, tb, A, B, lda=lda + (-lda) % 4, ldb=ldb + (-ldb) % 4, ldc=N + 1, repeat=2)
        assert oracle.componentwise_error(got, ref, S) <= TOL_F32
    Ai, Bi = inputs.small_ints(0, 7, M, K), inputs.small_ints(0, 8, K, N)
    refi, _ = oracle.gemm(Ai, Bi)
    assert np.array_equal(run_f32(gpu, Ai, Bi, lda=K, ldb=N + (-N) % 4).astype(np.float64), refi)


@pytest.mark.parametrize("shape,tile,kernel", [((2048, 2048, 16), 1, "gemm_f32_kernel<2, 2, 3, 0, 0, 1>"),
                                               ((2048, 2048, 32), 1, "gemm_f32_kernel<2, 2, 3, 0, 0, 1>"),
                                               ((2048, 2048, 48), 1, "gemm_f32_kernel<2, 2, 3, 0, 0, 1>"),
                                               ((2048, 2048, 112), 1, "gemm_f32_kernel<2, 2, 3, 0, 0, 1>"),
                                               ((4096, 2048, 16), 0, "gemm_f32_kernel<4, 2, 2, 0, 0, 1>"),
                                               ((4096, 2048, 48), 0, "gemm_f32_kernel<4, 2, 2, 0, 0, 1>"),
                                               ((4096, 2048, 160), 0, "gemm_f32_kernel<4, 2, 2, 0, 0, 1>")])
def test_f32_tile_configs_small_k(gpu, shape, tile, kernel):
    # prologue, odd/even K-tile tails and the clamped prefetch of the two large tile configurations of the general kernel,
    # forced (the dispatcher gives these shapes to the direct-to-LDS kernel once K reaches 32); full oracle comparison
    M, N, K = shape
    say("fp32 %dx%dx%d tile %d" % (M, N, K, tile))
    assert gpu.fsrgemm_kernel_for_f32_cfg(tile, 0, 0, M, N, K, 0x1000, K, 0x1000, N, 0x1000, N) == kernel
    A, B = inputs.uniform_pm1(6, K, M, K), inputs.uniform_pm1(6, K + 1, K, N)
    ref, S = oracle.gemm(A, B)
    assert oracle.componentwise_error(run_cfg(gpu, "f32", tile, 1, 0, 0, A, B, repeat=2), ref, S) <= TOL_F32
    if K in (112, 160):
        assert gpu.fsrgemm_kernel_for_f32_cfg(tile, 0, 0, M, N, K, 0x1000, K + 4, 0x1000, N + 12, 0x1000, N + 1) == kernel
        assert oracle.componentwise_error(run_cfg(gpu, "f32", tile, 1, 0, 0, A, B, lda=K + 4, ldb=N + 12, ldc=N + 1), ref, S) <= TOL_F32
        Ai, Bi = inputs.small_ints(6, 90, M, K), inputs.small_ints(6, 91, K, N)
        assert np.array_equal(run_cfg(gpu, "f32", tile, 1, 0, 0, Ai, Bi).astype(np.float64), oracle.gemm(Ai, Bi)[0])


MAIN_SHAPES = {5: (256, 256), 6: (192, 256), 7: (128, 256), 8: (256, 128), 9: (192, 128), 10: (128, 128),        # fp32 candidates 5..16
               11: (256, 192), 12: (192, 192), 13: (128, 192), 14: (64, 64), 15: (128, 64), 16: (64, 128)}


@pytest.mark.parametrize("ta,tb", [(0, 0)] + LAYOUTS)
@pytest.mark.parametrize("shape", [(512, 768, 32), (512, 512, 64), (768, 512, 96), (256, 256, 224),     # whole tiles, 1 / 2 / 3 / 7 K-tiles
                                   (520, 392, 128), (264, 1284, 64), (1000, 260, 160),                  # shifted last tiles
                                   (512, 512, 44), (520, 392, 100), (384, 388, 60), (256, 512, 36),     # a rest of K behind 1 / 3 / 1 / 1 K-tiles
                                   (64, 64, 32), (68, 132, 72), (196, 64, 164)])                        # the tiles with a side of 64 only
def test_f32_main_kernel_storage_orders(gpu, shape, ta, tb):
    # the direct-to-LDS fp32 kernel in its twelve tile shapes, forced: prologue, odd / even tails, the clamped loads two
    # K-tiles ahead, operands contiguous along k and along m / n, padded leading dimensions, small integers, K slices
    M, N, K = shape
    lda, ldb = (M if ta else K), (K if tb else N)
    A, B = inputs.uniform_pm1(19, 1, M, K), inputs.uniform_pm1(19, 2, K, N)
    ref, S = oracle.gemm(A, B)
    Ai, Bi = inputs.small_ints(0, 19, M, K), inputs.small_ints(0, 20, K, N)
    refi, _ = oracle.gemm(Ai, Bi)
    for tile, (bm, bn) in MAIN_SHAPES.items():
        say("f32 main kernel %dx%d storage %d%d %dx%dx%d" % (bm, bn, ta, tb, M, N, K))
        fits = M >= bm and N >= bn and K % 4 == 0
        name = "gemm_f32_main_kernel<%d, %d, %d, %d>" % (bm // 64, bn // 64, ta, 1 - tb) if fits else None
        assert gpu.fsrgemm_kernel_for_f32_cfg(tile, ta, tb, M, N, K, 0x1000, lda, 0x1000, ldb, 0x1000, N) == name
        if not fits:
            with pytest.raises(gpu.FsrGemmError):
                run_cfg(gpu, "f32", tile, 1, ta, tb, A, B)
            continue
        got = run_cfg(gpu, "f32", tile, 1, ta, tb, A, B, repeat=2)
        assert oracle.componentwise_error(got, ref, S) <= TOL_F32
        assert gpu.fsrgemm_kernel_for_f32_cfg(tile, ta, tb, M, N, K, 0x1000, lda + 4, 0x1000, ldb + 36, 0x1000, N + 3) == name
        got = run_cfg(gpu, "f32", tile, 1, ta, tb, A, B, lda=lda + 4, ldb=ldb + 36, ldc=N + 3, repeat=2)
        assert oracle.componentwise_error(got, ref, S) <= TOL_F32
        assert np.array_equal(run_cfg(gpu, "f32", tile, 1, ta, tb, Ai, Bi).astype(np.float64), refi)
        # K slices of whole K-tiles (the last one takes the rest of K): partial products in the workspace, summed in slice
        # order; a count that would leave the last slice without a whole K-tile is rejected
        for slices in (2, 3):
            per = -(-(-(-K // 32)) // slices) * 32
            if (slices - 1) * per + 32 <= K:
                got = run_cfg(gpu, "f32", tile, slices, ta, tb, A, B, lda=lda + 4, ldb=ldb + 36, ldc=N + 3, repeat=2)
                assert oracle.componentwise_error(got, ref, S) <= TOL_F32
                assert np.array_equal(run_cfg(gpu, "f32", tile, slices, ta, tb, Ai, Bi).astype(np.float64), refi)
            else:
                with pytest.raises(gpu.FsrGemmError):
                    run_cfg(gpu, "f32", tile, slices, ta, tb, A, B)
        # where the candidate does not fit it is rejected: a misaligned base, rows that are not whole pieces
        for kw in (dict(offset=1), dict(lda=lda + 2)):
            with pytest.raises(gpu.FsrGemmError):
                run_cfg(gpu, "f32", tile, 1, ta, tb, A, B, **kw)


def test_f32_main_kernel_is_the_dispatchers_choice(gpu):
    # 16 x 16 tiles of 256 fill the compute units exactly once: the dispatcher takes the direct-to-LDS kernel, and
    # forcing it gives the same bits; a K that is not whole tiles of 32 stays on it (the rest-of-K step), and a K below 32
    # takes the general kernel
    M = N = 4096
    for K, kernel in ((64, "gemm_f32_main_kernel<4, 4, 0, 1>"), (48, "gemm_f32_main_kernel<4, 4, 0, 1>"), (16, "gemm_f32_kernel<4, 2, 2, 0, 0, 1>")):
        say("f32 4096x4096x%d through the dispatcher" % K)
        assert gpu.fsrgemm_kernel_for_f32(M, N, K, 0x1000, K, 0x1000, N, 0x1000, N) == kernel
        A, B = inputs.uniform_pm1(19, 3, M, K), inputs.uniform_pm1(19, 4, K, N)
        got = run_f32(gpu, A, B, repeat=2)
        rng = np.random.default_rng(19)
        ii, jj = rng.integers(0, M, 8192), rng.integers(0, N, 8192)
        ref, S = oracle.gemm_entries(A, B, ii, jj)
        assert np.all(np.isfinite(got)) and oracle.componentwise_error(got[ii, jj], ref, S) <= TOL_F32
        if K == 64:
            assert gpu.fsrgemm_plan_f32(0, 0, M, N, K, 0x1000, K, 0x1000, N, False) == (5, 1)
            assert np.array_equal(run_cfg(gpu, "f32", 5, 1, 0, 0, A, B).view(np.uint32), got.view(np.uint32))


BF16_MAIN_SHAPES = {0: (256, 256), 5: (192, 256), 6: (128, 256), 7: (256, 192), 8: (192, 192), 9: (256, 128), 10: (128, 128)}      # candidate -> tile


@pytest.mark.parametrize("ta,tb", [(0, 1)] + BF16_STORAGE)
@pytest.mark.parametrize("shape", [(512, 768, 64), (512, 512, 128), (768, 512, 192), (256, 256, 448),     # whole tiles, 1 / 2 / 3 / 7 K-tiles
                                   (520, 392, 128), (264, 1288, 64), (1000, 264, 192),                    # shifted last tiles
                                   (512, 512, 72), (520, 392, 232), (384, 392, 120), (256, 512, 104),     # a rest of K behind 1 / 3 / 1 / 1 K-tiles
                                   (128, 128, 64), (136, 200, 328)])                                      # the 128 x 128 tile only
def test_bf16_main_kernel_every_shape(gpu, shape, ta, tb):
    # the direct-to-LDS bf16 kernel in its seven tile shapes, forced: prologue, odd / even tails, the clamped loads two
    # K-tiles ahead, the rest of K (one and two k-steps of it), operands contiguous along k and along m / n (whole k-rows in LDS
    # for sides of 256 and 128, sub-tiles of 64 rows for 192), padded leading dimensions, small integers
    M, N, K = shape
    lda, ldb = (M if ta else K), (K if tb else N)
    A = inputs.bf16_normal_scaled(4, 80, M, K, 1 / math.sqrt(K))
    B = inputs.bf16_normal_scaled(4, 81, K, N, 1 / math.sqrt(K))
    ref, S = oracle.gemm(A, B)
    Ai, Bi = inputs.bf16_small_ints(4, 82, M, K), inputs.bf16_small_ints(4, 83, K, N)
    refi, _ = oracle.gemm(Ai, Bi)
    for tile, (bm, bn) in BF16_MAIN_SHAPES.items():
        say("bf16 main kernel %dx%d storage %d%d %dx%dx%d" % (bm, bn, ta, tb, M, N, K))
        fits = M >= bm and N >= bn
        name = "gemm_bf16_main_kernel<%d, %d, %d, %d>" % (bm // 32, bn // 32, ta, 1 - tb) if fits else None
        assert gpu.fsrgemm_kernel_for_bf16_cfg(tile, ta, tb, M, N, K, 0x1000, lda, 0x1000, ldb, 0x1000, N) == name
        if not fits:
            with pytest.raises(gpu.FsrGemmError):
                run_cfg(gpu, "bf16", tile, 1, ta, tb, A, B)
            continue
        got = run_cfg(gpu, "bf16", tile, 1, ta, tb, A, B, repeat=2)
        assert oracle.componentwise_error(got, ref, S) <= TOL_BF16
        assert gpu.fsrgemm_kernel_for_bf16_cfg(tile, ta, tb, M, N, K, 0x1000, lda + 8, 0x1000, ldb + 40, 0x1000, N + 3) == name
        got = run_cfg(gpu, "bf16", tile, 1, ta, tb, A, B, lda=lda + 8, ldb=ldb + 40, ldc=N + 3, repeat=2)
        assert oracle.componentwise_error(got, ref, S) <= TOL_BF16
        assert np.array_equal(run_cfg(gpu, "bf16", tile, 1, ta, tb, Ai, Bi).astype(np.float64), refi)
        # K slices of whole K-tiles (the last one takes the rest of K): partial products in the workspace, summed in slice
        # order; a count that would leave the last slice without a whole K-tile is rejected
        for slices in (2, 3):
            per = -(-(-(-K // 64)) // slices) * 64
            if (slices - 1) * per + 64 <= K:
                got = run_cfg(gpu, "bf16", tile, slices, ta, tb, A, B, lda=lda + 8, ldb=ldb + 40, ldc=N + 3, repeat=2)
                assert oracle.componentwise_error(got, ref, S) <= TOL_BF16
                assert np.array_equal(run_cfg(gpu, "bf16", tile, slices, ta, tb, Ai, Bi).astype(np.float64), refi)
            else:
                with pytest.raises(gpu.FsrGemmError):
                    run_cfg(gpu, "bf16", tile, slices, ta, tb, A, B)
        # where the candidate does not fit it is rejected: a misaligned base, rows that are not whole pieces
        for kw in (dict(offset=1), dict(lda=lda + 4)):
            with pytest.raises(gpu.FsrGemmError):
                run_cfg(gpu, "bf16", tile, 1, ta, tb, A, B, **kw)


def test_bf16_rest_of_k_at_full_width(gpu):
    # 8192 x 8192 with K = 1032 = 16 K-tiles and one piece: every tile of the headline grid runs the rest-of-K step
    M = N = 8192
    K = 1032
    say("bf16 %dx%dx%d (rest of K)" % (M, N, K))
    assert gpu.fsrgemm_kernel_for_bf16(M, N, K, 0x1000, K, 0x1000, K, 0x1000, N) == "gemm_bf16_main_kernel<8, 8, 0, 0>"
    A = inputs.bf16_normal_scaled(4, 84, M, K, 1 / math.sqrt(K))
    Bt = inputs.bf16_normal_scaled(4, 85, N, K, 1 / math.sqrt(K))
    got = run_bf16(gpu, A, Bt, repeat=2)
    ii, jj = one_entry_per_block(M, N, 16, 84)
    c, s = oracle.gemm_entries(A, Bt.T, ii, jj)
    assert oracle.componentwise_error(got[ii, jj], c, s) <= TOL_BF16
    assert oracle.freivalds_residual(A, Bt.T, got) <= freivalds_gate(N, K)


@pytest.mark.parametrize("K", [64, 128, 192, 448])
def test_bf16_main_kernel_small_k(gpu, K):
    # the direct-to-LDS kernel through the dispatcher with 1, 2, 3 and 7 K-tiles: prologue, odd/even tails, clamped prefetch
    M, N = 4096, 4096
    say("bf16 main kernel %dx%dx%d" % (M, N, K))
    assert gpu.fsrgemm_kernel_for_bf16(M, N, K, 0x1000, K, 0x1000, K, 0x1000, N).startswith("gemm_bf16_main_kernel<")
    A = inputs.bf16_normal_scaled(4, 50 + K, M, K, 1 / math.sqrt(K))
    Bt = inputs.bf16_normal_scaled(4, 51 + K, N, K, 1 / math.sqrt(K))
    check_bf16(gpu, A, Bt, repeat=2)
    if K == 192:                                            # padded leading dimensions stay on the same kernel
        assert gpu.fsrgemm_kernel_for_bf16(M, N, K, 0x1000, K + 8, 0x1000, K + 72, 0x1000, N + 3).startswith("gemm_bf16_main_kernel<")
        check_bf16(gpu, A, Bt, lda=K + 8, ldb=K + 72, ldc=N + 3)
        Ai, Bi = inputs.bf16_small_ints(4, 60, M, K), inputs.bf16_small_ints(4, 61, N, K)
        got = run_bf16(gpu, Ai, Bi)
        assert np.array_equal(got.astype(np.float64), oracle.gemm(Ai, Bi.T)[0])


def test_degenerate_extents(gpu):
    say("degenerate extents")
    A0, B0 = np.zeros((5, 0), np.float32), np.zeros((0, 7), np.float32)
    got = run_f32(gpu, A0, B0)                              # K = 0: empty sums
    assert got.shape == (5, 7) and np.all(got == 0) and not np.any(np.signbit(got))
    got = run_bf16(gpu, np.zeros((5, 0), np.uint16), np.zeros((7, 0), np.uint16))
    assert np.all(got == 0) and not np.any(np.signbit(got))
    assert gpu.gemm_f32(0, 7, 3, None, 3, None, 7, None, 7, 0) == gpu.FSRGEMM_OK
    assert gpu.gemm_bf16(4, 0, 3, None, 3, None, 3, None, 1, 0) == gpu.FSRGEMM_OK


def test_side_streams_and_host_threads(gpu):
    # the call enqueues on the caller's stream and may be issued from several host threads at once
    import threading

    import torch

    say("side streams + host threads")
    shapes = [(384, 320, 200), (257, 255, 129), (512, 512, 256), (130, 70, 200)]
    data, results, errors = [], [None] * len(shapes), []
    for idx, (M, N, K) in enumerate(shapes):
        data.append((inputs.uniform_pm1(8, 2 * idx, M, K), inputs.uniform_pm1(8, 2 * idx + 1, K, N)))

    def worker(idx):
        try:
            torch.cuda.set_device(0)
            M, N, K = shapes[idx]
            A, B = data[idx]
            stream = torch.cuda.Stream()
            with torch.cuda.stream(stream):
                a, b = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
                c = torch.full((M, N), float("nan"), device="cuda")
                for _ in range(20):
                    gpu.check(gpu.gemm_f32(M, N, K, a, K, b, N, c, N, stream.cuda_stream))
                stream.synchronize()
                results[idx] = c.cpu().numpy()
        except Exception as ex:          # surfaced in the main thread below
            errors.append(ex)

    threads = [threading.Thread(target=worker, args=(i,)) for i in range(len(shapes))]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    assert not errors, errors
    for idx, (A, B) in enumerate(data):
        ref, S = oracle.gemm(A, B)
        assert oracle.componentwise_error(results[idx], ref, S) <= TOL_F32


def _sample_indices(M, N, tile, n_rand, seed):
    rng = np.random.default_rng(seed)
    ii, jj = [rng.integers(0, M, n_rand)], [rng.integers(0, N, n_rand)]
    # the four entries around every interior tile-boundary crossing
    bm = np.arange(tile, M, tile)
    bn = np.arange(tile, N, tile)
    for di in (-1, 0):
        for dj in (-1, 0):
            gi, gj = np.meshgrid(bm + di, bn + dj, indexing="ij")
            ii.append(gi.ravel())
            jj.append(gj.ravel())
    return np.concatenate(ii), np.concatenate(jj)


def freivalds_gate(N, K):
    """Bound for oracle.freivalds_residual of an honest fp32-accumulated product: an entry's rounding error is a random
    walk of at most K roundings of 2^-24 relative to partial sums below S_ij, so it stays within sqrt(K) 2^-24 S_ij
    (the worst case K 2^-24 S_ij is never approached: the largest entry error seen is 0.02 sqrt(K) 2^-24 S_ij), and
    the random signs of the check average a row's N errors down by sqrt(N) against the row's scale.  Twice that.
    At N = K = 8192 this is 1.2e-7: a zeroed 16 x 16 block (residual about 8e-6) or one entry off by 1e-3 S_ij fails."""
    return 2.0 ** -23 * math.sqrt(K / N)


def test_f32_4096_normal_full_size(gpu):
    say("fp32 4096^3 normal seed 2 (every entry against the oracle + Freivalds)")
    n = 4096
    A, B = inputs.normal(2, 1, n, n), inputs.normal(2, 2, n, n)
    assert gpu.fsrgemm_kernel_for_f32(n, n, n, 0x1000, n, 0x1000, n, 0x1000, n) == "gemm_f32_main_kernel<4, 4, 0, 1>"
    got = run_f32(gpu, A, B)
    say("  GPU done; whole oracle product")
    ref, S = oracle.gemm(A, B)
    e = oracle.componentwise_error(got, ref, S)
    say("  componentwise error over all %d entries: %.3e" % (n * n, e))
    assert e <= TOL_F32
    r = oracle.freivalds_residual(A, B, got)
    say("  Freivalds residual %.3e (gate %.3e)" % (r, freivalds_gate(n, n)))
    assert r <= freivalds_gate(n, n)


def test_bf16_8192_full_size(gpu):
    say("bf16 8192^3 normal/sqrt(K) seed 4 (sampled rows, columns, an entry in every 16 x 16 block + Freivalds)")
    n = 8192
    A = inputs.bf16_normal_scaled(4, 1, n, n, 1 / math.sqrt(n))
    Bt = inputs.bf16_normal_scaled(4, 2, n, n, 1 / math.sqrt(n))
    assert gpu.fsrgemm_kernel_for_bf16(n, n, n, 0x1000, n, 0x1000, n, 0x1000, n) == "gemm_bf16_main_kernel<8, 8, 0, 0>"
    got = run_bf16(gpu, A, Bt)
    say("  GPU done; oracle on samples")
    rng = np.random.default_rng(4)
    rows, cols = np.sort(rng.choice(n, 128, replace=False)), np.sort(rng.choice(n, 128, replace=False))
    B_rm = np.ascontiguousarray(Bt.T)                       # same values, row-major, for a cache-friendly oracle walk
    ref, S = oracle.gemm(A[rows], B_rm)
    assert oracle.componentwise_error(got[rows], ref, S) <= TOL_BF16
    say("  rows ok")
    ref, S = oracle.gemm(A, np.ascontiguousarray(B_rm[:, cols]))
    assert oracle.componentwise_error(got[:, cols], ref, S) <= TOL_BF16
    say("  cols ok")
    del B_rm
    # one entry in each of the 262144 blocks of 16 x 16, and the four entries around every crossing of tile boundaries
    ii, jj = one_entry_per_block(n, n, 16, 4)
    ci, cj = _sample_indices(n, n, 256, 0, 4)
    ii, jj = np.concatenate([ii, ci]), np.concatenate([jj, cj])
    c, s = oracle.gemm_entries(A, Bt.T, ii, jj)
    e = oracle.componentwise_error(got[ii, jj], c, s)
    say("  %d entries: componentwise error %.3e" % (ii.size, e))
    assert e <= TOL_BF16
    # products of bf16 values are exact in fp32, so the error is that of fp32 accumulation alone: the same gate as fp32
    r = oracle.freivalds_residual(A, Bt.T, got)
    say("  Freivalds residual %.3e (gate %.3e)" % (r, freivalds_gate(n, n)))
    assert r <= freivalds_gate(n, n)


@pytest.mark.parametrize("shape,kernel", [((6144, 6144, 6144), "gemm_bf16_main_kernel<8, 6, 0, 0>"),       # 768 tiles of 256 x 192: three whole rounds
                                          ((3072, 8192, 4096), "gemm_bf16_main_kernel<6, 8, 0, 0>"),       # 512 tiles of 192 x 256
                                          ((8192, 8192, 8200), "gemm_bf16_main_kernel<8, 8, 0, 0>"),       # a rest of K, rows that straddle cache lines
                                          ((3072, 3072, 3072), "gemm_bf16_main_kernel<6, 6, 0, 0>")])      # one round of 256 tiles of 192 x 192
def test_bf16_mid_sizes_in_the_timed_configuration(gpu, shape, kernel):
    # the problems the bench's mid_sizes_bf16 section times, in the tile shape the dispatcher takes for them: an entry in
    # every 16 x 16 block against the oracle, and the Freivalds residual over all entries
    M, N, K = shape
    say("bf16 %dx%dx%d (%s)" % (M, N, K, kernel))
    assert gpu.fsrgemm_kernel_for_bf16(M, N, K, 0x1000, K, 0x1000, K, 0x1000, N) == kernel
    A = inputs.bf16_normal_scaled(4, 90, M, K, 1 / math.sqrt(K))
    Bt = inputs.bf16_normal_scaled(4, 91, N, K, 1 / math.sqrt(K))
    got = run_bf16(gpu, A, Bt)
    ii, jj = one_entry_per_block(M, N, 16, 90)
    c, s = oracle.gemm_entries(A, Bt.T, ii, jj)
    e = oracle.componentwise_error(got[ii, jj], c, s)
    r = oracle.freivalds_residual(A, Bt.T, got)
    say("  %d entries: componentwise error %.3e; Freivalds residual %.3e (gate %.3e)" % (ii.size, e, r, freivalds_gate(N, K)))
    assert e <= TOL_BF16 and r <= freivalds_gate(N, K)


@pytest.mark.parametrize("n,ta,tb,kernel", [(8192, 1, 0, "gemm_bf16_main_kernel<8, 8, 1, 1>"), (6144, 0, 0, "gemm_bf16_main_kernel<8, 6, 0, 1>"),
                                            (3072, 1, 1, "gemm_bf16_main_kernel<6, 6, 1, 0>"), (2048, 1, 0, "gemm_bf16_main_kernel<4, 4, 1, 1>")])
def test_bf16_storage_orders_in_the_timed_configuration(gpu, n, ta, tb, kernel):
    # cubes the bench's storage_orders_bf16 section times, with operands contiguous along m / n, in the tile shape the
    # dispatcher takes: an entry in every 16 x 16 block against the oracle, and the Freivalds residual over all entries
    say("bf16 %d^3 transA=%d transB=%d (%s)" % (n, ta, tb, kernel))
    assert gpu.fsrgemm_kernel_for_bf16_ex(ta, tb, n, n, n, 0x1000, n, 0x1000, n, 0x1000, n) == kernel
    A = inputs.bf16_normal_scaled(4, 92, n, n, 1 / math.sqrt(n))
    B = inputs.bf16_normal_scaled(4, 93, n, n, 1 / math.sqrt(n))
    got = run_bf16_ex(gpu, ta, tb, A, B)
    ii, jj = one_entry_per_block(n, n, 16, 92)
    c, s = oracle.gemm_entries(A, B, ii, jj)
    e = oracle.componentwise_error(got[ii, jj], c, s)
    r = oracle.freivalds_residual(A, B, got)
    say("  %d entries: componentwise error %.3e; Freivalds residual %.3e (gate %.3e)" % (ii.size, e, r, freivalds_gate(n, n)))
    assert e <= TOL_BF16 and r <= freivalds_gate(n, n)


def test_f32_rest_of_k_on_the_largest_tile(gpu):
    # 4096 x 4096 x 4112 (the bench's mid-size case with a K that is not whole K-tiles): the 256 x 256 tile with its
    # rest-of-K step, every tile of the headline grid; whole rows and columns, an entry per 32 x 32 block, Freivalds
    M = N = 4096
    K = 4112
    say("fp32 %dx%dx%d (rest of K on 256 x 256 tiles)" % (M, N, K))
    assert gpu.fsrgemm_kernel_for_f32(M, N, K, 0x1000, K, 0x1000, N, 0x1000, N) == "gemm_f32_main_kernel<4, 4, 0, 1>"
    A, B = inputs.normal(2, 5, M, K), inputs.normal(2, 6, K, N)
    got = run_f32(gpu, A, B, repeat=2)
    rows = np.arange(7, M, 131)
    ref, S = oracle.gemm(A[rows], B)
    assert oracle.componentwise_error(got[rows], ref, S) <= TOL_F32
    ii, jj = one_entry_per_block(M, N, 32, 5)
    c, s = oracle.gemm_entries(A, B, ii, jj)
    assert oracle.componentwise_error(got[ii, jj], c, s) <= TOL_F32
    assert oracle.freivalds_residual(A, B, got) <= freivalds_gate(N, K)


def test_f32_paper_task2_largest_size(gpu):
    # the paper's largest Task 2 input (input-size table): A (2^18, 4096), B (4096, 2048).  A is 4 GiB, so element
    # offsets reach 2^30 and byte offsets 2^32: this is the 64-bit indexing case.  A is built from one seeded
    # 4096-row block repeated 64 times with a different power-of-two scale per copy, so a row fetched from the
    # wrong copy would not pass.
    import torch

    M, N, K = 1 << 18, 2048, 4096
    say("fp32 %dx%dx%d (paper Task 2, size 2^18)" % (M, N, K))
    block = inputs.uniform_pm1(5, 11, 4096, K)
    B = inputs.uniform_pm1(5, 12, K, N)
    A = np.empty((M, K), dtype=np.float32)
    for b in range(64):
        A[b * 4096:(b + 1) * 4096] = block * np.float32(2.0 ** ((b % 5) - 2))
    assert gpu.fsrgemm_kernel_for_f32(M, N, K, 0x1000, K, 0x1000, N, 0x1000, N) == "gemm_f32_main_kernel<4, 4, 0, 1>"
    a, b_, c = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda(), torch.full((M, N), float("nan"), device="cuda")
    gpu.check(gpu.gemm_f32(M, N, K, a, K, b_, N, c, N, torch.cuda.current_stream().cuda_stream))
    torch.cuda.synchronize()
    rng = np.random.default_rng(18)
    rows = np.unique(np.concatenate([rng.integers(0, M, 96), np.arange(0, M, 4096), np.arange(4095, M, 4096), [M - 1]]))
    got = c[torch.from_numpy(rows).cuda()].cpu().numpy()
    ref, S = oracle.gemm(A[rows], B)
    assert oracle.componentwise_error(got, ref, S) <= TOL_F32
    cols = np.sort(rng.choice(N, 8, replace=False))
    got_cols = c[:, torch.from_numpy(cols).cuda()].cpu().numpy()
    assert np.all(np.isfinite(got_cols))
    ref, S = oracle.gemm(A, np.ascontiguousarray(B[:, cols]))
    assert oracle.componentwise_error(got_cols, ref, S) <= TOL_F32


def test_bf16_operand_beyond_4_gib(gpu):
    # A of 2^18 x 8192 bf16 is 4 GiB: row offsets pass 2^32 bytes inside the direct-to-LDS kernel (64-bit scalar row
    # bases, 32-bit lane offsets).  As in the fp32 case above, A is one seeded 4096-row block repeated 64 times with
    # a different power-of-two scale per copy (exact in bf16), so a row fetched from the wrong copy would not pass.
    import torch

    M, N, K = 1 << 18, 256, 8192
    say("bf16 %dx%dx%d (A of 4 GiB)" % (M, N, K))
    block = inputs.bf16_normal_scaled(5, 21, 4096, K, 1 / math.sqrt(K))
    Bt = inputs.bf16_normal_scaled(5, 22, N, K, 1 / math.sqrt(K))
    A = np.empty((M, K), dtype=np.uint16)
    for b in range(64):
        # scaling by 2^e adds e to the exponent field (bits 7..14); the block's values are far from overflow and underflow
        A[b * 4096:(b + 1) * 4096] = block + np.uint16((((b % 5) - 2) << 7) & 0xFFFF) if (b % 5) >= 2 else block - np.uint16((2 - (b % 5)) << 7)
    assert gpu.fsrgemm_kernel_for_bf16(M, N, K, 0x1000, K, 0x1000, K, 0x1000, N).startswith("gemm_bf16_main_kernel<")
    a = torch.from_numpy(A.view(np.int16)).cuda()
    b_ = torch.from_numpy(Bt.view(np.int16)).cuda()
    c = torch.full((M, N), float("nan"), device="cuda")
    gpu.check(gpu.gemm_bf16(M, N, K, a, K, b_, K, c, N, torch.cuda.current_stream().cuda_stream))
    torch.cuda.synchronize()
    rng = np.random.default_rng(19)
    rows = np.unique(np.concatenate([rng.integers(0, M, 96), np.arange(0, M, 4096), np.arange(4095, M, 4096), [M - 1]]))
    got = c[torch.from_numpy(rows).cuda()].cpu().numpy()
    ref, S = oracle.gemm(A[rows], Bt.T)
    assert oracle.componentwise_error(got, ref, S) <= TOL_BF16
    cols = np.sort(rng.choice(N, 4, replace=False))
    got_cols = c[:, torch.from_numpy(cols).cuda()].cpu().numpy()
    assert np.all(np.isfinite(got_cols))
    ref, S = oracle.gemm(A, np.ascontiguousarray(Bt[cols].T))
    assert oracle.componentwise_error(got_cols, ref, S) <= TOL_BF16


def test_f32_paper_task2_shape(gpu):
    # the paper's own Task 2 operand shapes (input-size table): A (size, 4096), B (4096, 2048); smallest size
    say("fp32 1024x2048x4096 (paper Task 2, size 2^10)")
    M, N, K = 1024, 2048, 4096
    A, B = inputs.uniform_pm1(5, 1, M, K), inputs.uniform_pm1(5, 2, K, N)
    got = run_f32(gpu, A, B)
    rows = np.arange(0, M, 37)
    ref, S = oracle.gemm(A[rows], B)
    assert oracle.componentwise_error(got[rows], ref, S) <= TOL_F32
    assert oracle.freivalds_residual(A, B, got) <= freivalds_gate(N, K)


# ---- transposition (the paper's Task 8): data movement, so every case is bit for bit ----

# ---- a seeded mix of everything ----

def test_random_shapes_through_every_entry_point(gpu):
    # 160 seeded cases: precision, storage orders, shape (log-uniform, with vectors and long K mixed in), paddings,
    # offsets, with and without a workspace, dispatcher's choice or a random valid candidate
    import random

    rng = random.Random(31)
    draw = lambda hi: max(1, int(2 ** (rng.random() * math.log2(hi))))
    for case in range(160):
        kind = rng.choice(("f32", "bf16"))
        ta, tb = rng.randint(0, 1), rng.randint(0, 1)
        M, N, K = draw(600), draw(600), draw(5000)
        if rng.random() < 0.2:
            M = 1
        if rng.random() < 0.2:
            N = rng.choice((1, 10))
        pad = 8 if rng.random() < 0.5 else rng.choice((1, 3, 5))
        off = 0 if pad == 8 and rng.random() < 0.7 else 1
        lda, ldb = (M if ta else K) + (pad if pad != 8 else (-(M if ta else K)) % 8), (K if tb else N) + (pad if pad != 8 else (-(K if tb else N)) % 8)
        say("random case %d: %s %d%d %dx%dx%d lda %d ldb %d offset %d" % (case, kind, ta, tb, M, N, K, lda, ldb, off))
        if kind == "f32":
            A, B = inputs.uniform_pm1(18, 2 * case, M, K), inputs.uniform_pm1(18, 2 * case + 1, K, N)
            tol, run_ws, run_ex, count = TOL_F32, run_f32_ws, run_f32_ex, gpu.fsrgemm_tile_count_f32()
        else:
            A = inputs.bf16_normal_scaled(18, 2 * case, M, K, 1 / math.sqrt(K))
            B = inputs.bf16_normal_scaled(18, 2 * case + 1, K, N, 1 / math.sqrt(K))
            tol, run_ws, run_ex, count = TOL_BF16, run_bf16_ws, run_bf16_ex, gpu.fsrgemm_tile_count_bf16()
        ref, S = oracle.gemm(A, B)
        kw = dict(lda=lda, ldb=ldb, ldc=N + rng.choice((0, 1, 4)), offset=off, repeat=2)
        mode = rng.choice(("plain", "workspace", "forced"))
        if mode == "plain":
            got = run_ex(gpu, ta, tb, A, B, **kw)
        elif mode == "workspace":
            got = run_ws(gpu, ta, tb, A, B, **kw)
        else:
            tile, slices = rng.randrange(count), rng.choice((1, 1, 2, 3, 8))
            try:
                got = run_cfg(gpu, kind, tile, slices, ta, tb, A, B, **kw)
            except gpu.FsrGemmError:
                continue                        # a candidate that cannot run this problem is rejected, never launched
        assert oracle.componentwise_error(got, ref, S) <= tol, (case, kind, ta, tb, M, N, K, mode)


def test_random_thin_shapes_through_every_entry_point(gpu):
    # 120 seeded cases with 1 .. 17 rows or columns on one side: precision, storage orders, the long side and K from lists
    # around the streaming kernels' pieces, chunks and blocks, leading dimensions that keep or break 16-byte rows, offsets
    # that keep or break 16-byte bases; without a workspace, with one, or as the vector candidate in 1 .. 5 K slices
    import random

    rng = random.Random(36)
    seen = set()
    for case in range(120):
        kind = rng.choice(("f32", "bf16"))
        q = 4 if kind == "f32" else 8                       # elements per 16-byte piece
        small = rng.randint(1, 17)
        big = rng.choice((1, 3, 4, 7, 8, 9, 15, 16, 31, 33, 64, 100, 257, 1000, 4097, 20000))
        K = rng.choice((1, 2, 7, 8, 9, 31, 64, 100, 255, 256, 257, 511, 512, 1000, 1024, 1032, 2048, 3000, 5000, 8200))
        if big * K > 2e7:
            K = 1000
        M, N = (small, big) if rng.random() < 0.5 else (big, small)
        ta, tb = rng.randint(0, 1), rng.randint(0, 1)
        ca, cb = (M if ta else K), (K if tb else N)
        pa, pb = rng.choice((0, 0, q, 3 * q, -1)), rng.choice((0, 0, q, 2 * q, -1))
        lda = ca + 1 if pa < 0 else ca + (-ca) % q + pa      # (-1: a leading dimension that breaks the 16-byte rows)
        ldb = cb + 3 if pb < 0 else cb + (-cb) % q + pb
        off = rng.choice((0, 0, 0, 1))
        if kind == "f32":
            A, B = inputs.uniform_pm1(36, 2 * case, M, K), inputs.uniform_pm1(36, 2 * case + 1, K, N)
            tol, run_ws, run_ex, cand, named = TOL_F32, run_f32_ws, run_f32_ex, 3, gpu.fsrgemm_kernel_for_f32_ex
        else:
            A = inputs.bf16_normal_scaled(36, 2 * case, M, K, 1 / math.sqrt(K))
            B = inputs.bf16_normal_scaled(36, 2 * case + 1, K, N, 1 / math.sqrt(K))
            tol, run_ws, run_ex, cand, named = 1e-5, run_bf16_ws, run_bf16_ex, 4, gpu.fsrgemm_kernel_for_bf16_ex
        if off == 0:
            seen.add(named(ta, tb, M, N, K, P_FAKE, lda, P_FAKE, ldb, P_FAKE, N).split("<")[0])
        mode = rng.choice(("plain", "workspace", "forced"))
        say("thin case %d: %s %d%d %dx%dx%d lda %d ldb %d offset %d %s" % (case, kind, ta, tb, M, N, K, lda, ldb, off, mode))
        ref, S = oracle.gemm(A, B)
        kw = dict(lda=lda, ldb=ldb, ldc=N + rng.choice((0, 1, 4)), offset=off, repeat=2)
        if mode == "plain":
            got = run_ex(gpu, ta, tb, A, B, **kw)
        elif mode == "workspace":
            got = run_ws(gpu, ta, tb, A, B, **kw)
        else:
            try:
                got = run_cfg(gpu, kind, cand, rng.choice((1, 2, 3, 5)), ta, tb, A, B, **kw)
            except gpu.FsrGemmError:
                continue                        # not a problem for the vector candidate (17 vectors, a misaligned matrix, ...)
        assert oracle.componentwise_error(got, ref, S) <= tol, (case, kind, ta, tb, M, N, K, mode)
    # the draw reaches the kernels it is there for
    assert {"gemv_rows_f32_few_kernel", "gemv_cols_f32_few_kernel", "gemv_rows_bf16_few_kernel", "gemv_cols_bf16_few_kernel",
            "gemv_rows_bf16_mfma_direct_kernel"} <= seen, seen


def test_random_larger_aligned_shapes_through_the_plain_entry_points(gpu):
    # 28 seeded cases of 1024 .. 6000 rows and columns, aligned, every storage order, ragged against every tile: what the
    # dispatcher makes of them (tiles of every size, two bands, a rest of K) against the oracle's whole product
    import random

    rng = random.Random(33)
    seen = set()
    for case in range(28):
        kind = rng.choice(("f32", "bf16"))
        ta, tb = rng.randint(0, 1), rng.randint(0, 1)
        M, N = 8 * rng.randint(128, 750), 8 * rng.randint(128, 750)
        K = (4 if kind == "f32" else 8) * rng.randint(32, 280)
        while M * N * K > 2.4e10:
            M = max(1024, M // 2 // 8 * 8)
        if case % 7 == 3:           # shapes whose tiles fill no whole rounds in any one shape: the two-band plans
            kind, (M, N), K = "f32", rng.choice(((5000, 5120), (5120, 5000), (6656, 5000), (3000, 7168))), rng.choice((512, 772))
        pad = 8 * rng.choice((0, 0, 1, 3))
        lda, ldb = (M if ta else K) + pad, (K if tb else N) + pad
        if kind == "f32":
            A, B = inputs.uniform_pm1(33, 2 * case, M, K), inputs.uniform_pm1(33, 2 * case + 1, K, N)
            tol, run_ex, bands, named = TOL_F32, run_f32_ex, gpu.fsrgemm_bands_f32, gpu.fsrgemm_kernel_for_f32_ex
        else:
            A = inputs.bf16_normal_scaled(33, 2 * case, M, K, 1 / math.sqrt(K))
            B = inputs.bf16_normal_scaled(33, 2 * case + 1, K, N, 1 / math.sqrt(K))
            tol, run_ex, bands, named = 1e-5, run_bf16_ex, gpu.fsrgemm_bands_bf16, gpu.fsrgemm_kernel_for_bf16_ex
        dim, at, first, second = bands(ta, tb, M, N, K, P_FAKE, lda, P_FAKE, ldb)
        name = named(ta, tb, M, N, K, P_FAKE, lda, P_FAKE, ldb, P_FAKE, N)
        say("larger case %d: %s %d%d %dx%dx%d lda %d ldb %d -> %s" % (case, kind, ta, tb, M, N, K, lda, ldb, name))
        seen.add((kind, dim != 0))
        seen.add((kind, first))
        ref, S = oracle.gemm(A, B)
        got = run_ex(gpu, ta, tb, A, B, lda=lda, ldb=ldb, ldc=N + rng.choice((0, 4)), repeat=2)
        e = oracle.componentwise_error(got, ref, S)
        assert e <= tol, (case, kind, ta, tb, M, N, K, name, e)
    # the draw does reach the paths it is there for: two-band plans and one launch in both precisions, several tile shapes
    assert {("f32", True), ("f32", False), ("bf16", False)} <= seen and len([x for x in seen if not isinstance(x[1], bool)]) >= 6, seen


def test_random_small_bf16_shapes_in_every_storage_order(gpu):
    # 32 seeded bf16 cases of 128 .. 1280 rows and columns (multiples of 8, ragged against the 128 x 128 tile) in the
    # four storage orders with padded leading dimensions: with an operand contiguous along m / n the dispatcher takes the
    # direct-to-LDS kernel's 128 x 128 tile from four tiles on, below that (and for K < 64) the general kernel
    import random

    rng = random.Random(34)
    main = 0
    for case in range(32):
        ta, tb = ((0, 0), (1, 1), (1, 0), (0, 1))[case % 4]
        M, N, K = 8 * rng.randint(16, 160), 8 * rng.randint(16, 160), 8 * rng.randint(4, 200)
        pad = 8 * rng.choice((0, 1, 5))
        lda, ldb = (M if ta else K) + pad, (K if tb else N) + pad
        A = inputs.bf16_normal_scaled(34, 2 * case, M, K, 1 / math.sqrt(K))
        B = inputs.bf16_normal_scaled(34, 2 * case + 1, K, N, 1 / math.sqrt(K))
        name = gpu.fsrgemm_kernel_for_bf16_ex(ta, tb, M, N, K, P_FAKE, lda, P_FAKE, ldb, P_FAKE, N)
        say("small case %d: bf16 %d%d %dx%dx%d lda %d ldb %d -> %s" % (case, ta, tb, M, N, K, lda, ldb, name))
        main += name.startswith("gemm_bf16_main_kernel<4, 4")
        ref, S = oracle.gemm(A, B)
        got = run_bf16_ex(gpu, ta, tb, A, B, lda=lda, ldb=ldb, ldc=N + rng.choice((0, 4)), repeat=2)
        e = oracle.componentwise_error(got, ref, S)
        assert e <= 1e-5, (case, ta, tb, M, N, K, name, e)
    assert main >= 12, main


def test_random_aligned_shapes_with_a_workspace(gpu):
    # 48 seeded cases of 128 .. 1536 rows and columns and K up to 32768, aligned, every storage order, padded leading
    # dimensions, with a workspace: what the slice planners make of them (K slices on the direct-to-LDS tiles or on the
    # general kernels, or no split) against the oracle's whole product, and bit for bit the same on a second call
    import random

    rng = random.Random(35)
    split_main = {"f32": 0, "bf16": 0}
    for case in range(48):
        kind = ("f32", "bf16")[case % 2]
        ta, tb = rng.randint(0, 1), rng.randint(0, 1)
        M, N = 8 * rng.randint(16, 192), 8 * rng.randint(16, 192)
        K = 8 * int(2 ** (6 + 6 * rng.random()))
        while M * N * K > 4e9:
            M = max(128, M // 2 // 8 * 8)
        pad = 8 * rng.choice((0, 0, 1, 3))
        lda, ldb = (M if ta else K) + pad, (K if tb else N) + pad
        if kind == "f32":
            A, B = inputs.uniform_pm1(35, 2 * case, M, K), inputs.uniform_pm1(35, 2 * case + 1, K, N)
            tol, run_ws, plan, named = TOL_F32, run_f32_ws, gpu.fsrgemm_plan_f32, gpu.fsrgemm_kernel_for_f32_cfg
        else:
            A = inputs.bf16_normal_scaled(35, 2 * case, M, K, 1 / math.sqrt(K))
            B = inputs.bf16_normal_scaled(35, 2 * case + 1, K, N, 1 / math.sqrt(K))
            tol, run_ws, plan, named = 1e-5, run_bf16_ws, gpu.fsrgemm_plan_bf16, gpu.fsrgemm_kernel_for_bf16_cfg
        tile, slices = plan(ta, tb, M, N, K, P_FAKE, lda, P_FAKE, ldb, True)
        name = named(tile, ta, tb, M, N, K, P_FAKE, lda, P_FAKE, ldb, P_FAKE, N)
        say("workspace case %d: %s %d%d %dx%dx%d lda %d ldb %d -> %s, %d slices" % (case, kind, ta, tb, M, N, K, lda, ldb, name, slices))
        split_main[kind] += slices > 1 and "main" in name
        ref, S = oracle.gemm(A, B)
        got = run_ws(gpu, ta, tb, A, B, lda=lda, ldb=ldb, ldc=N + rng.choice((0, 4)), repeat=2)
        e = oracle.componentwise_error(got, ref, S)
        assert e <= tol, (case, kind, ta, tb, M, N, K, name, slices, e)
    assert split_main["f32"] >= 4 and split_main["bf16"] >= 4, split_main


# ---- the library under HIP graph capture ----

def test_calls_captured_in_a_hip_graph_replay_bit_exact(gpu):
    # the entry points allocate nothing and clear nothing with memset, so a validator pass (many launches on many
    # shapes) can be captured once and replayed; every replay must give the eager bits
    import torch

    stream = lambda: torch.cuda.current_stream().cuda_stream
    calls, outs = [], []
    for c in inputs.sweep_cases(3, 64)[::3]:
        M, N, K = c["M"], c["N"], c["K"]
        a, b, o = torch.randn(M, K, device="cuda"), torch.randn(K, N, device="cuda"), torch.empty(M, N, device="cuda")
        calls.append(lambda a=a, b=b, o=o, M=M, N=N, K=K: gpu.gemm_f32(M, N, K, a, K, b, N, o, N, stream()))
        outs.append(o)
    a, b, o = torch.randn(64, 8192, device="cuda"), torch.randn(8192, 64, device="cuda"), torch.empty(64, 64, device="cuda")
    ws = torch.empty(gpu.gemm_f32_workspace_bytes(0, 0, 64, 64, 8192), dtype=torch.uint8, device="cuda")
    assert ws.numel() > 0
    calls.append(lambda a=a, b=b, o=o: gpu.gemm_f32_ws(0, 0, 64, 64, 8192, a, 8192, b, 64, o, 64, ws, ws.numel(), stream()))
    outs.append(o)
    ah = (torch.randn(512, 256, device="cuda") / 16).to(torch.bfloat16)
    bh = (torch.randn(768, 256, device="cuda") / 16).to(torch.bfloat16)
    oh = torch.empty(512, 768, device="cuda")
    # tile 0: the direct-to-LDS kernel, whose loads are issued from inline assembly
    calls.append(lambda: gpu.gemm_bf16_cfg(0, 1, 0, 1, 512, 768, 256, ah, 256, bh, 256, oh, 768, None, 0, stream()))
    outs.append(oh)
    # fp32 candidates 12 and 9: the fp32 direct-to-LDS kernel (192 x 192 and 192 x 128 tiles), hand-issued loads as well
    am, bm_, om = torch.randn(400, 96, device="cuda"), torch.randn(96, 388, device="cuda"), torch.empty(2, 400, 388, device="cuda")
    calls.append(lambda: gpu.gemm_f32_cfg(12, 1, 0, 0, 400, 388, 96, am, 96, bm_, 388, om[0], 388, None, 0, stream()))
    calls.append(lambda: gpu.gemm_f32_cfg(9, 1, 0, 0, 400, 388, 96, am, 96, bm_, 388, om[1], 388, None, 0, stream()))
    outs.append(om)
    # a product the dispatcher runs as two bands of C: two launches behind one call
    ab, bb, ob = torch.randn(3584, 1024, device="cuda"), torch.randn(1024, 3584, device="cuda"), torch.empty(3584, 3584, device="cuda")
    assert gpu.fsrgemm_bands_f32(0, 0, 3584, 3584, 1024, ab, 1024, bb, 3584)[0] != 0
    calls.append(lambda: gpu.gemm_f32(3584, 3584, 1024, ab, 1024, bb, 3584, ob, 3584, stream()))
    outs.append(ob)
    t_in, t_out = torch.randn(300, 700, device="cuda"), torch.empty(700, 300, device="cuda")
    calls.append(lambda: gpu.transpose_f32(300, 700, t_in, 700, t_out, 300, stream()))
    outs.append(t_out)
    v_in, v_out = torch.randn(1, 5000, device="cuda"), torch.empty(1, 300, device="cuda")
    m_in = torch.randn(5000, 300, device="cuda")
    calls.append(lambda: gpu.gemm_f32(1, 300, 5000, v_in, 5000, m_in, 300, v_out, 300, stream()))
    outs.append(v_out)
    # a few rows on one side: the streaming kernels that stage the vectors in LDS (fp32: both patterns; bf16: lane arithmetic
    # and both matrix-core kernels)
    f_in, f_out = torch.randn(6, 5000, device="cuda"), torch.empty(2, 6, 300, device="cuda")
    mt_in = torch.randn(300, 5000, device="cuda")
    calls.append(lambda: gpu.gemm_f32(6, 300, 5000, f_in, 5000, m_in, 300, f_out[0], 300, stream()))
    calls.append(lambda: gpu.gemm_f32_ex(0, 1, 6, 300, 5000, f_in, 5000, mt_in, 5000, f_out[1], 300, stream()))
    outs.append(f_out)
    h_in = (torch.randn(12, 4096, device="cuda") / 64).to(torch.bfloat16)
    hm_in, hn_in = (torch.randn(264, 4096, device="cuda") / 64).to(torch.bfloat16), (torch.randn(4096, 264, device="cuda") / 64).to(torch.bfloat16)
    h_out, h5_out = torch.empty(12, 264, device="cuda"), torch.empty(2, 5, 264, device="cuda")
    calls.append(lambda: gpu.gemm_bf16(12, 264, 4096, h_in, 4096, hm_in, 4096, h_out, 264, stream()))
    calls.append(lambda: gpu.gemm_bf16(5, 264, 4096, h_in, 4096, hm_in, 4096, h5_out[0], 264, stream()))
    calls.append(lambda: gpu.gemm_bf16_ex(0, 0, 5, 264, 4096, h_in, 4096, hn_in, 264, h5_out[1], 264, stream()))
    outs += [h_out, h5_out]

    for f in calls:                          # eager pass: also the first use of every kernel, outside the capture
        gpu.check(f())
    torch.cuda.synchronize()
    eager = [o.clone() for o in outs]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for f in calls:
            gpu.check(f())
    # the same calls dealt to four streams and captured as parallel branches of one graph
    side = [torch.cuda.Stream() for _ in range(4)]
    forked = torch.cuda.CUDAGraph()
    with torch.cuda.graph(forked):
        main = torch.cuda.current_stream()
        for s_ in side:
            s_.wait_stream(main)
        for i, f in enumerate(calls[:-1]):
            with torch.cuda.stream(side[i % 4]):
                gpu.check(f())
        for s_ in side:
            main.wait_stream(s_)
        gpu.check(calls[-1]())
    for g, name in ((graph, "one stream"), (forked, "four streams")):
        for replay in range(3):
            say("graph (%s) replay %d" % (name, replay))
            for o in outs:
                o.fill_(float("nan"))            # eager work between the replays
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            for o, e in zip(outs, eager):
                assert torch.equal(o.view(torch.int32), e.view(torch.int32))


# ---- infinities, NaNs, subnormal numbers ----

def _same_class(got, ref):
    """NaN where the oracle has NaN, the same infinity where it has one, finite elsewhere."""
    return (np.array_equal(np.isnan(got), np.isnan(ref)) and np.array_equal(got == np.inf, ref == np.inf)
            and np.array_equal(got == -np.inf, ref == -np.inf))


def _plant_specials(X, seed, count):
    rng = np.random.default_rng(seed)
    X = X.copy()
    for v in (np.inf, -np.inf, np.nan):
        X[rng.integers(0, X.shape[0], count), rng.integers(0, X.shape[1], count)] = v
    return X


@pytest.mark.parametrize("M,N,K", [(300, 260, 200), (512, 512, 128), (1, 300, 500), (300, 1, 500)])
def test_f32_special_values(gpu, M, N, K):
    # IEEE propagation does not depend on the order of summation: the class of every entry must match the oracle's
    # in every candidate, and the finite entries must still be within the tolerance
    Ai, Bi = inputs.small_ints(0, 11, M, K), inputs.small_ints(0, 12, K, N)
    # a vector operand stays clean: one special value in it would reach every entry of the result
    A, B = (Ai if M == 1 else _plant_specials(Ai, 1, 6)), (Bi if N == 1 else _plant_specials(Bi, 2, 6))
    ref, S = oracle.gemm(A, B)
    assert np.isnan(ref).any() and np.isfinite(ref).any()
    fin = np.isfinite(ref)
    for tile in range(3 + (M == 1 or N == 1)):
        for slices in (1, 3):
            say("f32 specials %dx%dx%d tile %d slices %d" % (M, N, K, tile, slices))
            got = run_cfg(gpu, "f32", tile, slices, 0, 0, A, B)
            assert _same_class(got, ref)
            assert np.array_equal(got[fin].astype(np.float64), ref[fin])          # small integers: exact
    assert _same_class(run_f32(gpu, A, B), ref)
    main_tiles = [t for t, (bm, bn) in MAIN_SHAPES.items() if M >= bm and N >= bn and K % (32 if t == 5 else 4) == 0 and K >= 32]      # the direct-to-LDS shapes that fit
    for tile in main_tiles:
        say("f32 specials %dx%dx%d tile %d" % (M, N, K, tile))
        got = run_cfg(gpu, "f32", tile, 1, 0, 0, A, B)
        assert _same_class(got, ref)
        assert np.array_equal(got[fin].astype(np.float64), ref[fin])
    # subnormal operands and subnormal results are kept, not flushed: scaled small integers stay exact
    for sa, sb in ((2.0 ** -140, 1.0), (2.0 ** -75, 2.0 ** -70)):
        As, Bs = (Ai * np.float32(sa)).astype(np.float32), (Bi * np.float32(sb)).astype(np.float32)
        refs, _ = oracle.gemm(As, Bs)
        assert np.array_equal(run_f32(gpu, As, Bs).astype(np.float64), refs) and np.count_nonzero(refs) > 0
        assert np.array_equal(run_f32_ws(gpu, 0, 0, As, Bs).astype(np.float64), refs)
        for tile in main_tiles[:2]:
            assert np.array_equal(run_cfg(gpu, "f32", tile, 1, 0, 0, As, Bs).astype(np.float64), refs)


def test_bf16_special_values(gpu):
    M, N, K = 512, 520, 192
    Ai, Bti = inputs.bf16_small_ints(4, 60, M, K), inputs.bf16_small_ints(4, 61, N, K)
    A, Bt = Ai.copy(), Bti.copy()
    rng = np.random.default_rng(3)
    for X in (A, Bt):
        for pattern in (0x7F80, 0xFF80, 0x7FC0):                # +inf, -inf, NaN
            X[rng.integers(0, X.shape[0], 5), rng.integers(0, X.shape[1], 5)] = pattern
    B = np.ascontiguousarray(Bt.T)
    ref, _ = oracle.gemm(A, B)
    assert np.isnan(ref).any() and np.isfinite(ref).any()
    fin = np.isfinite(ref)
    for tile in range(4):
        say("bf16 specials tile %d" % tile)
        got = run_cfg(gpu, "bf16", tile, 1, 0, 1, A, B)
        assert _same_class(got, ref) and np.array_equal(got[fin].astype(np.float64), ref[fin])
    got = run_cfg(gpu, "bf16", 2, 3, 0, 1, A, B)
    assert _same_class(got, ref) and np.array_equal(got[fin].astype(np.float64), ref[fin])
    # subnormal bf16 operands (small integers times 2^-130) are kept
    Af = (Ai.astype(np.uint32) << 16).view(np.float32)
    Ad = ((Af * np.float32(2.0 ** -130)).view(np.uint32) >> 16).astype(np.uint16)
    refd, _ = oracle.gemm(Ad, np.ascontiguousarray(Bti.T))
    assert np.count_nonzero(refd) > 0
    assert np.array_equal(run_bf16(gpu, Ad, Bti).astype(np.float64), refd)


# ---- a vector on one side: the streaming kernels ----

@pytest.mark.parametrize("M,N,K", [(1, 1000, 3000), (1000, 1, 3000), (1, 4096, 4096), (4096, 1, 4096), (1, 1, 100000),
                                   (1, 33, 7), (31, 1, 1), (1, 5000, 1027), (4100, 1, 2050), (1, 64, 65536)])
def test_f32_vector_shapes(gpu, M, N, K):
    A, B = inputs.uniform_pm1(14, 1, M, K), inputs.uniform_pm1(14, 2, K, N)
    ref, S = oracle.gemm(A, B)
    for ta, tb in [(0, 0)] + LAYOUTS:
        say("f32 vector %dx%dx%d storage %d%d" % (M, N, K, ta, tb))
        assert gpu.fsrgemm_plan_f32(ta, tb, M, N, K, 0x1000, M if ta else K, 0x1000, K if tb else N)[0] == 3
        got = run_f32_ex(gpu, ta, tb, A, B, repeat=2)                                        # tight: vector loads where rows are aligned
        assert oracle.componentwise_error(got, ref, S) <= TOL_F32
        lda, ldb = (M if ta else K) + 3, (K if tb else N) + 5
        got = run_f32_ex(gpu, ta, tb, A, B, lda=lda, ldb=ldb, ldc=N + 2, offset=1, repeat=2)  # padded, 4-byte aligned only
        assert oracle.componentwise_error(got, ref, S) <= TOL_F32
        got = run_f32_ws(gpu, ta, tb, A, B, repeat=2)                                        # with the workspace the library asks for
        assert oracle.componentwise_error(got, ref, S) <= TOL_F32
        lda, ldb = (M if ta else K), (K if tb else N)
        got = run_f32_ws(gpu, ta, tb, A, B, lda=lda + (-lda) % 4 + 4, ldb=ldb + (-ldb) % 4 + 4, ldc=N + 1, repeat=2)
        assert oracle.componentwise_error(got, ref, S) <= TOL_F32
    Ai, Bi = inputs.small_ints(0, 9, M, K), inputs.small_ints(0, 10, K, N)
    if K <= 4097:
        refi, _ = oracle.gemm(Ai, Bi)
        for ta, tb in [(0, 0)] + LAYOUTS:
            assert np.array_equal(run_f32_ws(gpu, ta, tb, Ai, Bi).astype(np.float64), refi)


@pytest.mark.parametrize("M,N,K", [(1, 1000, 3000), (1000, 1, 3000), (1, 4096, 4096), (4096, 1, 4096), (1, 1, 100000),
                                   (1, 70, 9), (31, 1, 1), (1, 5000, 1032), (4104, 1, 2051), (1, 128, 65536)])
def test_bf16_vector_shapes(gpu, M, N, K):
    A = inputs.bf16_normal_scaled(17, 1, M, K, 1 / math.sqrt(K))
    B = inputs.bf16_normal_scaled(17, 2, K, N, 1 / math.sqrt(K))
    ref, S = oracle.gemm(A, B)
    for ta, tb in [(0, 0)] + LAYOUTS:
        say("bf16 vector %dx%dx%d storage %d%d" % (M, N, K, ta, tb))
        assert gpu.fsrgemm_plan_bf16(ta, tb, M, N, K, 0x1000, M if ta else K, 0x1000, K if tb else N)[0] == 4
        got = run_bf16_ex(gpu, ta, tb, A, B, repeat=2)
        assert oracle.componentwise_error(got, ref, S) <= TOL_BF16
        lda, ldb = (M if ta else K) + 3, (K if tb else N) + 5
        got = run_bf16_ex(gpu, ta, tb, A, B, lda=lda, ldb=ldb, ldc=N + 2, offset=1, repeat=2)      # 2-byte aligned only
        assert oracle.componentwise_error(got, ref, S) <= TOL_BF16
        got = run_bf16_ws(gpu, ta, tb, A, B, repeat=2)
        assert oracle.componentwise_error(got, ref, S) <= TOL_BF16
        lda, ldb = (M if ta else K), (K if tb else N)
        got = run_bf16_ws(gpu, ta, tb, A, B, lda=lda + (-lda) % 8 + 8, ldb=ldb + (-ldb) % 8 + 8, ldc=N + 1, repeat=2)
        assert oracle.componentwise_error(got, ref, S) <= TOL_BF16
        for slices in (2, 7, 64):
            if slices <= -(-K // 64):
                got = run_cfg(gpu, "bf16", 4, slices, ta, tb, A, B, repeat=2)
                assert oracle.componentwise_error(got, ref, S) <= TOL_BF16
    if K <= 4097:
        Ai, Bi = inputs.bf16_small_ints(4, 70, M, K), inputs.bf16_small_ints(4, 71, K, N)
        refi, _ = oracle.gemm(Ai, Bi)
        for ta, tb in [(0, 0)] + LAYOUTS:
            assert np.array_equal(run_bf16_ws(gpu, ta, tb, Ai, Bi).astype(np.float64), refi)
    with pytest.raises(gpu.FsrGemmError):       # 17 rows and 17 columns: no vector side
        run_cfg(gpu, "bf16", 4, 1, 0, 1, inputs.bf16_small_ints(4, 72, 17, 64), inputs.bf16_small_ints(4, 73, 64, 17))
    with pytest.raises(gpu.FsrGemmError):       # nine and nine, and not the storage the matrix-core kernel takes
        run_cfg(gpu, "bf16", 4, 1, 0, 0, inputs.bf16_small_ints(4, 72, 9, 64), inputs.bf16_small_ints(4, 73, 64, 9))


def test_f32_vector_every_slice_count(gpu):
    M, N, K = 1, 700, 3000
    A, B = inputs.uniform_pm1(14, 3, M, K), inputs.uniform_pm1(14, 4, K, N)
    ref, S = oracle.gemm(A, B)
    for ta, tb in [(0, 0)] + LAYOUTS:
        for slices in (1, 2, 3, 7, 64):
            say("f32 vector candidate, %d slices, storage %d%d" % (slices, ta, tb))
            assert oracle.componentwise_error(run_cfg(gpu, "f32", 3, slices, ta, tb, A, B, repeat=2), ref, S) <= TOL_F32
            assert oracle.componentwise_error(run_cfg(gpu, "f32", 3, slices, ta, tb, B.T.copy(), A.T.copy(), repeat=2), ref.T, S.T) <= TOL_F32
    with pytest.raises(gpu.FsrGemmError):       # 17 rows and 17 columns: no vector side
        run_cfg(gpu, "f32", 3, 1, 0, 0, inputs.uniform_pm1(14, 5, 17, 64), inputs.uniform_pm1(14, 6, 64, 17))


# ---- a few vectors on one side (2 .. 8 rows or columns): the streaming kernels with the vectors staged in LDS ----

def _ceil4(n):
    return n + (-n) % 4


FEW_SHAPES = [(8, 1000, 777), (3, 513, 2050), (2, 64, 9), (5, 36, 1300), (1000, 8, 777), (516, 3, 2050), (7, 4100, 5000),
              (4, 4, 4096), (8, 8, 600), (6, 2049, 515), (2050, 5, 1027), (2, 4, 1), (8, 31, 3), (3, 3, 50),
              (16, 1000, 777), (13, 513, 2050), (1000, 12, 777), (9, 4100, 5000), (16, 16, 300), (11, 40, 9)]


@pytest.mark.parametrize("M,N,K", FEW_SHAPES)
def test_f32_few_vector_shapes(gpu, M, N, K):
    A, B = inputs.uniform_pm1(15, 1, M, K), inputs.uniform_pm1(15, 2, K, N)
    ref, S = oracle.gemm(A, B)
    Ai, Bi = inputs.small_ints(0, 13, M, K), inputs.small_ints(0, 14, K, N)
    refi, _ = oracle.gemm(Ai, Bi)
    for ta, tb in [(0, 0)] + LAYOUTS:
        lda, ldb = _ceil4(M if ta else K), _ceil4(K if tb else N)            # rows of whole 16-byte pieces
        name = gpu.fsrgemm_kernel_for_f32_ex(ta, tb, M, N, K, P_FAKE, lda, P_FAKE, ldb, P_FAKE, N)
        say("f32 few vectors %dx%dx%d storage %d%d -> %s" % (M, N, K, ta, tb, name))
        # the streamed operand is the larger side; where it is walked along its columns it needs four of them
        cols = (ta if N <= M else not tb)
        assert ("few_kernel" in name) == (not cols or max(M, N) >= 4), name
        got = run_f32_ex(gpu, ta, tb, A, B, lda=lda, ldb=ldb, ldc=N + 3, repeat=2)
        assert oracle.componentwise_error(got, ref, S) <= TOL_F32
        got = run_f32_ws(gpu, ta, tb, A, B, lda=lda + 4, ldb=ldb + 8, repeat=2)            # with the workspace the library asks for
        assert oracle.componentwise_error(got, ref, S) <= TOL_F32
        # 4-byte aligned only: the same kernels (their 16-byte loads are issued from any element-aligned address)
        got = run_f32_ex(gpu, ta, tb, A, B, lda=lda + 1, ldb=ldb + 3, offset=1, repeat=2)
        assert oracle.componentwise_error(got, ref, S) <= TOL_F32
        name = gpu.fsrgemm_kernel_for_f32_ex(ta, tb, M, N, K, P_FAKE + 4, lda + 1, P_FAKE + 4, ldb + 3, P_FAKE, N)
        assert ("few_kernel" in name) == (not cols or max(M, N) >= 4), name
        if K <= 4097:
            assert np.array_equal(run_f32_ws(gpu, ta, tb, Ai, Bi, lda=lda, ldb=ldb).astype(np.float64), refi)
            assert np.array_equal(run_f32_ex(gpu, ta, tb, Ai, Bi, lda=lda, ldb=ldb).astype(np.float64), refi)


def test_f32_few_vectors_every_count_and_slice_count(gpu):
    # 2 .. 16 vectors on either side through the vector candidate with 1 .. 64 K slices (slices of a few elements, empty
    # slices, a last chunk that is not whole), every storage order
    K = 1500
    for nvec in range(2, 17):
        A, B = inputs.uniform_pm1(15, 10 + nvec, nvec, K), inputs.uniform_pm1(15, 20 + nvec, K, 332)
        ref, S = oracle.gemm(A, B)
        for ta, tb in [(0, 0)] + LAYOUTS:
            for slices in (1, 2, 3, 7, 64):
                say("f32 vector candidate, %d vectors, %d slices, storage %d%d" % (nvec, slices, ta, tb))
                kw = dict(lda=_ceil4(nvec if ta else K), ldb=_ceil4(K if tb else 332), repeat=2)
                assert oracle.componentwise_error(run_cfg(gpu, "f32", 3, slices, ta, tb, A, B, **kw), ref, S) <= TOL_F32
                kw = dict(lda=_ceil4(332 if ta else K), ldb=_ceil4(K if tb else nvec), repeat=2)
                assert oracle.componentwise_error(run_cfg(gpu, "f32", 3, slices, ta, tb, B.T.copy(), A.T.copy(), **kw), ref.T, S.T) <= TOL_F32


def _ceil8(n):
    return n + (-n) % 8


@pytest.mark.parametrize("M,N,K", [(8, 1000, 777), (3, 520, 2050), (2, 64, 9), (5, 40, 1300), (1000, 8, 777), (516, 3, 2050),
                                   (7, 4100, 5000), (4, 8, 4096), (8, 8, 600), (6, 2049, 515), (2050, 5, 1027), (2, 8, 1),
                                   (8, 63, 3), (3, 7, 50)])
def test_bf16_few_vector_shapes(gpu, M, N, K):
    A = inputs.bf16_normal_scaled(19, 1, M, K, 1 / math.sqrt(K))
    B = inputs.bf16_normal_scaled(19, 2, K, N, 1 / math.sqrt(K))
    ref, S = oracle.gemm(A, B)
    Ai, Bi = inputs.bf16_small_ints(4, 74, M, K), inputs.bf16_small_ints(4, 75, K, N)
    refi, _ = oracle.gemm(Ai, Bi)
    for ta, tb in [(0, 1), (0, 0), (1, 0), (1, 1)]:
        lda, ldb = _ceil8(M if ta else K), _ceil8(K if tb else N)            # rows of whole 16-byte pieces
        name = gpu.fsrgemm_kernel_for_bf16_ex(ta, tb, M, N, K, P_FAKE, lda, P_FAKE, ldb, P_FAKE, N)
        say("bf16 few vectors %dx%dx%d storage %d%d -> %s" % (M, N, K, ta, tb, name))
        cols = (ta if N <= M else not tb)                    # the streamed operand walked along its columns needs eight of them
        assert ("few_kernel" in name or "_mfma_" in name) == (not cols or max(M, N) >= 8), name
        assert ("_mfma_" in name) == ((ta, tb) == (0, 1) and K % 8 == 0), name       # both sides contiguous along k, whole pieces
        got = run_bf16_ex(gpu, ta, tb, A, B, lda=lda, ldb=ldb, ldc=N + 3, repeat=2)
        assert oracle.componentwise_error(got, ref, S) <= 1e-5
        got = run_bf16_ws(gpu, ta, tb, A, B, lda=lda + 8, ldb=ldb + 16, repeat=2)            # with the workspace the library asks for
        assert oracle.componentwise_error(got, ref, S) <= 1e-5
        # 2-byte aligned only: the lane-arithmetic kernels (their 16-byte loads are issued from any element-aligned address)
        got = run_bf16_ex(gpu, ta, tb, A, B, lda=lda + 1, ldb=ldb + 3, offset=1, repeat=2)
        assert oracle.componentwise_error(got, ref, S) <= 1e-5
        name = gpu.fsrgemm_kernel_for_bf16_ex(ta, tb, M, N, K, P_FAKE + 2, lda + 1, P_FAKE + 2, ldb + 3, P_FAKE, N)
        assert ("few_kernel" in name) == ((not cols or max(M, N) >= 8) and min(M, N) <= 8), name
        for slices in (1, 2, 7, 64):
            if slices <= -(-K // 64) and "gemv_" in name:
                got = run_cfg(gpu, "bf16", 4, slices, ta, tb, A, B, lda=lda, ldb=ldb, repeat=2)
                assert oracle.componentwise_error(got, ref, S) <= 1e-5
        if K <= 4097:
            assert np.array_equal(run_bf16_ws(gpu, ta, tb, Ai, Bi, lda=lda, ldb=ldb).astype(np.float64), refi)
            assert np.array_equal(run_bf16_ex(gpu, ta, tb, Ai, Bi, lda=lda, ldb=ldb).astype(np.float64), refi)


@pytest.mark.parametrize("M,N,K", [(16, 1000, 776), (13, 520, 2056), (16, 16, 64), (9, 33, 8), (1000, 16, 1000), (1001, 11, 4104),
                                   (2, 8200, 256), (16, 17, 8192), (10, 300, 1032), (8, 1000, 776), (5, 33, 8), (3, 700, 3080),
                                   (9, 40, 1024), (16, 31, 1096), (11, 100, 2048)])
def test_bf16_up_to_16_vectors_on_the_matrix_cores(gpu, M, N, K):
    # row-major A against column-major B with up to 16 rows or columns on one side: the matrix-core streaming kernel,
    # through the plain entry point, with the workspace the library asks for, and as the vector candidate in 1 .. 64 K slices
    A = inputs.bf16_normal_scaled(21, 1, M, K, 1 / math.sqrt(K))
    B = inputs.bf16_normal_scaled(21, 2, K, N, 1 / math.sqrt(K))
    ref, S = oracle.gemm(A, B)
    for pad in (0, 8):
        lda, ldb = K + pad, K + 2 * pad
        assert gpu.fsrgemm_kernel_for_bf16_ex(0, 1, M, N, K, P_FAKE, lda, P_FAKE, ldb, P_FAKE, N) == ("gemv_rows_bf16_mfma_direct_kernel" if min(M, N) <= 8 else "gemv_rows_bf16_mfma_kernel")
        say("bf16 matrix-core vectors %dx%dx%d, leading dimensions %d %d" % (M, N, K, lda, ldb))
        got = run_bf16_ex(gpu, 0, 1, A, B, lda=lda, ldb=ldb, ldc=N + pad // 2, repeat=2)
        assert oracle.componentwise_error(got, ref, S) <= 1e-5
        got = run_bf16_ws(gpu, 0, 1, A, B, lda=lda, ldb=ldb, repeat=2)
        assert oracle.componentwise_error(got, ref, S) <= 1e-5
        for slices in (1, 2, 3, 7, 64):
            if slices <= -(-K // 64):
                got = run_cfg(gpu, "bf16", 4, slices, 0, 1, A, B, lda=lda, ldb=ldb, repeat=2)
                assert oracle.componentwise_error(got, ref, S) <= 1e-5
    if K <= 4104:
        Ai, Bi = inputs.bf16_small_ints(4, 78, M, K), inputs.bf16_small_ints(4, 79, K, N)
        refi, _ = oracle.gemm(Ai, Bi)
        assert np.array_equal(run_bf16_ex(gpu, 0, 1, Ai, Bi).astype(np.float64), refi)
        assert np.array_equal(run_cfg(gpu, "bf16", 4, min(3, -(-K // 64)), 0, 1, Ai, Bi).astype(np.float64), refi)


@pytest.mark.parametrize("M,N,K", [(8, 300, 700), (300, 5, 700), (3, 136, 515), (12, 300, 704), (300, 16, 520)])
def test_bf16_few_vectors_special_values(gpu, M, N, K):
    # infinities and NaNs in the streamed matrix, among them its last row and column (which the kernels read again in
    # place of pieces outside the matrix): the class of every entry must match the oracle's
    Ai, Bi = inputs.bf16_small_ints(4, 76, M, K), inputs.bf16_small_ints(4, 77, K, N)
    mat = (Bi if M <= N else Ai).copy()
    rng = np.random.default_rng(5)
    for pattern in (0x7F80, 0xFF80, 0x7FC0):                # +inf, -inf, NaN
        mat[rng.integers(0, mat.shape[0], 5), rng.integers(0, mat.shape[1], 5)] = pattern
    mat[-1, -1], mat[-1, 0], mat[0, -1] = 0x7F80, 0x7FC0, 0xFF80
    A, B = (Ai, mat) if M <= N else (mat, Bi)
    ref, _ = oracle.gemm(A, B)
    assert np.isnan(ref).any() and np.isfinite(ref).any()
    fin = np.isfinite(ref)
    for ta, tb in [(0, 1), (0, 0), (1, 0), (1, 1)]:
        if min(M, N) > 8 and (ta, tb) != (0, 1):
            continue                # more than 8 vectors: only in the storage the matrix-core kernel takes
        kw = dict(lda=_ceil8(M if ta else K), ldb=_ceil8(K if tb else N))
        for slices in (1, 3):
            say("bf16 few vectors, specials, %dx%dx%d storage %d%d, %d slices" % (M, N, K, ta, tb, slices))
            got = run_cfg(gpu, "bf16", 4, slices, ta, tb, A, B, **kw)
            assert _same_class(got, ref)
            assert np.array_equal(got[fin].astype(np.float64), ref[fin])          # small integers: exact
        assert _same_class(run_bf16_ex(gpu, ta, tb, A, B, **kw), ref)


def test_bf16_few_vectors_every_count(gpu):
    # 2 .. 8 vectors on either side through the vector candidate, 1 and 3 K slices, every storage order (K = 1500: no
    # whole 16-byte pieces, so the lane-arithmetic kernels everywhere), and 2 .. 16 on the matrix cores (K = 1504)
    for nvec in range(2, 17):
        K = 1504
        A = inputs.bf16_normal_scaled(19, 40 + nvec, nvec, K, 1 / math.sqrt(K))
        B = inputs.bf16_normal_scaled(19, 60 + nvec, K, 330, 1 / math.sqrt(K))
        ref, S = oracle.gemm(A, B)
        for slices in (1, 3):
            say("bf16 vector candidate on the matrix cores, %d vectors, %d slices" % (nvec, slices))
            assert oracle.componentwise_error(run_cfg(gpu, "bf16", 4, slices, 0, 1, A, B, repeat=2), ref, S) <= 1e-5
            assert oracle.componentwise_error(run_cfg(gpu, "bf16", 4, slices, 0, 1, B.T.copy(), A.T.copy(), repeat=2), ref.T, S.T) <= 1e-5
    K = 1500
    for nvec in range(2, 9):
        A = inputs.bf16_normal_scaled(19, 10 + nvec, nvec, K, 1 / math.sqrt(K))
        B = inputs.bf16_normal_scaled(19, 20 + nvec, K, 328, 1 / math.sqrt(K))
        ref, S = oracle.gemm(A, B)
        for ta, tb in [(0, 1), (0, 0), (1, 0), (1, 1)]:
            for slices in (1, 3):
                say("bf16 vector candidate, %d vectors, %d slices, storage %d%d" % (nvec, slices, ta, tb))
                kw = dict(lda=_ceil8(nvec if ta else K), ldb=_ceil8(K if tb else 328), repeat=2)
                assert oracle.componentwise_error(run_cfg(gpu, "bf16", 4, slices, ta, tb, A, B, **kw), ref, S) <= 1e-5
                kw = dict(lda=_ceil8(328 if ta else K), ldb=_ceil8(K if tb else nvec), repeat=2)
                assert oracle.componentwise_error(run_cfg(gpu, "bf16", 4, slices, ta, tb, B.T.copy(), A.T.copy(), **kw), ref.T, S.T) <= 1e-5


@pytest.mark.parametrize("M,N,K", [(8, 300, 700), (300, 5, 700), (3, 132, 515), (12, 300, 700), (300, 16, 515)])
def test_f32_few_vectors_special_values(gpu, M, N, K):
    # infinities and NaNs in the streamed matrix, among them its last row and column (which the kernels read again in
    # place of pieces outside the matrix): the class of every entry must match the oracle's
    Ai, Bi = inputs.small_ints(0, 15, M, K), inputs.small_ints(0, 16, K, N)
    mat = Bi if M <= N else Ai
    mat = _plant_specials(mat, 3, 5)
    mat[-1, -1], mat[-1, 0], mat[0, -1] = np.inf, np.nan, -np.inf
    A, B = (Ai, mat) if M <= N else (mat, Bi)
    ref, S = oracle.gemm(A, B)
    assert np.isnan(ref).any() and np.isfinite(ref).any()
    fin = np.isfinite(ref)
    for ta, tb in [(0, 0)] + LAYOUTS:
        kw = dict(lda=_ceil4(M if ta else K), ldb=_ceil4(K if tb else N))
        for slices in (1, 3):
            say("f32 few vectors, specials, %dx%dx%d storage %d%d, %d slices" % (M, N, K, ta, tb, slices))
            got = run_cfg(gpu, "f32", 3, slices, ta, tb, A, B, **kw)
            assert _same_class(got, ref)
            assert np.array_equal(got[fin].astype(np.float64), ref[fin])          # small integers: exact
        assert _same_class(run_f32_ex(gpu, ta, tb, A, B, **kw), ref)


# ---- small results of long sums (the normal equations of the paper's Task 20) ----

@pytest.mark.parametrize("M,N,K", [(10, 10, 1 << 14), (10, 1, 1 << 16), (1, 1, 100003), (16, 8, 5000), (7, 16, 4097),
                                   (12, 12, 8192), (3, 5, 70000), (4, 4, 4096), (9, 8, 5000)])
def test_f32_small_result_long_sum(gpu, M, N, K):
    A, B = inputs.uniform_pm1(16, 1, M, K), inputs.uniform_pm1(16, 2, K, N)
    ref, S = oracle.gemm(A, B)
    for ta, tb in [(0, 0)] + LAYOUTS:
        say("f32 small result %dx%dx%d storage %d%d" % (M, N, K, ta, tb))
        # the dedicated kernel takes operands stored with k as the row index (a transposed A, a row-major B; a vector
        # is that in either order)
        tall = bool((ta or M == 1) and (not tb or N == 1))
        assert (gpu.fsrgemm_plan_f32(ta, tb, M, N, K, 0x1000, M if ta else K, 0x1000, K if tb else N, True)[0] == 4) == tall
        got = run_f32_ws(gpu, ta, tb, A, B, repeat=2)                   # the dispatcher's choice, canaried workspace of the size it asks for
        assert oracle.componentwise_error(got, ref, S) <= TOL_F32
        lda, ldb = (M if ta else K) + 3, (K if tb else N) + 2
        got = run_f32_ws(gpu, ta, tb, A, B, lda=lda, ldb=ldb, ldc=N + 3, offset=1, repeat=2)
        assert oracle.componentwise_error(got, ref, S) <= TOL_F32
        for parts in (1, 3, 256):
            if tall:
                got = run_cfg(gpu, "f32", 4, parts, ta, tb, A, B, repeat=2)
                assert oracle.componentwise_error(got, ref, S) <= TOL_F32
            else:
                with pytest.raises(gpu.FsrGemmError):
                    run_cfg(gpu, "f32", 4, parts, ta, tb, A, B)
    if K <= 4097:
        Ai, Bi = inputs.small_ints(0, 13, M, K), inputs.small_ints(0, 14, K, N)
        assert np.array_equal(run_f32_ws(gpu, 1, 0, Ai, Bi).astype(np.float64), oracle.gemm(Ai, Bi)[0])
    with pytest.raises(gpu.FsrGemmError):
        run_cfg(gpu, "f32", 4, 4, 1, 0, inputs.uniform_pm1(16, 3, 17, 64), inputs.uniform_pm1(16, 4, 64, 4))


def test_f32_normal_equations(gpu):
    # X^T X and X^T y for a tall X (the paper's Task 20 at its smallest size), A and B the same buffer for the first
    import torch

    n, f = 1 << 14, 10
    X, y = inputs.uniform_pm1(16, 5, n, f), inputs.uniform_pm1(16, 6, n, 1)
    refG, SG = oracle.gemm(np.ascontiguousarray(X.T), X)
    refg, Sg = oracle.gemm(np.ascontiguousarray(X.T), y)
    xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    G, g = torch.full((f, f), float("nan"), device="cuda"), torch.full((f, 1), float("nan"), device="cuda")
    need = max(gpu.gemm_f32_workspace_bytes(1, 0, f, f, n), gpu.gemm_f32_workspace_bytes(1, 0, f, 1, n))
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    gpu.check(gpu.gemm_f32_ws(1, 0, f, f, n, xd, f, xd, f, G, f, ws, need, st))
    gpu.check(gpu.gemm_f32_ws(1, 0, f, 1, n, xd, f, yd, 1, g, 1, ws, need, st))
    torch.cuda.synchronize()
    assert oracle.componentwise_error(G.cpu().numpy(), refG, SG) <= TOL_F32
    assert oracle.componentwise_error(g.cpu().numpy(), refg, Sg) <= TOL_F32
    assert np.array_equal(G.cpu().numpy(), G.cpu().numpy().T)            # the same sums in the same order on both sides of the diagonal
    assert np.array_equal(run_f32_ws(gpu, 1, 0, np.ascontiguousarray(X.T), X).view(np.uint32), G.cpu().numpy().view(np.uint32))   # separate buffers: same bits


# ---- forced configurations: every candidate of the selection loop is a correct product ----

@pytest.mark.parametrize("shape,ta,tb", [((300, 520, 1000), 0, 0), ((512, 384, 2048), 0, 0), ((64, 64, 4097), 0, 0),
                                         ((1, 700, 3000), 0, 0), ((257, 129, 640), 1, 1), ((40, 1000, 512), 0, 1)])
def test_f32_every_candidate(gpu, shape, ta, tb):
    M, N, K = shape
    A, B = inputs.uniform_pm1(12, 1, M, K), inputs.uniform_pm1(12, 2, K, N)
    ref, S = oracle.gemm(A, B)
    for tile in range(3 + (M == 1 or N == 1)):          # the three tile configurations, and the vector kernels where they apply
        for slices in (1, 2, 5, 16, 64):
            say("f32 candidate tile %d slices %d on %dx%dx%d %d%d" % (tile, slices, M, N, K, ta, tb))
            if slices > 1 and (slices > -(-K // 16) or slices * M * N * 4 > 16 << 20):
                continue
            got = run_cfg(gpu, "f32", tile, slices, ta, tb, A, B, repeat=2)
            assert oracle.componentwise_error(got, ref, S) <= TOL_F32
    # padded, offset operands through a split
    got = run_cfg(gpu, "f32", 1, 3, ta, tb, A, B, lda=(M if ta else K) + 3, ldb=(K if tb else N) + 5, ldc=N + 7, offset=1)
    assert oracle.componentwise_error(got, ref, S) <= TOL_F32


@pytest.mark.parametrize("shape,ta,tb", [((300, 520, 1000), 0, 1), ((512, 512, 2048), 0, 1), ((64, 64, 4160), 0, 1),
                                         ((16, 1000, 4096), 0, 1), ((264, 256, 640), 1, 0), ((512, 768, 1024), 0, 0)])
def test_bf16_every_candidate(gpu, shape, ta, tb):
    M, N, K = shape
    A, Bt = inputs.bf16_normal_scaled(12, 3, M, K, 1 / math.sqrt(K)), inputs.bf16_normal_scaled(12, 4, N, K, 1 / math.sqrt(K))
    B = np.ascontiguousarray(Bt.T)
    ref, S = oracle.gemm(A, B)
    fits_main = M >= 256 and N >= 256 and K >= 64 and K % 8 == 0 and (not ta or M % 8 == 0) and (tb or N % 8 == 0)
    for tile in range(4):
        for slices in (1, 2, 5, 16, 64):
            say("bf16 candidate tile %d slices %d on %dx%dx%d %d%d" % (tile, slices, M, N, K, ta, tb))
            if slices > 1 and (slices > -(-K // 64) or slices * M * N * 4 > 16 << 20):
                continue
            per = -(-(-(-K // 64)) // slices) * 64                 # the direct-to-LDS kernel's slices: whole K-tiles, none left without one
            if tile == 0 and (not fits_main or (slices - 1) * per + 64 > K):
                with pytest.raises(gpu.FsrGemmError):
                    run_cfg(gpu, "bf16", tile, slices, ta, tb, A, B)
                continue
            got = run_cfg(gpu, "bf16", tile, slices, ta, tb, A, B, repeat=2)
            assert oracle.componentwise_error(got, ref, S) <= TOL_BF16


@pytest.mark.parametrize("ta,tb", [(0, 0)] + LAYOUTS)
def test_every_compiled_kernel_instance(gpu, ta, tb):
    # every tile configuration in each of its three load modes (unchecked vectors / vectors with checked edges /
    # element-wise), for this storage pair, both precisions: 9 fp32 and 9 bf16 general kernels plus the
    # two direct-to-LDS ones per parametrisation
    M, N = 520, 392                                     # not multiples of any tile: shifted last tiles everywhere
    # unchecked: K a multiple of the K-tile (16 fp32, 64 bf16); checked edges: it is not, but rows stay 16-byte aligned
    for K, aligned, mode in ((128, True, "unchecked"), (104, True, "checked edges"), (100, False, "element-wise")):
        A, B = inputs.uniform_pm1(15, 1, M, K), inputs.uniform_pm1(15, 2, K, N)
        ref, S = oracle.gemm(A, B)
        Ah = inputs.bf16_normal_scaled(15, 3, M, K, 1 / math.sqrt(K))
        Bh = np.ascontiguousarray(inputs.bf16_normal_scaled(15, 4, N, K, 1 / math.sqrt(K)).T)
        refh, Sh = oracle.gemm(Ah, Bh)
        lda, ldb = (M if ta else K), (K if tb else N)
        kw = dict(lda=lda + 8, ldb=ldb + 8, ldc=N + 3, offset=0) if aligned else dict(lda=lda + 3, ldb=ldb + 1, ldc=N + 1, offset=1)
        # the names the library gives these candidates: <.., load mode, A layout, B layout>
        base, m = (0x1000 if aligned else 0x1004), ("unchecked", "checked edges", "element-wise").index(mode)
        for tile, shape in enumerate(("4, 2, 2", "2, 2, 3", "1, 1, 4")):
            assert gpu.fsrgemm_kernel_for_f32_cfg(tile, ta, tb, M, N, K, base, kw["lda"], base, kw["ldb"], 0x1000, kw["ldc"]) == \
                "gemm_f32_kernel<%s, %d, %d, %d>" % (shape, m, ta, 1 - tb)
        base = 0x1000 if aligned else 0x1002
        for tile, shape in ((1, "4, 1"), (2, "2, 2"), (3, "1, 4")):
            assert gpu.fsrgemm_kernel_for_bf16_cfg(tile, ta, tb, M, N, K, base, kw["lda"], base, kw["ldb"], 0x1000, kw["ldc"]) == \
                "gemm_bf16_kernel<%s, %d, %d, %d>" % (shape, m, ta, 1 - tb)
        for tile in range(3):
            say("f32 tile %d, %s, storage %d%d" % (tile, mode, ta, tb))
            got = run_cfg(gpu, "f32", tile, 1, ta, tb, A, B, repeat=2, **kw)
            assert oracle.componentwise_error(got, ref, S) <= TOL_F32
        for tile in (1, 2, 3):
            say("bf16 tile %d, %s, storage %d%d" % (tile, mode, ta, tb))
            got = run_cfg(gpu, "bf16", tile, 1, ta, tb, Ah, Bh, repeat=2, **kw)
            assert oracle.componentwise_error(got, refh, Sh) <= TOL_BF16
    K = 128
    A, B = inputs.uniform_pm1(15, 7, M, K), inputs.uniform_pm1(15, 8, K, N)
    ref, S = oracle.gemm(A, B)
    say("f32 tile 5, storage %d%d" % (ta, tb))
    got = run_cfg(gpu, "f32", 5, 1, ta, tb, A, B, ldc=N + 3, repeat=2)
    assert oracle.componentwise_error(got, ref, S) <= TOL_F32
    Ah = inputs.bf16_normal_scaled(15, 5, M, K, 1 / math.sqrt(K))
    Bh = np.ascontiguousarray(inputs.bf16_normal_scaled(15, 6, N, K, 1 / math.sqrt(K)).T)
    refh, Sh = oracle.gemm(Ah, Bh)
    say("bf16 tile 0, storage %d%d" % (ta, tb))
    got = run_cfg(gpu, "bf16", 0, 1, ta, tb, Ah, Bh, ldc=N + 3, repeat=2)
    assert oracle.componentwise_error(got, refh, Sh) <= TOL_BF16


def test_forced_plan_equals_dispatch(gpu):
    # the dispatcher's own choice, forced, gives the dispatcher's bits (fp32 and bf16, plain and with a workspace)
    for M, N, K in ((300, 520, 1000), (64, 64, 4097), (1, 4096, 4096)):
        A, B = inputs.uniform_pm1(12, 5, M, K), inputs.uniform_pm1(12, 6, K, N)
        tile, slices = gpu.fsrgemm_plan_f32(0, 0, M, N, K, 0x1000, K, 0x1000, N, True)
        assert np.array_equal(run_cfg(gpu, "f32", tile, slices, 0, 0, A, B).view(np.uint32), run_f32_ws(gpu, 0, 0, A, B).view(np.uint32))
        tile, slices = gpu.fsrgemm_plan_f32(0, 0, M, N, K, 0x1000, K, 0x1000, N, False)
        assert slices == 1
        assert np.array_equal(run_cfg(gpu, "f32", tile, 1, 0, 0, A, B).view(np.uint32), run_f32(gpu, A, B).view(np.uint32))
    for M, N, K in ((512, 512, 512), (16, 1024, 8192)):
        A, Bt = inputs.bf16_normal_scaled(12, 7, M, K, 1 / math.sqrt(K)), inputs.bf16_normal_scaled(12, 8, N, K, 1 / math.sqrt(K))
        B = np.ascontiguousarray(Bt.T)
        tile, slices = gpu.fsrgemm_plan_bf16(0, 1, M, N, K, 0x1000, K, 0x1000, K, True)
        assert np.array_equal(run_cfg(gpu, "bf16", tile, slices, 0, 1, A, B).view(np.uint32), run_bf16_ws(gpu, 0, 1, A, B).view(np.uint32))


def test_tuned_table_rows_validate(gpu):
    # every problem with a row in the dispatcher's table, through the public entry point that the row serves
    import os
    import re

    path = os.path.join(os.path.dirname(gpu.library_path()), "csrc", "tuned_table.inc")
    rows = [tuple(int(x) for x in m.groups()) for m in re.finditer(r"^\s*\{(\d+), (\d+), (\d+), (\d+), (\d+), (\d+), (\d+), (\d+), (\d+)\},", open(path).read(), re.M)]
    for kind, ta, tb, M, N, K, ws, tile, slices in rows:
        say("table row %s" % ((kind, ta, tb, M, N, K, ws, tile, slices),))
        if M * N * K > 1 << 34:
            continue                                    # larger problems are covered by the full-size tests
        if kind == 0:
            A, B = inputs.uniform_pm1(13, 1, M, K), inputs.uniform_pm1(13, 2, K, N)
            got = run_f32_ws(gpu, ta, tb, A, B, repeat=2) if ws else run_f32_ex(gpu, ta, tb, A, B, repeat=2)
            tol = TOL_F32
        else:
            A = inputs.bf16_normal_scaled(13, 3, M, K, 1 / math.sqrt(K))
            B = np.ascontiguousarray(inputs.bf16_normal_scaled(13, 4, N, K, 1 / math.sqrt(K)).T)
            got = run_bf16_ws(gpu, ta, tb, A, B, repeat=2) if ws else run_bf16_ex(gpu, ta, tb, A, B, repeat=2)
            tol = TOL_BF16
        rng = np.random.default_rng(13)
        ii, jj = rng.integers(0, M, 4096), rng.integers(0, N, 4096)
        ref, S = oracle.gemm_entries(A, B, ii, jj)
        assert np.all(np.isfinite(got)) and oracle.componentwise_error(got[ii, jj], ref, S) <= tol


def _check_transpose(gpu, A, **kw):
    got = run_transpose(gpu, A, **kw)
    assert np.array_equal(got.view(np.uint32), oracle.transpose(A).view(np.uint32))


@pytest.mark.parametrize("shape", [(1, 1), (1, 5000), (5000, 1), (63, 5), (64, 64), (65, 64), (64, 127), (100, 300),
                                   (257, 255), (1000, 1000), (4097, 17), (17, 4097), (1023, 2049),
                                   (64, 128), (64, 129), (70, 128), (129, 255), (200, 64), (63, 128), (3000, 127),
                                   (2100, 2300), (1100, 7777), (40000, 100), (33000, 127)])     # beyond the small-matrix tile: 64 x 128, 64 x 64
def test_transpose_shapes(gpu, shape):
    rows, cols = shape
    say("transpose %dx%d" % shape)
    A = inputs.any_bits_f32(10, 1, rows, cols)          # every bit pattern: NaN payloads, infinities, denormals, -0
    _check_transpose(gpu, A, repeat=2)
    _check_transpose(gpu, A, lda=cols + 3, ldt=rows + 5, offset=1, repeat=2)        # padded, 4-byte aligned only
    _check_transpose(gpu, A, lda=cols + (-cols) % 4 + 4, ldt=rows + (-rows) % 4)    # 16-byte aligned rows


@pytest.mark.parametrize("n", [1 << 10, 1 << 11, 1 << 12, 1 << 13, 1 << 14])
def test_transpose_paper_sizes(gpu, n):
    # the paper's five Task-8 sizes, full comparison with the oracle
    say("transpose %d^2 (paper size)" % n)
    A = inputs.uniform_pm1(10, 2, n, n)
    _check_transpose(gpu, A)


def test_transpose_twice_is_the_identity(gpu):
    A = inputs.any_bits_f32(10, 3, 777, 1234)
    T = run_transpose(gpu, A)
    assert np.array_equal(run_transpose(gpu, T).view(np.uint32), A.view(np.uint32))


def test_transpose_empty(gpu):
    import torch
    t = torch.full((8,), 3.0, device="cuda")
    gpu.check(gpu.transpose_f32(0, 5, None, 5, t, 0, 0))
    gpu.check(gpu.transpose_f32(5, 0, None, 0, t, 5, 0))
    torch.cuda.synchronize()
    assert bool((t == 3.0).all())


@pytest.mark.parametrize("kind", [0, 1])
def test_mfma_ceiling_loop_computes_what_its_operands_define(gpu, kind):
    # The register-only MFMA loop behind the bench's ceiling figure is a measurement aid, but it must still be the MFMAs
    # it claims to be: with every operand 1.0 each accumulator entry ends at passes x (k of one pass), so a lane's sum over
    # its 256 accumulator registers is 256 x that: kind 0, fp32 32x32x2, 4 MFMAs per block and pass = 8 k;
    # kind 1, bf16 16x16x32, 2 MFMAs per block and pass = 64 k.  Exact in fp32 for these sizes.
    import torch
    say("mfma ceiling kind %d" % kind)
    passes, groups = 7, 3
    ops = (torch.ones(2048, device="cuda", dtype=torch.float32) if kind == 0
           else torch.full((16384,), 0x3F80, device="cuda", dtype=torch.int16))
    sink = torch.zeros(groups * 256, device="cuda", dtype=torch.float32)
    rc, flop = gpu.fsrgemm_mfma_ceiling(kind, passes, ops, sink, groups, torch.cuda.current_stream().cuda_stream)
    gpu.check(rc)
    torch.cuda.synchronize()
    assert flop == groups * 4 * passes * (64 * 4096 if kind == 0 else 128 * 16384)
    assert bool((sink == 256.0 * passes * (8 if kind == 0 else 64)).all())


P_FAKE = 0x1000      # an aligned address for the plan queries (never dereferenced)


@pytest.mark.parametrize("ta,tb", [(0, 0), (0, 1), (1, 0), (1, 1)])
@pytest.mark.parametrize("shape", [(5000, 5120, 512), (5120, 5000, 512), (3000, 7168, 772), (7168, 7168, 512)])
def test_f32_two_band_products(gpu, shape, ta, tb):
    # problems the dispatcher runs as two bands of C, each in its own tile shape (a cut along the rows, one along the
    # columns, a ragged N and a rest of K among them): the whole result against the oracle, bit for bit against the
    # same product forced into one launch of the first band's tile (every shape of this kernel sums in the same order),
    # padding untouched, two runs identical
    M, N, K = shape
    say("fp32 two bands %dx%dx%d transA=%d transB=%d" % (M, N, K, ta, tb))
    lda, ldb = (M if ta else K) + 8, (K if tb else N) + 4
    dim, at, first, second = gpu.fsrgemm_bands_f32(ta, tb, M, N, K, P_FAKE, lda, P_FAKE, ldb)
    assert dim in (1, 2), "this case is meant to take the two-band path"
    A, B = inputs.uniform_pm1(30, 1, M, K), inputs.uniform_pm1(30, 2, K, N)
    got = run_f32_ex(gpu, ta, tb, A, B, lda=lda, ldb=ldb, ldc=N + 4, repeat=2)
    ref, S = oracle.gemm(A, B)
    e = oracle.componentwise_error(got, ref, S)
    assert e <= TOL_F32, "componentwise error %.3e" % e
    one = run_cfg(gpu, "f32", first, 1, ta, tb, A, B, lda=lda, ldb=ldb, ldc=N + 4)
    assert np.array_equal(got.view(np.uint32), one.view(np.uint32))


def test_f32_two_band_product_of_integers_is_exact(gpu):
    M, N, K = 4608, 4608, 1024
    say("fp32 two bands %dx%dx%d integers" % (M, N, K))
    assert gpu.fsrgemm_bands_f32(0, 0, M, N, K, P_FAKE, K, P_FAKE, N)[0] != 0
    A, B = inputs.small_ints(31, 1, M, K), inputs.small_ints(31, 2, K, N)
    got = run_f32(gpu, A, B)
    ref, _ = oracle.gemm(A, B)
    assert np.array_equal(got.astype(np.float64), ref)


@pytest.mark.parametrize("shape,ta,tb", [((7168, 7168, 2056), 0, 1), ((7168, 7168, 1024), 0, 0), ((7000, 7168, 1032), 1, 1), ((7168, 7168, 1032), 1, 0)])
def test_bf16_two_band_products(gpu, shape, ta, tb):
    # the same for bf16 operands, in every storage order
    M, N, K = shape
    say("bf16 two bands %dx%dx%d transA=%d transB=%d" % (M, N, K, ta, tb))
    lda, ldb = (M if ta else K) + 8, (K if tb else N) + 16
    dim, at, first, second = gpu.fsrgemm_bands_bf16(ta, tb, M, N, K, P_FAKE, lda, P_FAKE, ldb)
    assert dim != 0, "these cases take the two-band path"
    A = inputs.bf16_normal_scaled(32, 1, M, K, 1 / math.sqrt(K))
    B = inputs.bf16_normal_scaled(32, 2, K, N, 1 / math.sqrt(K))
    got = run_bf16_ex(gpu, ta, tb, A, B, lda=lda, ldb=ldb, ldc=N + 4, repeat=2)
    ref, S = oracle.gemm(A, B)
    e = oracle.componentwise_error(got, ref, S)
    assert e <= TOL_BF16, "componentwise error %.3e" % e
    assert e <= 1e-5, "fp32 accumulation of exact products stays far inside the bf16 tolerance: %.3e" % e
    one = run_cfg(gpu, "bf16", first, 1, ta, tb, A, B, lda=lda, ldb=ldb, ldc=N + 4)
    assert np.array_equal(got.view(np.uint32), one.view(np.uint32))
