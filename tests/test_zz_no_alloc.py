"""gemm_f32_noalloc, the entry point for callers that cannot allocate device memory: the same kernels as gemm_f32_ws
on a fixed scratch array inside the library.  Checked against gemm_f32_ws with the workspace the library asks for
(bit for bit: same plan, same order of summation) and against the CPU oracle, on calls in a row that share the
array, the second with a smaller problem."""
import numpy as np
import pytest

import oracle
import paper_2506_09092_amd as lib
from paper_2506_09092_amd import inputs
from paper_2506_09092_amd.harness import run_f32_ws, run_noalloc

TOL_F32 = 1e-5
P = 0x1000      # fake aligned address for calls that are rejected before any launch


def test_rejected_before_any_launch():
    bad, limit = lib.FSRGEMM_ERR_INVALID_ARG, lib.FSRGEMM_ERR_SCRATCH_LIMIT
    f = lambda M, N, K, a=P, lda=None, c=P: lib.gemm_f32_noalloc(0, 0, M, N, K, a, lda or K, P, N, c, N, 0)
    assert f(-1, 4, 4) == bad and f(4, 4, 4, lda=3) == bad and f(4, 4, 4, a=None) == bad and f(4, 4, 4, c=None) == bad
    assert f(0, 4, 4, a=None, c=None) == lib.FSRGEMM_OK             # empty: nothing to launch
    # the array holds the largest workspace the library ever asks for, so no problem is turned away for its size
    import random

    rng = random.Random(5)
    dims = [1, 2, 10, 16, 64, 100, 256, 384, 512, 640, 1000, 1024, 2048, 4096, 1 << 14, 1 << 16, 1 << 20, 1 << 22]
    worst = max(lib.gemm_f32_workspace_bytes(rng.randint(0, 1), rng.randint(0, 1), rng.choice(dims[:14]), rng.choice(dims[:14]), rng.choice(dims))
                for _ in range(3000))
    assert lib.gemm_f32_workspace_bytes(0, 0, 1024, 1024, 16384) == 16 << 20 == lib.FSRGEMM_NOALLOC_SCRATCH_BYTES and worst <= 16 << 20
    assert "scratch" in lib.fsrgemm_status_string(limit)
    with pytest.raises(lib.FsrGemmError):
        lib.check(limit)


def _noalloc(gpu, ta, tb, A, B, ldc=None):
    return run_noalloc(gpu, ta, tb, A, B, ldc=ldc)


@pytest.mark.gpu
def test_no_alloc_entry_point_matches_the_workspace_entry_point(gpu):
    # (transA, transB, M, N, K): a larger problem first, then smaller ones on the same array -- split tile kernels
    # (64 x 64 and 128 x 128 tiles), the small-result kernel, split vector kernels, and problems that need no scratch
    calls = [(0, 0, 1024, 1024, 16384), (0, 0, 512, 512, 16384), (0, 0, 64, 64, 4097), (1, 0, 10, 10, 1 << 16), (1, 0, 10, 1, 1 << 14),
             (0, 0, 1, 4096, 4096), (0, 0, 256, 256, 65536), (0, 0, 130, 70, 2050), (0, 0, 300, 260, 200), (0, 0, 1, 1, 100003),
             (0, 0, 8, 1024, 16384), (0, 1, 12, 2048, 8192), (1, 0, 3000, 5, 4100)]        # a few rows or columns: streaming kernels in K slices
    seen = set()
    for ta, tb, M, N, K in calls:
        print("no-alloc %d%d %dx%dx%d" % (ta, tb, M, N, K), flush=True)
        need = gpu.gemm_f32_workspace_bytes(ta, tb, M, N, K)
        assert need <= gpu.FSRGEMM_NOALLOC_SCRATCH_BYTES
        seen.add(need > 0)
        A, B = inputs.uniform_pm1(21, 1, M, K), inputs.uniform_pm1(21, 2, K, N)
        want = run_f32_ws(gpu, ta, tb, A, B)                     # the existing entry point with the workspace it asks for
        got = _noalloc(gpu, ta, tb, A, B)
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), (ta, tb, M, N, K)
        ref, S = oracle.gemm(A, B)
        assert oracle.componentwise_error(got, ref, S) <= TOL_F32
        again = _noalloc(gpu, ta, tb, A, B, ldc=N + 5)            # the array keeps the last call's contents: same bits again
        assert np.array_equal(again.view(np.uint32), got.view(np.uint32))
    assert seen == {True, False}
    # small integers: exactly one correct result
    Ai, Bi = inputs.small_ints(0, 13, 64, 4097), inputs.small_ints(0, 14, 4097, 64)
    assert np.array_equal(_noalloc(gpu, 0, 0, Ai, Bi).astype(np.float64), oracle.gemm(Ai, Bi)[0])
