"""Oracle-backed checks used by the bench's validator leg: the sweep pass rate and a
sampled check of the headline workloads.  Kept under tests/ because, like the parity
tests, it compares the HIP path with the CPU oracle."""
from __future__ import annotations

import numpy as np

import oracle
from paper_2506_09092_amd import inputs
from paper_2506_09092_amd.harness import run_bf16, run_f32


def run_validator(lib, log=print):
    """Pass rate of the 64-shape sweep (fp32, and the same shapes with bf16 operands) plus the small fixed configurations,
    against the CPU oracle."""
    passed, total, worst = 0, 0, 0.0
    for c in inputs.sweep_cases(3, 64):
        A = inputs.uniform_pm1(3, 2 * c["index"] + 10, c["M"], c["K"])
        B = inputs.uniform_pm1(3, 2 * c["index"] + 11, c["K"], c["N"])
        total += 1
        try:
            got = run_f32(lib, A, B, lda=c["lda"], ldb=c["ldb"], ldc=c["ldc"], offset=c["offset"], repeat=2)
            ref, S = oracle.gemm(A, B)
            e = oracle.componentwise_error(got, ref, S)
            worst = max(worst, e)
            passed += int(e <= 1e-5)
        except Exception as ex:       # a failed launch or a trampled canary counts as a failed case
            log("sweep case %d failed: %s" % (c["index"], ex))
    # the same shapes through gemm_bf16 (A row-major, B column-major; bf16 tolerance 1e-2)
    passed16, worst16 = 0, 0.0
    for c in inputs.sweep_cases(3, 64):
        M, N, K = c["M"], c["N"], c["K"]
        A = inputs.bf16_normal_scaled(3, 2 * c["index"] + 10, M, K, 1 / np.sqrt(max(K, 1)))
        Bt = inputs.bf16_normal_scaled(3, 2 * c["index"] + 11, N, K, 1 / np.sqrt(max(K, 1)))
        try:
            got = run_bf16(lib, A, Bt, lda=max(c["lda"], 1), ldb=max(K + c["ldb"] - N, 1), ldc=c["ldc"], offset=c["offset"], repeat=2)
            ref, S = oracle.gemm(A, np.ascontiguousarray(Bt.T))
            e = oracle.componentwise_error(got, ref, S)
            worst16 = max(worst16, e)
            passed16 += int(e <= 1e-2)
        except Exception as ex:
            log("bf16 sweep case %d failed: %s" % (c["index"], ex))
    fixed = {}
    A, B = inputs.small_ints(0, 3, 256, 256), inputs.small_ints(0, 4, 256, 256)
    fixed["f32_256_int_bit_exact"] = bool(np.array_equal(run_f32(lib, A, B).astype(np.float64), oracle.gemm(A, B)[0]))
    A, B = inputs.uniform_pm1(0, 1, 256, 256), inputs.uniform_pm1(0, 2, 256, 256)
    ref, S = oracle.gemm(A, B)
    fixed["f32_256"] = bool(oracle.componentwise_error(run_f32(lib, A, B), ref, S) <= 1e-5)
    A, B = inputs.uniform_pm1(1, 1, 1024, 1024), inputs.uniform_pm1(1, 2, 1024, 1024)
    ref, S = oracle.gemm(A, B)
    fixed["f32_1024"] = bool(oracle.componentwise_error(run_f32(lib, A, B), ref, S) <= 1e-5)
    A, Bt = inputs.bf16_small_ints(4, 30, 512, 512), inputs.bf16_small_ints(4, 31, 512, 512)
    fixed["bf16_512_int_bit_exact"] = bool(np.array_equal(run_bf16(lib, A, Bt).astype(np.float64), oracle.gemm(A, Bt.T)[0]))
    return dict(passed=passed, total=total, pass_rate=passed / total, worst_componentwise_error=worst,
                tolerance=1e-5, fixed_configs=fixed,
                bf16_sweep=dict(passed=passed16, total=total, pass_rate=passed16 / total, worst_componentwise_error=worst16, tolerance=1e-2))


def one_entry_per_block(M, N, block, seed):
    """A random entry inside every block x block square of an M x N matrix (the squares an MFMA instruction or a
    wavefront writes as a unit are multiples of 16): no such square goes unsampled."""
    rng = np.random.default_rng(seed)
    bi, bj = np.meshgrid(np.arange(0, M, block), np.arange(0, N, block), indexing="ij")
    ii = np.minimum(bi.ravel() + rng.integers(0, block, bi.size), M - 1)
    jj = np.minimum(bj.ravel() + rng.integers(0, block, bj.size), N - 1)
    return ii, jj


def check_headline(w, lib, torch):
    """Oracle check of a headline workload's output, in the launch configuration that is timed: one entry in every
    16 x 16 block of the result."""
    a, b, c = w["sets"][0]
    fn = lib.gemm_f32 if w["kind"] == "f32" else lib.gemm_bf16
    c.fill_(float("nan"))
    lib.check(fn(w["M"], w["N"], w["K"], a, w["lda"], b, w["ldb"], c, w["ldc"], torch.cuda.current_stream().cuda_stream))
    torch.cuda.synchronize()
    got = c.cpu().numpy()
    ii, jj = one_entry_per_block(w["M"], w["N"], 16, 7)
    Bm = w["hostB"] if w["kind"] == "f32" else w["hostB"].T
    ref, s = oracle.gemm_entries(w["hostA"], Bm, ii, jj)
    e = oracle.componentwise_error(got[ii, jj], ref, s)
    tol = 1e-5 if w["kind"] == "f32" else 1e-2
    return dict(sampled_entries=int(ii.size), sampling="one entry in every 16 x 16 block", componentwise_error=e, tolerance=tol,
                ok=bool(e <= tol and np.all(np.isfinite(got))))
