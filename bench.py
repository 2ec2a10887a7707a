#!/usr/bin/env python3
"""Validator + profiler bench for the GEMM library, in the spirit of the paper's
Function Validator and Performance Profiler (Section 3.2): a correctness pass
rate over a seeded shape sweep against the CPU oracle, then measured kernel
latency on the two headline workloads.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload f32_4096|bf16_8192]

Prints one JSON line.  A "step" is one GEMM call on the headline workload with
operands already resident in HBM; buffers rotate between steps so that no step
finds its operands in the Infinity Cache left by the previous one.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"f32": 157.3, "bf16": 2500.0}     # MI355X dense MFMA peaks

# HBM-side bytes per launch from the FETCH_SIZE / WRITE_SIZE counter runs summarised in
# profiles/gemm_f32_4096_bf16_8192_hbm_traffic.txt (scaled by a 1 GiB copy).  Each entry is tied to the
# kernel sources it was measured on: once those change the figure is stale and the bench reports null.
TRAFFIC = {
    "f32_4096": {"bytes": 470113020, "sources": {"gemm_f32_main.hip": "d31f2c4fcf463724", "common.hpp": "fcd7c27e4bf90732"}},
    "bf16_8192": {"bytes": 2091149134, "sources": {"gemm_bf16_main.hip": "931ab26717423255", "common.hpp": "fcd7c27e4bf90732"}},
}
# the same for the transposes (profiles/transpose_f32_paper_sizes.txt), by N
_T8_SOURCES = {"transpose.hip": "5bcb289871390c86", "common.hpp": "fcd7c27e4bf90732"}
TRAFFIC.update({"transpose_%d" % n: {"bytes": b, "sources": _T8_SOURCES}
                for n, b in ((1024, 8417187), (2048, 33582523), (4096, 134260464), (8192, 536906752), (16384, 2147493058))})


def measured_traffic(name):
    import hashlib

    entry = TRAFFIC.get(name)
    if entry is None:
        return None
    for fname, digest in entry["sources"].items():
        path = os.path.join(ROOT, "paper_2506_09092_amd", "csrc", fname)
        try:
            if hashlib.sha256(open(path, "rb").read()).hexdigest()[:16] != digest:
                return None
        except OSError:
            return None
    return entry["bytes"]


def log(msg):
    print(msg, file=sys.stderr, flush=True)


def make_workload(name, torch, inputs):
    """Device operands for a headline workload: returns dict(call sets, flops, ...)."""
    import numpy as np

    if name == "f32_4096":
        n, n_sets = 4096, 4
        A, B = inputs.normal(2, 1, n, n), inputs.normal(2, 2, n, n)
        sets = []
        for s in range(n_sets):
            # every set holds the same seeded matrices, at its own addresses
            sets.append((torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda(),
                         torch.empty(n, n, device="cuda", dtype=torch.float32)))
        return dict(name=name, kind="f32", M=n, N=n, K=n, lda=n, ldb=n, ldc=n, sets=sets, hostA=A, hostB=B,
                    desc="fp32 GEMM M=N=K=4096, row-major, N(0,1), seed 2",
                    bytes=3 * n * n * 4, flops=2.0 * n ** 3)
    if name == "bf16_8192":
        n, n_sets = 8192, 3
        A = inputs.bf16_normal_scaled(4, 1, n, n, 1 / math.sqrt(n))
        Bt = inputs.bf16_normal_scaled(4, 2, n, n, 1 / math.sqrt(n))
        sets = []
        for s in range(n_sets):
            sets.append((torch.from_numpy(A.view(np.int16)).cuda(), torch.from_numpy(Bt.view(np.int16)).cuda(),
                         torch.empty(n, n, device="cuda", dtype=torch.float32)))
        return dict(name=name, kind="bf16", M=n, N=n, K=n, lda=n, ldb=n, ldc=n, sets=sets, hostA=A, hostB=Bt,
                    desc="bf16 GEMM M=N=K=8192, A row-major, B column-major, fp32 accumulate/output, N(0,1)/sqrt(K), seed 4",
                    bytes=2 * n * n * 2 + n * n * 4, flops=2.0 * n ** 3)
    raise SystemExit("unknown workload %r" % name)


def mfma_ceiling(w, lib, torch, inputs, launches=120):
    """The register-only loop of the workload's MFMA instruction (fsrgemm_mfma_ceiling) on operands drawn like the
    workload's, one workgroup per compute unit, about 1 ms a launch: TFLOP/s from the median of the last third of
    the launches (HIP events per launch)."""
    import numpy as np

    kind = 0 if w["kind"] == "f32" else 1
    if kind == 0:
        ops = torch.from_numpy(inputs.normal(2, 40, 1, 2048)).cuda()
    else:
        ops = torch.from_numpy(inputs.bf16_normal_scaled(4, 40, 1, 16384, 1 / math.sqrt(w["K"])).view(np.int16)).cuda()
    groups = torch.cuda.get_device_properties(0).multi_processor_count
    sink = torch.empty(groups * 256, device="cuda", dtype=torch.float32)
    passes = 500 if kind == 0 else 1000
    stream = torch.cuda.current_stream().cuda_stream
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(launches)]
    flop = 0.0
    for e0, e1 in evs:
        e0.record()
        rc, flop = lib.fsrgemm_mfma_ceiling(kind, passes, ops, sink, groups, stream)
        lib.check(rc)
        e1.record()
    torch.cuda.synchronize()
    ms = [e0.elapsed_time(e1) for e0, e1 in evs]
    tail = sorted(ms[-(launches // 3):])
    rate = lambda t: flop / (t * 1e-3) / 1e12
    return {"kernel": lib.fsrgemm_kernel_for_mfma_ceiling(kind), "operands": "drawn like the workload's", "workgroups": groups,
            "launches": launches, "tflops": rate(tail[len(tail) // 2]), "tflops_first_5_launches": rate(sum(ms[:5]) / 5),
            "ms_median": tail[len(tail) // 2]}


def time_workload(w, lib, torch, steps, warmup, settle=True):
    """Let the clocks settle, warm up, then time exactly `steps` calls: wall clock around the whole region
    (synchronised on both sides) and a HIP event pair around every launch."""
    fn = lib.gemm_f32 if w["kind"] == "f32" else lib.gemm_bf16
    stream = torch.cuda.current_stream().cuda_stream
    sets = w["sets"]

    def call(i):
        a, b, c = sets[i % len(sets)]
        lib.check(fn(w["M"], w["N"], w["K"], a, w["lda"], b, w["ldb"], c, w["ldc"], stream))

    # The device has idled while the host prepared operands and checked results, and its clocks take tens of launches to
    # come back (a cold device's first launches of the bf16 workload are 20 % slower).  Untimed launches of the workload
    # itself, in blocks of 10, until a block is no faster than the one before (within 0.5 %), at most 20 blocks: what
    # follows -- the warm-up the caller asked for and the timed steps -- then runs at the clocks this workload sustains.
    settle_blocks = []
    while settle and len(settle_blocks) < 20:
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(10):
            call(i)
        e1.record()
        torch.cuda.synchronize()
        settle_blocks.append(e0.elapsed_time(e1) / 10)
        if len(settle_blocks) >= 2 and settle_blocks[-1] >= 0.995 * settle_blocks[-2]:
            break
    for i in range(warmup):
        call(i)
    torch.cuda.synchronize()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    t0 = time.perf_counter()
    for i, (e0, e1) in enumerate(evs):
        e0.record()
        call(warmup + i)
        e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    series = [e0.elapsed_time(e1) for e0, e1 in evs]
    per = sorted(series)
    head = series[:min(5, len(series))]
    tail = series[-min(5, len(series)):]
    # the other cache regime: the same operand set launch after launch (what fits the caches stays there)
    warm = steady_ms(torch, lambda: call(0))
    return dict(wall_ms_per_step=wall_ms / steps, launch_ms_avg=sum(per) / len(per),
                launch_ms_median=per[len(per) // 2], launch_ms_min=per[0], launch_ms_max=per[-1],
                launch_ms_first_5=sum(head) / len(head), launch_ms_last_5=sum(tail) / len(tail), launch_ms_same_buffers=warm,
                settle_ms_per_launch_by_block=settle_blocks)


def report(w, t, lib, ceiling):
    peak = PEAK_TFLOPS[w["kind"]]
    q = lib.fsrgemm_kernel_for_f32 if w["kind"] == "f32" else lib.fsrgemm_kernel_for_bf16
    a, b, c = w["sets"][0]
    achieved = w["flops"] / (t["launch_ms_avg"] * 1e-3) / 1e12
    return dict(
        workload=w["desc"],
        tflops=w["flops"] / (t["wall_ms_per_step"] * 1e-3) / 1e12,
        ms_per_step=t["wall_ms_per_step"],
        # the timed launches in order: a device that was still ramping its clocks shows first_5 above last_5
        launch_ms={"avg": t["launch_ms_avg"], "median": t["launch_ms_median"], "min": t["launch_ms_min"], "max": t["launch_ms_max"],
                   "first_5": t["launch_ms_first_5"], "last_5": t["launch_ms_last_5"],
                   "same_buffers_median": t["launch_ms_same_buffers"],
                   # untimed launches in front of the warm-up, in blocks of 10 (ms per launch of each block), that bring an
                   # idle device's clocks to what this workload sustains
                   "settle_blocks_of_10": t["settle_ms_per_launch_by_block"]},
        roofline={"bound": "mfma", "kernel": q(w["M"], w["N"], w["K"], a, w["lda"], b, w["ldb"], c, w["ldc"]),
                  "achieved": achieved, "peak": peak, "unit": "TFLOP/s", "frac": achieved / peak,
                  # a register-only loop of the kernel's MFMA on the same kind of data, whole chip, measured in this
                  # run directly after the workload
                  "register_only_mfma_loop": ceiling["tflops"] if ceiling else None,
                  "frac_of_register_only_loop": achieved / ceiling["tflops"] if ceiling else None,
                  "traffic": measured_traffic(w["name"]),
                  "hbm_GBps_algorithmic": w["bytes"] / (t["launch_ms_avg"] * 1e-3) / 1e9,
                  "launch_ms": {"avg": t["launch_ms_avg"], "min": t["launch_ms_min"], "first_5": t["launch_ms_first_5"],
                                "last_5": t["launch_ms_last_5"]}},
        mfma_ceiling=ceiling,
    )


def steady_ms(torch, fn, samples=7, warm_ms=20.0, min_ms=0.5):
    """Median time of one call of fn (a launch on the current stream) in ms, at steady clocks: fn first runs for
    about warm_ms, then each of `samples` timings covers a run of calls that lasts about min_ms (at least one
    call), so that neither the idle-clock ramp nor the gap between launches is part of the figure.  The calls
    reuse their operands: problems that fit the caches are timed with warm caches."""
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    fn()
    fn()
    e1.record()
    torch.cuda.synchronize()
    one = max(e0.elapsed_time(e1) / 2, 1e-3)
    for _ in range(int(min(512, warm_ms / one))):
        fn()
    # the first two calls may have paid for a first launch: size the runs by a run of warm calls
    e0.record()
    for _ in range(16):
        fn()
    e1.record()
    torch.cuda.synchronize()
    one = max(min(one, e0.elapsed_time(e1) / 16), 1e-3)
    reps = int(max(1, min(256, min_ms / one)))
    times = []
    for _ in range(samples):
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        times.append(e0.elapsed_time(e1) / reps)
    return sorted(times)[samples // 2]


def paper_task2_sizes(lib, torch):
    """Latency of the paper's own Task 2 shapes (appendix input-size table): A (size, 4096), B (4096, 2048), fp32,
    size = 2^10 .. 2^18.  Profiler leg only; values are random normal (correctness of these shapes is a GPU test)."""
    out = []
    K, N = 4096, 2048
    b = torch.randn(K, N, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    for e in (10, 12, 14, 16, 18):
        M = 1 << e
        a = torch.randn(M, K, device="cuda")
        c = torch.empty(M, N, device="cuda")
        ms = steady_ms(torch, lambda: lib.check(lib.gemm_f32(M, N, K, a, K, b, N, c, N, stream)))
        out.append({"size": M, "kernel": lib.fsrgemm_kernel_for_f32(M, N, K, a, K, b, N, c, N), "ms": ms,
                    "tflops": 2.0 * M * N * K / (ms * 1e-3) / 1e12})
        del a, c
    return out


def mid_sizes_f32(lib, torch):
    """fp32 problems between the small fixed configurations and the headline size, where the number of output tiles
    per compute unit decides: the kernel and tile shape the dispatcher takes (two kernels where it runs the product
    as two bands of C), its rate, and torch.matmul (the vendor library) on the same buffers for scale.  Profiler leg only; these shapes' parity is covered by the GPU tests."""
    stream = torch.cuda.current_stream().cuda_stream
    out = []
    for M, N, K in ((2048, 2048, 2048), (3072, 3072, 3072), (3584, 3584, 3584), (4096, 2048, 4096), (4608, 4608, 4608), (5120, 5120, 2048),
                    (6144, 6144, 2048), (7168, 7168, 2048), (8192, 8192, 2048), (4096, 4096, 4112)):
        a, b, c = torch.randn(M, K, device="cuda"), torch.randn(K, N, device="cuda"), torch.empty(M, N, device="cuda")
        ms = steady_ms(torch, lambda: lib.check(lib.gemm_f32(M, N, K, a, K, b, N, c, N, stream)), samples=5)
        vendor = steady_ms(torch, lambda: torch.matmul(a, b, out=c), samples=5)
        out.append({"M": M, "N": N, "K": K, "kernel": lib.fsrgemm_kernel_for_f32(M, N, K, a, K, b, N, c, N), "ms": ms,
                    "tflops": 2.0 * M * N * K / (ms * 1e-3) / 1e12, "torch_matmul_tflops": 2.0 * M * N * K / (vendor * 1e-3) / 1e12})
        del a, b, c
    return out


def mid_sizes_bf16(lib, torch):
    """bf16 problems (A row-major, B column-major) whose 256 x 256 tiles do not fill whole rounds of the compute units (or,
    2048^3, do not give every unit one), or whose K is not whole K-tiles: the tile shape of the direct-to-LDS kernel the dispatcher took, its rate, and
    torch.matmul (the vendor library, bf16 output) on the same buffers for scale.  Profiler leg only; parity of every
    shape and of the rest-of-K step is covered by the GPU tests."""
    import math

    stream = torch.cuda.current_stream().cuda_stream
    out = []
    for M, N, K in ((2048, 2048, 2048), (4096, 4096, 4096), (5120, 5120, 5120), (6144, 6144, 6144), (7168, 7168, 7168), (3072, 8192, 4096),
                    (8192, 8192, 8200), (8000, 8000, 8000)):
        a = (torch.randn(M, K, device="cuda") / math.sqrt(K)).to(torch.bfloat16)
        b = (torch.randn(N, K, device="cuda") / math.sqrt(K)).to(torch.bfloat16)
        c, cb = torch.empty(M, N, device="cuda"), torch.empty(M, N, device="cuda", dtype=torch.bfloat16)
        ms = steady_ms(torch, lambda: lib.check(lib.gemm_bf16(M, N, K, a, K, b, K, c, N, stream)), samples=5)
        vendor = steady_ms(torch, lambda: torch.matmul(a, b.t(), out=cb), samples=5)
        out.append({"M": M, "N": N, "K": K, "kernel": lib.fsrgemm_kernel_for_bf16(M, N, K, a, K, b, K, c, N), "ms": ms,
                    "tflops": 2.0 * M * N * K / (ms * 1e-3) / 1e12, "torch_matmul_bf16_out_tflops": 2.0 * M * N * K / (vendor * 1e-3) / 1e12})
        del a, b, c, cb
    return out


def small_fixed_configs(lib, torch):
    """fp32 256^3 and 1024^3 (the small fixed configurations; parity is a GPU test): these are bound by launch
    latency and by the number of tiles, so the figure of interest is microseconds per launch."""
    stream = torch.cuda.current_stream().cuda_stream
    out = []
    for n in (256, 1024):
        a, b, c = torch.randn(n, n, device="cuda"), torch.randn(n, n, device="cuda"), torch.empty(n, n, device="cuda")
        ms = steady_ms(torch, lambda: lib.check(lib.gemm_f32(n, n, n, a, n, b, n, c, n, stream)))
        out.append({"n": n, "kernel": lib.fsrgemm_kernel_for_f32(n, n, n, a, n, b, n, c, n), "us": ms * 1e3,
                    "tflops": 2.0 * n ** 3 / (ms * 1e-3) / 1e12})
    return out


def transposed_storage_4096(lib, torch):
    """fp32 4096^3 with A, B or both handed over in transposed storage (gemm_f32_ex): median launch time of each
    of the four storage pairs on the same random operands.  Profiler leg only; parity of these paths is a GPU test."""
    n = 4096
    a, b, c = torch.randn(n, n, device="cuda"), torch.randn(n, n, device="cuda"), torch.empty(n, n, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    out = []
    for ta, tb in ((0, 0), (0, 1), (1, 0), (1, 1)):
        ms = steady_ms(torch, lambda: lib.check(lib.gemm_f32_ex(ta, tb, n, n, n, a, n, b, n, c, n, stream)))
        out.append({"transA": ta, "transB": tb, "kernel": lib.fsrgemm_kernel_for_f32_ex(ta, tb, n, n, n, a, n, b, n, c, n),
                    "ms": ms, "tflops": 2.0 * n ** 3 / (ms * 1e-3) / 1e12})
    return out


def storage_orders_bf16(lib, torch):
    """bf16 cubes in the four storage pairs of gemm_bf16_ex: (0, 1) is the headline kernel's pair; an operand that
    is contiguous along m / n goes through the transposing LDS reads of the same kernel, in every tile shape.
    Median launch time on random operands; parity of these paths is a GPU test."""
    import math

    stream = torch.cuda.current_stream().cuda_stream
    out = []
    for n in (8192, 6144, 3072, 2048):
        a = (torch.randn(n, n, device="cuda") / math.sqrt(n)).to(torch.bfloat16)
        b = (torch.randn(n, n, device="cuda") / math.sqrt(n)).to(torch.bfloat16)
        c = torch.empty(n, n, device="cuda")
        for ta, tb in ((0, 1), (0, 0), (1, 1), (1, 0)):
            ms = steady_ms(torch, lambda: lib.check(lib.gemm_bf16_ex(ta, tb, n, n, n, a, n, b, n, c, n, stream)))
            out.append({"n": n, "transA": ta, "transB": tb, "kernel": lib.fsrgemm_kernel_for_bf16_ex(ta, tb, n, n, n, a, n, b, n, c, n),
                        "ms": ms, "tflops": 2.0 * n ** 3 / (ms * 1e-3) / 1e12})
        del a, b, c
    return out


def split_k(lib, torch, kind):
    """Shapes with few output tiles and a long K (row or column vector times matrix, a few rows against a large
    weight matrix, small squares of long dot products): the plain entry point against the workspace one with the
    workspace the library asks for.  These are HBM-bound: bytes = the operands and the result once, against the
    8 TB/s peak; torch.matmul (the vendor library) on the same operands for scale.  kind: "f32" (row-major operands) or
    "bf16" (A row-major, B column-major)."""
    import math

    stream = torch.cuda.current_stream().cuda_stream
    ws = torch.empty(16 << 20, dtype=torch.uint8, device="cuda")
    out = []

    def median_ms(fn):
        return steady_ms(torch, fn)

    shapes = (((1, 4096, 4096), (4096, 1, 4096), (1, 16384, 16384), (8, 8192, 8192), (2, 8192, 8192), (16, 8192, 8192), (8192, 8, 8192),
               (8, 1024, 16384), (64, 64, 4097), (256, 256, 65536), (512, 512, 16384)) if kind == "f32" else
              ((1, 8192, 8192), (4, 8192, 8192), (8, 8192, 8192), (16, 8192, 8192), (32, 28672, 8192), (256, 256, 65536), (512, 512, 16384)))
    for M, N, K in shapes:
        c = torch.empty(M, N, device="cuda")
        if kind == "f32":
            a, b = torch.randn(M, K, device="cuda"), torch.randn(K, N, device="cuda")
            need = lib.gemm_f32_workspace_bytes(0, 0, M, N, K)
            plain = median_ms(lambda: lib.check(lib.gemm_f32(M, N, K, a, K, b, N, c, N, stream)))
            split = median_ms(lambda: lib.check(lib.gemm_f32_ws(0, 0, M, N, K, a, K, b, N, c, N, ws, need, stream)))
            vendor = median_ms(lambda: torch.matmul(a, b, out=c))
            byts = 4.0 * (M * K + K * N + M * N)
        else:
            a = (torch.randn(M, K, device="cuda") / math.sqrt(K)).to(torch.bfloat16)
            b = (torch.randn(N, K, device="cuda") / math.sqrt(K)).to(torch.bfloat16)
            need = lib.gemm_bf16_workspace_bytes(0, 1, M, N, K)
            plain = median_ms(lambda: lib.check(lib.gemm_bf16(M, N, K, a, K, b, K, c, N, stream)))
            split = median_ms(lambda: lib.check(lib.gemm_bf16_ws(0, 1, M, N, K, a, K, b, K, c, N, ws, need, stream)))
            ch = torch.empty(M, N, device="cuda", dtype=torch.bfloat16)
            vendor = median_ms(lambda: torch.matmul(a, b.t(), out=ch))          # (bf16 output: half the bytes written)
            byts = 2.0 * (M * K + K * N) + 4.0 * M * N
        out.append({"M": M, "N": N, "K": K, "slices": need // (4 * M * N), "workspace_bytes": need, "plain_ms": plain,
                    "ms": split, "torch_matmul_ms": vendor, "tflops": 2.0 * M * N * K / (split * 1e-3) / 1e12,
                    "hbm_GBps_algorithmic": byts / (split * 1e-3) / 1e9, "hbm_frac_of_8TBps": byts / (split * 1e-3) / 8e12})
        del a, b, c
    return out


def transpose_sizes(lib, torch):
    """The paper's Task 8 (matrix transposition) on its five sizes N x N, N = 2^10 .. 2^14: time per launch and
    the HBM roofline (every element read once and written once against 8 TB/s).  The smaller sizes stay in the
    chip's caches between launches (up to 4096^2 at least partly).  Parity is a GPU test."""
    stream = torch.cuda.current_stream().cuda_stream
    out = []
    for e in (10, 11, 12, 13, 14):
        n = 1 << e
        a = torch.randn(n, n, device="cuda")
        t = torch.empty(n, n, device="cuda")
        ms = steady_ms(torch, lambda: lib.check(lib.transpose_f32(n, n, a, n, t, n, stream)))
        byts = 8.0 * n * n
        out.append({"n": n, "ms": ms,
                    "roofline": {"bound": "hbm", "kernel": lib.fsrgemm_kernel_for_transpose_f32(n, n, a, n, t, n),
                                 "achieved": byts / (ms * 1e-3) / 1e9, "peak": 8000.0, "unit": "GB/s", "frac": byts / (ms * 1e-3) / 8e12,
                                 "traffic": measured_traffic("transpose_%d" % n)}})
        del a, t
    return out


def normal_equations(lib, torch):
    """The normal equations of the paper's Task 20 (ordinary least squares: X of n_samples x 10 features, sizes
    2^14 .. 2^22 as in the appendix table): G = X^T X and g = X^T y as two calls of gemm_f32_ws with X as a
    transposed A.  Both stream X from HBM once: 4 n f bytes for G (A and B are the same buffer), 4 n (f + 1) for g."""
    stream = torch.cuda.current_stream().cuda_stream
    f, out = 10, []
    for e in (14, 16, 18, 20, 22):
        n = 1 << e
        X, y = torch.randn(n, f, device="cuda"), torch.randn(n, 1, device="cuda")
        G, g = torch.empty(f, f, device="cuda"), torch.empty(f, 1, device="cuda")
        need = max(lib.gemm_f32_workspace_bytes(1, 0, f, f, n), lib.gemm_f32_workspace_bytes(1, 0, f, 1, n))
        ws = torch.empty(max(need, 4), dtype=torch.uint8, device="cuda")
        t_gram = steady_ms(torch, lambda: lib.check(lib.gemm_f32_ws(1, 0, f, f, n, X, f, X, f, G, f, ws, need, stream)))
        t_xty = steady_ms(torch, lambda: lib.check(lib.gemm_f32_ws(1, 0, f, 1, n, X, f, y, 1, g, 1, ws, need, stream)))
        t_plain = steady_ms(torch, lambda: lib.check(lib.gemm_f32_ex(1, 0, f, f, n, X, f, X, f, G, f, stream)), samples=3, warm_ms=5.0)
        out.append({"n_samples": n, "kernel": lib.fsrgemm_kernel_for_f32_cfg(4, 1, 0, f, f, n, X, f, X, f, G, f),
                    "gram_ms": t_gram, "gram_GBps": 4.0 * n * f / t_gram / 1e6, "gram_frac_of_8TBps": 4.0 * n * f / t_gram / 8e9,
                    "xty_ms": t_xty, "xty_GBps": 4.0 * n * (f + 1) / t_xty / 1e6, "xty_frac_of_8TBps": 4.0 * n * (f + 1) / t_xty / 8e9,
                    "gram_ms_without_workspace": t_plain})
        del X, y
    return out


def validator_pass_in_a_graph(lib, torch, passes=20, n_streams=4):
    """One validator pass = the 64 shapes of the fp32 sweep, each launched once (operands random, tight leading
    dimensions).  Four ways to issue it, time per pass in ms: call by call on one stream; call by call dealt
    round-robin to four streams (the cases are independent, and most are too small to fill the device); one
    replay of a HIP graph that captured the one-stream pass; one replay of a graph that captured the four-stream
    pass (the library allocates nothing and launches plain kernels only, so its calls can be captured)."""
    from paper_2506_09092_amd import inputs

    cases = []
    for c in inputs.sweep_cases(3, 64):
        M, N, K = c["M"], c["N"], c["K"]
        cases.append((M, N, K, torch.randn(M, K, device="cuda"), torch.randn(K, N, device="cuda"), torch.empty(M, N, device="cuda")))
    side = [torch.cuda.Stream() for _ in range(n_streams)]       # default priority

    def one_stream():
        st = torch.cuda.current_stream().cuda_stream
        for M, N, K, a, b, o in cases:
            lib.check(lib.gemm_f32(M, N, K, a, K, b, N, o, N, st))

    def four_streams():
        main = torch.cuda.current_stream()
        for s in side:
            s.wait_stream(main)
        for i, (M, N, K, a, b, o) in enumerate(cases):
            lib.check(lib.gemm_f32(M, N, K, a, K, b, N, o, N, side[i % n_streams].cuda_stream))
        for s in side:
            main.wait_stream(s)

    def captured(fn):
        fn()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            fn()
        return g.replay

    out = {}
    for name, fn in (("one_stream_ms", one_stream), ("four_streams_ms", four_streams),
                     ("graph_one_stream_ms", captured(one_stream)), ("graph_four_streams_ms", captured(four_streams))):
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(passes):
            fn()
        torch.cuda.synchronize()
        out[name] = (time.perf_counter() - t0) * 1e3 / passes
    out["launches_per_pass"] = len(cases)
    return out


def selection_loop(lib, torch):
    """The selection loop (Algorithm 1 over tile configurations, validator = the CPU oracle) on three problems:
    where it starts (the dispatcher's choice), which candidates it visited, what it ends on, and the two timed
    against each other (for 3584^3 the dispatcher's rules run the product as two bands of C, and that plan, two
    launches, is what the loop's winner is timed against).  The loop's code and its oracle-backed validator live in
    fsr_search.py / tests/."""
    from paper_2506_09092_amd.fsr_search import Problem
    from tests import tune_dispatch

    out = []
    for p in (Problem("f32", 0, 0, 3584, 3584, 3584), Problem("f32", 0, 0, 768, 768, 768), Problem("bf16", 0, 1, 512, 512, 16384)):
        rows, rep = tune_dispatch.tune(lib, torch, p, 0.04, lambda msg: None)
        rep["new_table_rows"] = [r.strip() for r in rows]
        out.append(rep)
    return out


def cpu_baseline(w):
    """The oracle as it stands, timed on the host cores over a slab of rows of the same workload."""
    import oracle

    rows = w["M"] if w["kind"] == "f32" else 2048           # a few seconds to ~10 s of host time
    A = w["hostA"][:rows]
    B = w["hostB"] if w["kind"] == "f32" else w["hostB"].T.copy()       # row-major copy: same values
    t0 = time.perf_counter()
    oracle.gemm(A, B, want_scale=False)
    dt = time.perf_counter() - t0
    return {"value": 2.0 * rows * w["N"] * w["K"] / dt / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(),
            "kind": "oracle", "seconds": dt,
            "sample": "%s %d of %d rows of C for the %s workload (fp64 triple loop, OpenMP over rows)" % ("all" if rows == w["M"] else "first", rows, w["M"], w["name"])}


def cpu_baseline_other_sizes(inputs):
    """The oracle on the other configurations, as context for cpu_baseline: one thread on 256^3 and 1024^3, all
    cores on 1024^3, and all cores on the first 512 rows of the bf16 8192^3 product (the whole product would
    take 16 times as long: the last entry is an extrapolation and says so)."""
    import math

    import oracle

    def timed(A, B, threads):
        old = oracle.num_threads()
        oracle.set_num_threads(threads)
        try:
            t0 = time.perf_counter()
            oracle.gemm(A, B, want_scale=False)
            return time.perf_counter() - t0
        finally:
            oracle.set_num_threads(old)

    cores, out = oracle.num_threads(), []
    for n, threads in ((256, 1), (1024, 1), (1024, cores)):
        A, B = inputs.uniform_pm1(1, 1, n, n), inputs.uniform_pm1(1, 2, n, n)
        dt = timed(A, B, threads)
        out.append({"workload": "fp32 %d^3" % n, "cores": threads, "seconds": dt, "gflops": 2.0 * n ** 3 / dt / 1e9})
    n, rows = 8192, 512
    A = inputs.bf16_normal_scaled(4, 1, rows, n, 1 / math.sqrt(n))
    B = inputs.bf16_normal_scaled(4, 2, n, n, 1 / math.sqrt(n)).T.copy()
    dt = timed(A, B, cores)
    out.append({"workload": "bf16 8192^3, first 512 rows of C", "cores": cores, "seconds": dt,
                "gflops": 2.0 * rows * n * n / dt / 1e9, "whole_product_seconds_extrapolated": dt * n / rows})
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=100, help="untimed launches of the workload before the timed ones")
    ap.add_argument("--workload", default="f32_4096", choices=["f32_4096", "bf16_8192"],
                    help="which headline workload fills the top-level fields (both are always measured)")
    ap.add_argument("--no-validate", action="store_true", help="skip the oracle sweep (profiling runs)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-ceiling", action="store_true", help="skip the register-only MFMA loop that is measured behind each headline workload")
    ap.add_argument("--no-settle", action="store_true",
                    help="skip the untimed launches in front of the warm-up that bring an idle device's clocks up (counter runs: fewer dispatches)")
    ap.add_argument("--headline-only", action="store_true",
                    help="time the two headline workloads only (profiling runs: keeps other shapes out of the kernel trace)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy, so that a counter run has a kernel of known traffic to scale by")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        raise SystemExit("bench.py: this library runs on one GPU; --gpus %d is not supported" % args.gpus)

    import torch

    import paper_2506_09092_amd as lib
    from paper_2506_09092_amd import inputs
    from tests import validator        # the oracle-backed checks live with the tests

    lib.load()                      # raises if the HIP library is missing: there is no fallback
    if not torch.cuda.is_available():
        raise SystemExit("bench.py: no GPU visible")
    torch.cuda.set_device(0)

    sweep = None
    if not args.no_validate:
        log("validator: 64-shape sweep + fixed configs against the oracle")
        sweep = validator.run_validator(lib, log)
        log("  pass rate %d/%d (fp32), %d/%d (bf16)" % (sweep["passed"], sweep["total"], sweep["bf16_sweep"]["passed"], sweep["bf16_sweep"]["total"]))

    results, baselines = {}, {}
    for name in ("f32_4096", "bf16_8192"):
        log("profiler: %s" % name)
        w = make_workload(name, torch, inputs)
        chk = None if args.no_validate else validator.check_headline(w, lib, torch)
        # The register-only MFMA loop's rate is measured after the timed region, over 120 launches: run in front, that
        # long a stretch at the chip's highest power draw leaves the next 20 ms measurably slower.
        t = time_workload(w, lib, torch, args.steps, args.warmup, settle=not args.no_settle)
        ceiling = None if args.no_ceiling else mfma_ceiling(w, lib, torch, inputs)
        results[name] = report(w, t, lib, ceiling)
        results[name]["oracle_check"] = chk
        if name == args.workload and not args.no_cpu_baseline:
            baselines[name] = cpu_baseline(w)
        del w
        torch.cuda.empty_cache()

    task2 = layouts = layouts_bf16 = skinny = skinny_bf16 = task8 = selection = graph = small = task20 = mid = mid16 = None
    if not args.headline_only:
        small = small_fixed_configs(lib, torch)
        task2 = paper_task2_sizes(lib, torch)
        mid = mid_sizes_f32(lib, torch)
        mid16 = mid_sizes_bf16(lib, torch)
        layouts = transposed_storage_4096(lib, torch)
        layouts_bf16 = storage_orders_bf16(lib, torch)
        skinny = split_k(lib, torch, "f32")
        skinny_bf16 = split_k(lib, torch, "bf16")
        task8 = transpose_sizes(lib, torch)
        task20 = normal_equations(lib, torch)
        graph = validator_pass_in_a_graph(lib, torch)
        if not args.no_validate:
            log("selection loop on three problems")
            selection = selection_loop(lib, torch)
    torch.cuda.empty_cache()

    if args.copy_calibration:
        src = torch.empty(1 << 28, device="cuda", dtype=torch.float32).fill_(1.0)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)                  # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    other_name = "bf16_8192" if args.workload == "f32_4096" else "f32_4096"
    top, other = results[args.workload], results[other_name]
    out = {
        "metric": "GEMM TFLOP/s + % MFMA peak at 4096^3 fp32, 8192^3 bf16; sweep pass rate",
        "value": top["tflops"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": top["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if args.workload == "f32_4096" else "bf16 in, f32 accumulate",
        "data": "synthetic (seeded; stands in for the paper's unstated random validator inputs)",
        "config": {"workload": top["workload"], "second_workload": other["workload"] + " (under roofline.%s)" % other_name, "buffers": "rotating operand/result sets", "timing": "wall clock over all steps; HIP events per launch"},
        # the top-level roofline is the top-level workload's; the other half of the metric sits inside it under its own name
        "roofline": dict(top["roofline"], **{other_name: dict(other["roofline"], workload=other["workload"], tflops=other["tflops"],
                                                              ms_per_step=other["ms_per_step"], oracle_check=other["oracle_check"])}),
        "launch_ms": top["launch_ms"], "oracle_check": top["oracle_check"], "mfma_ceiling": top["mfma_ceiling"],
        "cpu_baseline": baselines.get(args.workload),
        "cpu_baseline_other_sizes": None if args.no_cpu_baseline else cpu_baseline_other_sizes(inputs),
        "small_fixed_configs_f32": small,
        "other_workload": other,
        "sweep": sweep,
        "paper_task2_shapes": task2,
        "mid_sizes_f32": mid,
        "mid_sizes_bf16": mid16,
        "transposed_storage_f32_4096": layouts,
        "storage_orders_bf16": layouts_bf16,
        "split_k_f32": skinny,
        "split_k_bf16": skinny_bf16,
        "paper_task8_transpose": task8,
        "paper_task20_normal_equations": task20,
        "selection_loop": selection,
        "validator_pass_fp32_sweep": graph,
        "paper_context": "paper reports only speedups over hand-written CUDA for the group holding Task 2: 5.95-68.3x (RTX 3090 Ti), 6.06-60.0x (GTX 1660 SUPER)",
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
