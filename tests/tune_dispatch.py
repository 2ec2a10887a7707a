"""Runs the selection loop (paper_2506_09092_amd/fsr_search.py: the paper's Algorithm 1 over tile configurations)
on a list of problems with the CPU oracle as the function validator, and writes the rows of
paper_2506_09092_amd/csrc/tuned_table.inc for the problems whose measured best beats the dispatcher's rules.
Lives under tests/ because it compares the HIP path with the oracle.

    python -m tests.tune_dispatch --out <file> [--log <file>] [--only f32|bf16|bf16-orders|thin]        (on an MI355X)

A row is written only when the winner is at least `--gain` (default 4 %) faster than what the dispatcher's rules
alone would take, measured twice; everything else stays with the rules.  After replacing the table, rebuild the library.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import oracle                                                   # noqa: E402
from paper_2506_09092_amd import fsr_search, inputs             # noqa: E402
from paper_2506_09092_amd.fsr_search import Candidate, Problem  # noqa: E402

# The problems: cubes around the tile rules' thresholds, the paper's Task-2 family (A of size x 4096 against B of
# 4096 x 2048, appendix table of test sizes) as far as host-side generation stays cheap, and the few-tiles-long-K
# shapes that the workspace entry points exist for.  fp32 row-major operands, bf16 with both operands contiguous
# along k (the storage orders of gemm_f32 / gemm_bf16).
F32 = [(n, n, n) for n in (256, 512, 768, 1024, 1536, 2048, 2560, 3072, 3584, 4096, 5120, 6144, 7168, 8192)] + \
      [(1024, 2048, 4096), (4096, 2048, 4096), (16384, 2048, 4096)] + \
      [(1, 4096, 4096), (4096, 1, 4096), (8, 8192, 8192), (64, 64, 4097), (256, 256, 65536), (512, 512, 16384)]
BF16 = [(n, n, n) for n in (512, 1024, 1536, 2048, 2560, 3072, 3584, 4096, 5120, 6144, 7168, 8192)] + \
       [(1, 8192, 8192), (16, 8192, 8192), (256, 256, 65536), (512, 512, 16384)]

# bf16 cubes in the other three storage orders (an operand contiguous along m / n takes the transposing LDS reads of the
# direct-to-LDS kernel): (transA, transB) x size
BF16_ORDERS = [(ta, tb, n) for n in (1024, 1536, 2048, 2560, 3072, 3584, 4096, 5120, 6144) for ta, tb in ((0, 0), (1, 1), (1, 0))]


# the normal equations of the paper's Task 20: X^T X and X^T y for X of n x 10 (a transposed A against a row-major B)
F32_TALL = [(10, 10, 1 << e) for e in (14, 18, 22)] + [(10, 1, 1 << e) for e in (14, 18, 22)]


# a few rows or columns on one side (the streaming kernels, on the vector units or the matrix cores, against tiles with K slices):
# (kind, transA, transB, M, N, K)
THIN = [("f32", 0, 0, 8, 8192, 8192), ("f32", 0, 1, 8, 8192, 8192), ("f32", 0, 0, 4, 8192, 8192), ("f32", 0, 0, 8192, 8, 8192),
        ("f32", 1, 0, 8192, 8, 8192), ("f32", 0, 0, 8, 2048, 8192), ("f32", 0, 0, 8, 1024, 16384), ("f32", 0, 0, 3, 16384, 4096),
        ("bf16", 0, 1, 8, 8192, 8192), ("bf16", 0, 0, 8, 8192, 8192), ("bf16", 0, 1, 16, 8192, 8192), ("bf16", 0, 0, 4, 8192, 8192),
        ("bf16", 0, 1, 2, 8192, 8192), ("bf16", 0, 1, 12, 1024, 16384), ("bf16", 0, 1, 16, 28672, 8192), ("bf16", 0, 1, 8192, 16, 8192),
        ("bf16", 1, 1, 8192, 4, 8192), ("f32", 0, 0, 16, 8192, 8192), ("f32", 0, 1, 16, 8192, 8192), ("f32", 1, 0, 8192, 12, 8192),
        ("f32", 0, 0, 8192, 16, 8192), ("f32", 0, 1, 8, 2048, 8192), ("f32", 0, 1, 8, 1024, 16384)]


def host_operands(p: Problem, seed: int):
    if p.kind == "f32":
        A, B = inputs.uniform_pm1(seed, 1, p.M, p.K), inputs.uniform_pm1(seed, 2, p.K, p.N)
        return A, B, (A.T.copy() if p.transA else A), (B.T.copy() if p.transB else B)
    s = 1 / math.sqrt(max(p.K, 1))
    A, Bt = inputs.bf16_normal_scaled(seed, 1, p.M, p.K, s), inputs.bf16_normal_scaled(seed, 2, p.N, p.K, s)
    return A, Bt.T, (A.T.copy() if p.transA else A), (Bt if p.transB else Bt.T.copy())


class OracleValidator:
    """The function validator: the candidate's whole result against the oracle for small problems, 8192 sampled
    entries for large ones; the tolerance and the error measure of the parity tests."""

    def __init__(self, p: Problem, A, B, full_limit=1 << 27):
        self.p, self.tol = p, (1e-5 if p.kind == "f32" else 1e-2)
        if p.M * p.N * p.K <= full_limit:
            self.idx = None
            self.ref, self.S = oracle.gemm(A, B)
        else:
            rng = np.random.default_rng(11)
            self.idx = (rng.integers(0, p.M, 8192), rng.integers(0, p.N, 8192))
            self.ref, self.S = oracle.gemm_entries(A, B, *self.idx)

    def __call__(self, got) -> bool:
        if not np.all(np.isfinite(got)):
            return False
        g = got if self.idx is None else got[self.idx]
        return bool(oracle.componentwise_error(g, self.ref, self.S) <= self.tol)


def tune(lib, torch, p: Problem, gain: float, log):
    A, B, stA, stB = host_operands(p, 21)
    be = fsr_search.DeviceBackend(lib, torch, p, stA, stB)
    validator = OracleValidator(p, A, B)
    rows, report = [], dict(problem=p._asdict())
    for with_ws in (False, True):
        start, rules = (be.start, be.rules) if with_ws else (be.start_unsplit, be.rules_unsplit)
        be.offer_workspace = with_ws
        r = fsr_search.search(start, be.tile_count, be.runs, lambda c: validator(be.output(c)), be.latency,
                              rounds=3, per_round=4, max_slices=fsr_search.MAX_SLICES if with_ws else 1, log=log, chain=be.chain)
        best = r["best"]
        entry = dict(start=start, rules=rules, best=best, visited={"%d/%d" % k: v for k, v in r["visited"].items()})
        as_run = (be.rules_bands if with_ws else be.rules_bands_unsplit) or rules
        if best is not None and best != as_run and be.runs(rules) and validator(be.output(rules)):
            # the incumbent against the choice of the rules (their two-band plan where they make one), measured again,
            # both ways round; a row only for a clear gain
            entry["rules_as_run"] = as_run
            t_rules = min(be.latency(as_run), be.latency(as_run))
            t_best = max(be.latency(best), be.latency(best))
            entry.update(t_rules=t_rules, t_best=t_best)
            if t_best < (1 - gain) * t_rules:
                rows.append(fsr_search.table_row(p, with_ws, best))
        report["with_workspace" if with_ws else "plain"] = entry
    del be
    torch.cuda.empty_cache()
    return rows, report


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--out", required=True)
    ap.add_argument("--log", default=None)
    ap.add_argument("--only", choices=["f32", "bf16", "bf16-orders", "thin"], default=None)
    ap.add_argument("--gain", type=float, default=0.04)
    args = ap.parse_args()

    import torch

    import paper_2506_09092_amd as lib

    lib.load()
    assert torch.cuda.is_available(), "needs a GPU"
    torch.cuda.set_device(0)

    def log(msg):
        print(msg, flush=True)

    problems = [Problem("f32", 0, 0, *s) for s in F32 if args.only in (None, "f32")] + \
               [Problem("f32", 1, 0, *s) for s in F32_TALL if args.only in (None, "f32")] + \
               [Problem("bf16", 0, 1, *s) for s in BF16 if args.only in (None, "bf16")] + \
               [Problem("bf16", ta, tb, n, n, n) for ta, tb, n in BF16_ORDERS if args.only in (None, "bf16-orders")] + \
               [Problem(*t) for t in THIN if args.only in (None, "thin")]
    rows, reports = [], []
    for p in problems:
        log("== %s" % (p,))
        r, rep = tune(lib, torch, p, args.gain, log)
        rows += r
        reports.append(rep)
        log("   rows: %s" % (r,))
        with open(args.out, "w") as f:
            f.write("// {kind (0 fp32, 1 bf16), transA, transB, M, N, K, ws (1: for calls that bring a workspace), tile, K slices}:\n"
                    "// written by the selection loop, one row per problem whose measured best differs from the dispatcher's rules.\n")
            f.write("".join(x + "\n" for x in rows))
        if args.log:
            with open(args.log, "w") as f:
                json.dump(reports, f, indent=1, default=str)


if __name__ == "__main__":
    main()
