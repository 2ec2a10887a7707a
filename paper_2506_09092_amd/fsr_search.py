"""Selection of a tile configuration per problem, shaped like the paper's Algorithm 1 (Feature Search and
Reinforcement) with the language model taken out: the candidates of a round are configurations of the library's
own kernels -- an output tile and a number of K slices, the arguments of ``gemm_f32_cfg`` / ``gemm_bf16_cfg`` --
instead of generated kernels, and the refinement step proposes the neighbours of the round's fastest candidate
instead of prompting with it.  The feature functions keep their roles (Section 3.2): a candidate must run (the
library accepts it for the problem: the part of the compilation check), must validate (the caller's function
validator: this module knows no reference result), and is then ranked by measured time (performance profiler).

Nothing here computes a product: ``DeviceBackend`` calls the library through its binding, and the validator is
handed in by the caller.
"""
from __future__ import annotations

import collections

Problem = collections.namedtuple("Problem", "kind transA transB M N K")          # kind: "f32" | "bf16"
Candidate = collections.namedtuple("Candidate", "tile slices")
Bands = collections.namedtuple("Bands", "dim at first second")     # a two-band plan of the dispatcher (fsrgemm_bands_*)

MAX_SLICES = 64


# Candidate numbers are handed out in the order the kernels were written, not by likeness: for bf16 the 256 x 256 tile of
# the direct-to-LDS kernel is candidate 0, its other shapes 5 .. 9, the general tiles 1 .. 3, the vector kernels 4.
# "One tile size up or down" walks this chain instead (general 256 x 256, then the direct-to-LDS shapes by falling area,
# then the smaller general tiles, then the vector kernels).
TILE_CHAIN = {"bf16": (1, 0, 5, 7, 8, 6, 9, 10, 2, 3, 4)}


def neighbours(c: Candidate, tile_count: int, max_slices: int = MAX_SLICES, chain=None):
    """The refinement step: one tile size up or down with the same slices, half or twice the slices with the same
    tile (max_slices = 1: the search for callers without a workspace).  Nearest first; the order is part of the
    result's determinism.  chain: the candidate numbers in order of likeness (default: their own order)."""
    out = []
    if chain is not None and c.tile in chain:
        at = chain.index(c.tile)
        near = [chain[i] for i in (at + 1, at - 1) if 0 <= i < len(chain)]
    else:
        near = [c.tile + 1, c.tile - 1]
    for t in near:
        if 0 <= t < tile_count:
            out.append(Candidate(t, c.slices))
    if c.slices * 2 <= max_slices:
        out.append(Candidate(c.tile, c.slices * 2))
    if c.slices >= 2:
        out.append(Candidate(c.tile, c.slices // 2))
    return out


def search(start: Candidate, tile_count: int, runs, validates, latency, rounds: int = 3, per_round: int = 4,
           max_slices: int = MAX_SLICES, log=None, chain=None):
    """Algorithm 1 over configurations.

    start            the dispatcher's current choice: round 0 proposes it and its neighbours
    runs(c)          -> bool: the library accepts candidate c for the problem and the launch succeeds
    validates(c)     -> bool: c's result passes the function validator (called only when runs(c))
    latency(c)       -> float: measured time of c (called only for valid candidates); smaller is better
    max_slices       1 restricts the candidates to unsplit ones
    rounds           D of the algorithm: rounds that produced a valid candidate
    per_round        N of the algorithm: candidates per round

    Returns dict(best, best_latency, rounds=[{candidates, valid, winner, latency}], visited).  A round without a
    valid candidate does not count towards `rounds` (the algorithm repeats the round with what failed as feedback:
    here the failed candidates are dropped and their neighbours proposed); the loop also ends when nothing is
    left to propose, which a finite configuration space, unlike a language model, runs into.
    """
    visited, history = {}, []
    queue = [start] + neighbours(start, tile_count, max_slices, chain)
    best, best_t, d = None, float("inf"), 0
    while d < rounds:
        batch = []
        while queue and len(batch) < per_round:
            c = queue.pop(0)
            if c not in visited and c not in batch:
                batch.append(c)
        if not batch:
            break
        valid = []
        for c in batch:
            ok = bool(runs(c))
            visited[c] = "rejected" if not ok else ("valid" if validates(c) else "mismatch")
            if visited[c] == "valid":
                valid.append(c)
        if not valid:
            history.append(dict(candidates=batch, valid=[], winner=None, latency=None))
            for c in batch:                          # feedback of a failed round: look around what failed
                queue.extend(n for n in neighbours(c, tile_count, max_slices, chain) if n not in visited)
            if log:
                log("round without a valid candidate: %s" % (batch,))
            continue
        times = {c: float(latency(c)) for c in valid}
        winner = min(valid, key=lambda c: (times[c], c))
        if times[winner] < best_t:
            best, best_t = winner, times[winner]
        history.append(dict(candidates=batch, valid=valid, winner=winner, latency=times))
        if log:
            log("round %d: %s -> %s %.4f" % (d, ["%d/%d" % c for c in batch], "%d/%d" % winner, times[winner]))
        d += 1
        # refine around the round's winner first, then around the incumbent, then around the round's other
        # valid candidates, fastest first
        near = [n for c in (winner, best) for n in neighbours(c, tile_count, max_slices, chain)]
        others = sorted((c for c in valid if c != winner), key=lambda c: (times[c], c))
        far = [n for c in others for n in neighbours(c, tile_count, max_slices, chain)]
        queue = [n for n in near + queue + far if n not in visited]
    return dict(best=best, best_latency=best_t, rounds=history, visited=visited)


class DeviceBackend:
    """Runs and times candidates of one problem on the current GPU through the library's binding.

    hostA, hostB: the operands as numpy arrays in the storage the problem states (A: M x K, or K x M when transA;
    B: K x N, or N x K when transB; float32, or uint16 bf16 patterns).  Several copies of the operands are
    rotated through while timing so that a launch does not find its inputs in the caches of the one before.
    """

    def __init__(self, lib, torch, problem: Problem, hostA, hostB, copies_bytes: int = 1 << 30):
        self.lib, self.torch, self.p = lib, torch, problem
        p = problem
        assert hostA.shape == ((p.K, p.M) if p.transA else (p.M, p.K)) and hostB.shape == ((p.N, p.K) if p.transB else (p.K, p.N))
        per_set = hostA.nbytes + hostB.nbytes + 4 * p.M * p.N
        n_sets = int(max(1, min(4, copies_bytes // max(per_set, 1))))
        a0 = torch.from_numpy(hostA if p.kind == "f32" else hostA.view("int16")).to("cuda")
        b0 = torch.from_numpy(hostB if p.kind == "f32" else hostB.view("int16")).to("cuda")
        self.sets = [(a0, b0, torch.empty(p.M, p.N, device="cuda"))]
        for _ in range(n_sets - 1):
            self.sets.append((a0.clone(), b0.clone(), torch.empty(p.M, p.N, device="cuda")))
        self.lda, self.ldb = hostA.shape[1], hostB.shape[1]
        self.ws = torch.empty(16 << 20, dtype=torch.uint8, device="cuda")
        # set for a search on behalf of callers that bring a workspace: then every candidate is offered it (one
        # that needs none ignores it), otherwise only the split ones, which cannot run without
        self.offer_workspace = False
        self.fn = lib.gemm_f32_cfg if p.kind == "f32" else lib.gemm_bf16_cfg
        self.tile_count = lib.fsrgemm_tile_count_f32() if p.kind == "f32" else lib.fsrgemm_tile_count_bf16()
        self.chain = TILE_CHAIN.get(p.kind)
        plan = lib.fsrgemm_plan_f32 if p.kind == "f32" else lib.fsrgemm_plan_bf16
        args = (p.transA, p.transB, p.M, p.N, p.K, a0, self.lda, b0, self.ldb)
        # the dispatcher's choice with / without a workspace, and what its rules alone would take
        self.start, self.start_unsplit = Candidate(*plan(*args, True)), Candidate(*plan(*args, False))
        self.rules, self.rules_unsplit = Candidate(*plan(*args, True, True)), Candidate(*plan(*args, False, True))
        # where the rules run the product as two bands of C (one forced call each), that plan: (dim, at, first tile,
        # second tile) with dim 1 = rows, 2 = columns, at = the cut; None where they launch once
        bands = lib.fsrgemm_bands_f32 if p.kind == "f32" else lib.fsrgemm_bands_bf16
        two = lambda with_ws: (lambda b: Bands(*b) if b[0] else None)(bands(*args, with_ws, True))
        self.rules_bands, self.rules_bands_unsplit = two(True), two(False)

    def _call_bands(self, bd: "Bands", s: int) -> int:
        """The two forced calls of a two-band plan: each band is a product of its own on shifted operands."""
        p, (a, b, out) = self.p, self.sets[s]
        es = 4 if p.kind == "f32" else 2
        pa, pb, pc = a.data_ptr(), b.data_ptr(), out.data_ptr()
        stream = self.torch.cuda.current_stream().cuda_stream
        if bd.dim == 1:
            pa2, pb2, pc2 = pa + es * (bd.at if p.transA else bd.at * self.lda), pb, pc + 4 * bd.at * p.N
            shapes = ((bd.at, p.N), (p.M - bd.at, p.N))
        else:
            pa2, pb2, pc2 = pa, pb + es * (bd.at * self.ldb if p.transB else bd.at), pc + 4 * bd.at
            shapes = ((p.M, bd.at), (p.M, p.N - bd.at))
        rc = self.fn(bd.first, 1, p.transA, p.transB, shapes[0][0], shapes[0][1], p.K, pa, self.lda, pb, self.ldb, pc, p.N, None, 0, stream)
        if rc != self.lib.FSRGEMM_OK:
            return rc
        return self.fn(bd.second, 1, p.transA, p.transB, shapes[1][0], shapes[1][1], p.K, pa2, self.lda, pb2, self.ldb, pc2, p.N, None, 0, stream)

    def _call(self, c, s: int) -> int:
        if isinstance(c, Bands):
            return self._call_bands(c, s)
        p, (a, b, out) = self.p, self.sets[s]
        return self.fn(c.tile, c.slices, p.transA, p.transB, p.M, p.N, p.K, a, self.lda, b, self.ldb, out, p.N,
                       *((self.ws, self.ws.numel()) if self.offer_workspace or c.slices > 1 else (None, 0)),
                       self.torch.cuda.current_stream().cuda_stream)

    def runs(self, c: Candidate) -> bool:
        if self._call(c, 0) != self.lib.FSRGEMM_OK:
            return False
        self.torch.cuda.synchronize()
        return True

    def output(self, c: Candidate):
        """The candidate's product as a numpy array, computed into a NaN-filled result buffer."""
        self.sets[0][2].fill_(float("nan"))
        self.lib.check(self._call(c, 0))
        self.torch.cuda.synchronize()
        return self.sets[0][2].cpu().numpy()

    def latency(self, c, samples: int = 7, min_ms: float = 0.2, warm_ms: float = 20.0) -> float:
        """Median over `samples` timings of one call (a candidate, or a two-band plan) in ms.  Short launches are timed as a run of launches that
        lasts about min_ms, so that the gap between launches does not decide the ranking, and every candidate
        first runs for about warm_ms, so that the one measured first is not the one measured at idle clocks."""
        torch = self.torch
        n = len(self.sets)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for s in range(n):
            self.lib.check(self._call(c, s))
        e1.record()
        torch.cuda.synchronize()
        one = max(e0.elapsed_time(e1) / n, 1e-3)
        for r in range(int(min(256, warm_ms / one))):
            self._call(c, r % n)
        # the first calls may have paid for a first launch: size the runs by a run of warm calls
        e0.record()
        for r in range(16):
            self._call(c, r % n)
        e1.record()
        torch.cuda.synchronize()
        one = max(min(one, e0.elapsed_time(e1) / 16), 1e-3)
        reps = int(max(1, min(64, min_ms / one)))
        times = []
        for i in range(samples):
            e0.record()
            for r in range(reps):
                self._call(c, (i * reps + r) % n)
            e1.record()
            torch.cuda.synchronize()
            times.append(e0.elapsed_time(e1) / reps)
        return sorted(times)[samples // 2]


def table_row(problem: Problem, with_workspace: bool, c: Candidate) -> str:
    """One row of csrc/tuned_table.inc."""
    return "    {%d, %d, %d, %d, %d, %d, %d, %d, %d}," % (0 if problem.kind == "f32" else 1, int(bool(problem.transA)),
                                                        int(bool(problem.transB)), problem.M, problem.N, problem.K,
                                                        int(bool(with_workspace)), c.tile, c.slices)
