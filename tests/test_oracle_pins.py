"""Pins for the CPU oracle: everything here is fixed by the definition C = A x B
(paper, Task 2) and by arithmetic, never by the oracle's own output or by the GPU."""
import itertools
import math
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_2506_09092_amd import inputs

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _ints(rng, shape, lo=-4, hi=4):
    return rng.integers(lo, hi + 1, size=shape).astype(np.float32)


def test_golden_worked_examples():
    cases, cur = [], {}
    for line in open(os.path.join(GOLDEN, "task2_tiny.txt")):
        if line.startswith("#") or not line.strip():
            continue
        tok = line.split()
        if tok[0] == "M":
            cur = dict(M=int(tok[1]), N=int(tok[3]), K=int(tok[5]))
            cases.append(cur)
        else:
            cur[tok[0]] = [float(t) for t in tok[1:]]
    assert len(cases) == 2
    for c in cases:
        A = np.array(c["A"], dtype=np.float32).reshape(c["M"], c["K"])
        B = np.array(c["B"], dtype=np.float32).reshape(c["K"], c["N"])
        C, S = oracle.gemm(A, B)
        assert C.tolist() == np.array(c["C"]).reshape(c["M"], c["N"]).tolist()


def test_brute_force_tiny_shapes_exact_integers():
    rng = np.random.default_rng(11)
    shapes = list(itertools.product((1, 2, 3), repeat=3)) + [(2, 3, 4), (4, 2, 3), (3, 5, 2), (5, 1, 7)]
    for M, N, K in shapes:
        A, B = _ints(rng, (M, K), -9, 9), _ints(rng, (K, N), -9, 9)
        C, S = oracle.gemm(A, B)
        for i in range(M):
            for j in range(N):
                want = sum(int(A[i, k]) * int(B[k, j]) for k in range(K))
                wabs = sum(abs(int(A[i, k])) * abs(int(B[k, j])) for k in range(K))
                assert C[i, j] == want and S[i, j] == wabs, (M, N, K, i, j)


def test_exact_rational_on_random_fp32():
    # Exact value of each dot product in rational arithmetic; the oracle may differ
    # only by its K-1 fp64 roundings: |C - exact| <= K * 2^-53 * S.
    A = inputs.uniform_pm1(5, 1, 4, 37)
    B = inputs.uniform_pm1(5, 2, 37, 3)
    C, S = oracle.gemm(A, B)
    for i in range(4):
        for j in range(3):
            exact = sum(Fraction(float(A[i, k])) * Fraction(float(B[k, j])) for k in range(37))
            sabs = sum(abs(Fraction(float(A[i, k])) * Fraction(float(B[k, j]))) for k in range(37))
            assert abs(Fraction(C[i, j]) - exact) <= 37 * Fraction(1, 2 ** 53) * sabs
            assert abs(Fraction(S[i, j]) - sabs) <= 37 * Fraction(1, 2 ** 53) * sabs


def test_identity_is_bit_exact():
    A = inputs.uniform_pm1(1, 1, 19, 23)
    B = inputs.normal(1, 2, 23, 17)
    C, _ = oracle.gemm(A, np.eye(23, dtype=np.float32))
    assert np.array_equal(C, A.astype(np.float64))
    C, _ = oracle.gemm(np.eye(23, dtype=np.float32), B)
    assert np.array_equal(C, B.astype(np.float64))


def test_permutation_moves_rows_and_columns():
    rng = np.random.default_rng(3)
    A = inputs.uniform_pm1(2, 1, 7, 11)
    B = inputs.uniform_pm1(2, 2, 11, 5)
    p = rng.permutation(11)
    P = np.zeros((11, 11), dtype=np.float32)
    P[np.arange(11), p] = 1.0            # (A P)[:, p[k]] = A[:, k];  (P B)[k, :] = B[p[k], :]
    C, _ = oracle.gemm(A, P)
    want = np.empty_like(A)
    want[:, p] = A
    assert np.array_equal(C, want.astype(np.float64))
    C, _ = oracle.gemm(P, B)
    assert np.array_equal(C, B[p].astype(np.float64))


def test_rank_one_and_closed_forms():
    rng = np.random.default_rng(4)
    M, N, K = 9, 13, 21
    u, v = _ints(rng, (M,), -7, 7), _ints(rng, (N,), -7, 7)
    A = np.repeat(u[:, None], K, axis=1)
    B = np.repeat(v[None, :], K, axis=0)
    C, S = oracle.gemm(A, B)
    assert np.array_equal(C, K * np.outer(u, v).astype(np.float64))
    assert np.array_equal(S, K * np.abs(np.outer(u, v)).astype(np.float64))
    ones = lambda r, c: np.ones((r, c), dtype=np.float32)
    assert np.array_equal(oracle.gemm(ones(M, K), ones(K, N))[0], np.full((M, N), float(K)))
    ramp = np.repeat(np.arange(K, dtype=np.float32)[None, :], M, axis=0)
    assert np.array_equal(oracle.gemm(ramp, ones(K, N))[0], np.full((M, N), K * (K - 1) / 2.0))
    for KK in (20, 21):
        alt = np.repeat(((-1.0) ** np.arange(KK)).astype(np.float32)[None, :], M, axis=0)
        assert np.array_equal(oracle.gemm(alt, ones(KK, N))[0], np.full((M, N), float(KK % 2)))
    # outer product (K = 1) of non-integers: one exact fp64 product per entry
    a, b = inputs.uniform_pm1(6, 1, 5, 1), inputs.uniform_pm1(6, 2, 1, 4)
    assert np.array_equal(oracle.gemm(a, b)[0], a.astype(np.float64) * b.astype(np.float64))


def test_transpose_identity_through_strides():
    # (A B)^T = B^T A^T; passing transposed *views* makes the oracle walk the same
    # memory with swapped strides, and each sum has the same terms in the same order.
    A = inputs.uniform_pm1(7, 1, 6, 10)
    B = inputs.uniform_pm1(7, 2, 10, 8)
    C, S = oracle.gemm(A, B)
    Ct, St = oracle.gemm(B.T, A.T)
    assert np.array_equal(Ct.T, C) and np.array_equal(St.T, S)
    # column-major storage of B (as the bf16 entry point uses) gives the same numbers
    Bcol = np.asfortranarray(B)
    assert Bcol.strides != B.strides
    assert np.array_equal(oracle.gemm(A, Bcol)[0], C)


def test_block_splitting_and_k_additivity():
    A = inputs.normal(8, 1, 12, 30)
    B = inputs.normal(8, 2, 30, 14)
    C, S = oracle.gemm(A, B)
    assert np.array_equal(np.hstack([oracle.gemm(A, B[:, :5])[0], oracle.gemm(A, B[:, 5:])[0]]), C)
    assert np.array_equal(np.vstack([oracle.gemm(A[:4], B)[0], oracle.gemm(A[4:], B)[0]]), C)
    C2 = oracle.gemm(A[:, :13], B[:13])[0] + oracle.gemm(A[:, 13:], B[13:])[0]
    assert np.all(np.abs(C2 - C) <= 30 * 2.0 ** -52 * S)
    assert np.array_equal(oracle.gemm(A * np.float32(4.0), B * np.float32(0.125))[0], C * 0.5)


def test_leading_dimension_independence():
    A = inputs.uniform_pm1(9, 1, 10, 9)
    B = inputs.uniform_pm1(9, 2, 9, 7)
    C, S = oracle.gemm(A, B)
    Ap = inputs.embed(A, 9 + 5, np.nan, offset=3)[3:].reshape(10, 14)[:, :9]
    Bp = inputs.embed(B, 7 + 2, np.nan)[:].reshape(9, 9)[:, :7]
    Cp, Sp = oracle.gemm(Ap, Bp)
    assert np.array_equal(Cp, C) and np.array_equal(Sp, S)


def test_summation_order_within_bound_and_fsum():
    A = inputs.normal(10, 1, 5, 513)
    B = inputs.normal(10, 2, 513, 6)
    C, S = oracle.gemm(A, B)
    Cr, _ = oracle.gemm(A[:, ::-1], B[::-1])         # same products, reverse k
    assert np.all(np.abs(Cr - C) <= 513 * 2.0 ** -52 * S)
    for i in range(5):
        for j in range(6):
            terms = [float(A[i, k]) * float(B[k, j]) for k in range(513)]   # each exact in fp64
            assert abs(math.fsum(terms) - C[i, j]) <= 513 * 2.0 ** -53 * S[i, j]
            assert abs(math.fsum(abs(t) for t in terms) - S[i, j]) <= 513 * 2.0 ** -53 * S[i, j]


def test_integer_config_matches_int64_matmul():
    # the 256^3 integer-valued configuration: exact in every arithmetic
    A = inputs.small_ints(0, 3, 256, 256)
    B = inputs.small_ints(0, 4, 256, 256)
    C, S = oracle.gemm(A, B)
    want = A.astype(np.int64) @ B.astype(np.int64)
    assert np.array_equal(C, want.astype(np.float64))
    assert np.array_equal(S, (np.abs(A).astype(np.int64) @ np.abs(B).astype(np.int64)).astype(np.float64))


def test_bf16_path_widens_exactly():
    Ab = inputs.bf16_normal_scaled(4, 1, 9, 40, 1 / math.sqrt(40))
    Bb = inputs.bf16_normal_scaled(4, 2, 11, 40, 1 / math.sqrt(40))       # stored as N x K = column-major K x N
    C16, S16 = oracle.gemm(Ab, Bb.T)
    C32, S32 = oracle.gemm(inputs.bf16_bits_to_f32(Ab), inputs.bf16_bits_to_f32(Bb).T)
    assert np.array_equal(C16, C32) and np.array_equal(S16, S32)
    # known bit patterns: 0x3F80 = 1, 0xC000 = -2, 0x4040 = 3, 0x3F00 = 0.5
    A = np.array([[0x3F80, 0xC000, 0x4040]], dtype=np.uint16)
    B = np.array([[0x3F00], [0x3F80], [0xC000]], dtype=np.uint16)
    C, S = oracle.gemm(A, B)
    assert C[0, 0] == 0.5 - 2.0 - 6.0 and S[0, 0] == 8.5
    Ai, Bi = inputs.bf16_small_ints(0, 5, 16, 33), inputs.bf16_small_ints(0, 6, 33, 8)
    want = inputs.bf16_bits_to_f32(Ai).astype(np.int64) @ inputs.bf16_bits_to_f32(Bi).astype(np.int64)
    assert np.array_equal(oracle.gemm(Ai, Bi)[0], want.astype(np.float64))


def test_entries_agree_with_definition():
    A = inputs.normal(12, 1, 20, 70)
    B = inputs.normal(12, 2, 70, 30)
    rng = np.random.default_rng(0)
    ii, jj = rng.integers(0, 20, 50), rng.integers(0, 30, 50)
    c, s = oracle.gemm_entries(A, B, ii, jj)
    for t in range(50):
        terms = [float(A[ii[t], k]) * float(B[k, jj[t]]) for k in range(70)]
        assert abs(math.fsum(terms) - c[t]) <= 70 * 2.0 ** -53 * s[t]
    C, S = oracle.gemm(A, B)
    assert np.array_equal(c, C[ii, jj]) and np.array_equal(s, S[ii, jj])
    Ab, Bb = inputs.to_bf16_bits(A), inputs.to_bf16_bits(B.T.copy())
    c, s = oracle.gemm_entries(Ab, Bb.T, ii, jj)
    C, S = oracle.gemm(Ab, Bb.T)
    assert np.array_equal(c, C[ii, jj]) and np.array_equal(s, S[ii, jj])


def test_scale_is_product_of_magnitudes():
    A = inputs.normal(13, 1, 8, 33)
    B = inputs.normal(13, 2, 33, 9)
    _, S = oracle.gemm(A, B)
    Cabs, _ = oracle.gemm(np.abs(A), np.abs(B))
    assert np.array_equal(S, Cabs)


def test_thread_count_does_not_change_bits():
    A = inputs.normal(14, 1, 64, 100)
    B = inputs.normal(14, 2, 100, 48)
    n = oracle.num_threads()
    try:
        oracle.set_num_threads(1)
        C1, S1 = oracle.gemm(A, B)
        oracle.set_num_threads(max(2, n))
        C2, S2 = oracle.gemm(A, B)
    finally:
        oracle.set_num_threads(n)
    assert np.array_equal(C1, C2) and np.array_equal(S1, S2)


def test_degenerate_extents():
    A0 = np.zeros((3, 0), dtype=np.float32)
    B0 = np.zeros((0, 4), dtype=np.float32)
    C, S = oracle.gemm(A0, B0)
    assert C.shape == (3, 4) and np.all(C == 0) and not np.any(np.signbit(C)) and np.all(S == 0)
    assert oracle.gemm(np.zeros((0, 5), np.float32), np.zeros((5, 2), np.float32))[0].shape == (0, 2)
    with pytest.raises(ValueError):
        oracle.gemm(np.zeros((2, 3), np.float32), np.zeros((4, 2), np.float32))


def test_error_metric_and_freivalds_detect_planted_mistakes():
    A = inputs.uniform_pm1(15, 1, 40, 64)
    B = inputs.uniform_pm1(15, 2, 64, 50)
    C, S = oracle.gemm(A, B)
    good = C.astype(np.float32)
    assert oracle.componentwise_error(good, C, S) <= 2.0 ** -24
    assert oracle.freivalds_residual(A, B, good) <= 1e-6
    # a dropped k term, a transposed operand, one corrupted entry, a NaN
    drop, _ = oracle.gemm(A[:, :-1], B[:-1])
    assert oracle.componentwise_error(drop.astype(np.float32), C, S) > 1e-4
    assert oracle.freivalds_residual(A, B, drop) > 1e-4
    sq = inputs.uniform_pm1(15, 3, 64, 64)
    Ct, _ = oracle.gemm(A, sq.T)
    Cn, Sn = oracle.gemm(A, sq)
    assert oracle.componentwise_error(Ct, Cn, Sn) > 1e-2
    bad = good.copy()
    bad[17, 23] += 1e-2
    assert oracle.componentwise_error(bad, C, S) > 1e-4
    assert oracle.freivalds_residual(A, B, bad) > 1e-5
    bad[3, 3] = np.nan
    assert oracle.componentwise_error(bad, C, S) == float("inf")
    assert oracle.freivalds_residual(A, B, bad) == float("inf")
    assert oracle.componentwise_error(np.zeros((0, 3)), np.zeros((0, 3)), np.zeros((0, 3))) == 0.0


def test_bf16_widening_matches_the_format():
    # bfloat16 is the upper half of an IEEE binary32: 1 sign, 8 exponent, 7 fraction bits.  Known patterns, worked by
    # hand from the format, then every one of the 65536 patterns against a decoder written out from that definition.
    known = {0x3F80: 1.0, 0xC000: -2.0, 0x4040: 3.0, 0x3F00: 0.5, 0x0001: 2.0 ** -133, 0x0080: 2.0 ** -126, 0x7F7F: (2 - 2.0 ** -7) * 2.0 ** 127,
             0x3FC0: 1.5, 0xBF81: -(1 + 2.0 ** -7), 0x0000: 0.0, 0x4049: 3.140625}
    bits = np.array(sorted(known), dtype=np.uint16)
    assert list(oracle.bf16_bits_to_f64(bits)) == [known[int(b)] for b in bits]
    assert oracle.bf16_bits_to_f64(np.array([0x8000], dtype=np.uint16))[0] == 0.0 and np.signbit(oracle.bf16_bits_to_f64(np.array([0x8000], dtype=np.uint16))[0])
    assert oracle.bf16_bits_to_f64(np.array([0x7F80], dtype=np.uint16))[0] == np.inf and np.isnan(oracle.bf16_bits_to_f64(np.array([0x7FC1], dtype=np.uint16))[0])

    def decode(b):
        sign, e, f = -1.0 if b >> 15 else 1.0, (b >> 7) & 0xFF, b & 0x7F
        if e == 0xFF:
            return sign * np.inf if f == 0 else np.nan
        return sign * (f * 2.0 ** -7 * 2.0 ** -126 if e == 0 else (1 + f * 2.0 ** -7) * 2.0 ** (e - 127))

    every = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    want = np.array([decode(int(b)) for b in every])
    with np.errstate(invalid="ignore"):         # signalling NaN patterns are among the 65536
        got = oracle.bf16_bits_to_f64(every)
    assert np.array_equal(np.isnan(got), np.isnan(want)) and np.array_equal(got[~np.isnan(got)], want[~np.isnan(want)])
    assert np.array_equal(np.signbit(got[~np.isnan(got)]), np.signbit(want[~np.isnan(want)]))
    # a matrix keeps its shape, and the widening agrees with the C routine's (a 1 x 1 product with 1.0)
    m = every[:4096].reshape(64, 64)
    assert oracle.bf16_bits_to_f64(m).shape == (64, 64)
    one = np.array([[0x3F80]], dtype=np.uint16)
    finite = every[(every & 0x7F80) != 0x7F80][::97]
    via_c = np.array([oracle.gemm(np.array([[b]], dtype=np.uint16), one)[0][0, 0] for b in finite])
    assert np.array_equal(via_c, oracle.bf16_bits_to_f64(finite))


def test_freivalds_on_bf16_bit_patterns_detects_planted_mistakes():
    # the residual check is what covers all entries of the bf16 8192^3 product, so its bf16 branch is pinned on its
    # own: operands are uint16 bit patterns, B is handed over as the K x N view of a column-major (N x K) array
    import math

    M, N, K = 48, 80, 96
    A = inputs.bf16_normal_scaled(16, 1, M, K, 1 / math.sqrt(K))
    Bt = inputs.bf16_normal_scaled(16, 2, N, K, 1 / math.sqrt(K))
    C, S = oracle.gemm(A, Bt.T)
    good = C.astype(np.float32)
    # exact arithmetic on the widened values (Python integers scaled by 2^-300 would do as well; fractions are plainer)
    from fractions import Fraction
    x = np.ones(N)
    Af, Bf = oracle.bf16_bits_to_f64(A), oracle.bf16_bits_to_f64(Bt.T)
    row0 = sum(Fraction(float(Af[0, k])) * sum(Fraction(float(Bf[k, j])) for j in range(N)) for k in range(K))
    assert abs(float(row0) - float(C[0] @ x)) <= 1e-12
    base = oracle.freivalds_residual(A, Bt.T, good)
    assert base <= 2.0 ** -24                    # fp32 rounding of each entry, averaged down by the random signs
    assert oracle.freivalds_residual(A, Bt.T, C) <= 1e-14
    # a dropped k term; B taken row-major instead of column-major (same bytes); one corrupted entry; a wrong 16 x 16
    # block; operands widened as if they were integers; a NaN
    drop, _ = oracle.gemm(A[:, :-1], Bt.T[:-1])
    assert oracle.freivalds_residual(A, Bt.T, drop) > 1e-4
    sq = inputs.bf16_normal_scaled(16, 3, K, K, 1 / math.sqrt(K))
    Ct, _ = oracle.gemm(A, sq)
    assert oracle.freivalds_residual(A, sq.T, Ct) > 1e-3
    bad = good.copy()
    bad[17, 23] += np.float32(1e-2) * np.float32(S[17, 23])
    assert oracle.freivalds_residual(A, Bt.T, bad) > 1e-2 / N / 2
    blk = good.copy()
    blk[16:32, 32:48] = 0.0
    assert oracle.freivalds_residual(A, Bt.T, blk) > 1e-3
    as_ints = A.astype(np.float32) @ Bt.T.astype(np.float32)
    assert oracle.freivalds_residual(A, Bt.T, as_ints) > 1.0
    bad[3, 3] = np.nan
    assert oracle.freivalds_residual(A, Bt.T, bad) == float("inf")
    # the fp32 branch on the same values (bf16 widened to fp32 exactly) gives the same number: same vectors, same sums
    A32, B32 = Af.astype(np.float32), Bf.astype(np.float32)
    assert oracle.freivalds_residual(A32, B32, good) == base


# ---- transposition (Task 8) ----

def _golden_transposes():
    path = os.path.join(os.path.dirname(__file__), "golden", "task8_tiny.txt")
    cases, cur = [], {}
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        tok = line.split()
        if tok[0] == "ROWS":
            cur = {"rows": int(tok[1]), "cols": int(tok[3])}
            cases.append(cur)
        else:
            cur[tok[0]] = np.array([float(x) for x in tok[1:]], dtype=np.float32)
    return cases


def test_ieee_special_values_follow_the_standard():
    # what IEEE 754 fixes for sums of products with infinities, NaNs and subnormal numbers, worked by hand
    inf, nan = np.inf, np.nan
    A = np.array([[inf, 0, 1], [1, 2, 3], [inf, -inf, 0], [nan, 0, 0], [2.0 ** -149, 0, 0], [-inf, 1, 1]], dtype=np.float32)
    B = np.array([[0, 1], [1, 1], [1, 1]], dtype=np.float32)
    C, S = oracle.gemm(A, B)
    assert np.isnan(C[0, 0]) and C[0, 1] == inf                  # inf * 0 is NaN; inf + finite is inf
    assert list(C[1]) == [5.0, 6.0]                              # rows without special values are untouched by the others
    assert np.isnan(C[2, 0]) and np.isnan(C[2, 1])               # (inf * 0) and (inf - inf)
    assert np.isnan(C[3]).all()                                  # NaN times zero is NaN
    assert C[4, 0] == 0.0 and C[4, 1] == 2.0 ** -149             # the smallest subnormal survives (fp64 holds it exactly)
    assert np.isnan(C[5, 0]) and C[5, 1] == -inf
    assert S[0, 1] == inf and S[5, 1] == inf and np.isnan(S[0, 0])
    # products of subnormals are exact in fp64: 3 * 2^-149 times 5 * 2^-149
    a, b = np.array([[3 * 2.0 ** -149]], dtype=np.float32), np.array([[5 * 2.0 ** -149]], dtype=np.float32)
    assert oracle.gemm(a, b)[0][0, 0] == 15 * 2.0 ** -298
    # bf16 patterns: 0x7F80 = +inf, 0xFF80 = -inf, 0x7FC0 = NaN, 0x0001 = 2^-133 (smallest subnormal)
    Ab = np.array([[0x7F80, 0x3F80], [0xFF80, 0x0000], [0x7FC0, 0x3F80], [0x0001, 0x0000]], dtype=np.uint16)
    Bb = np.array([[0x3F80], [0x3F80]], dtype=np.uint16)
    Cb = oracle.gemm(Ab, Bb)[0][:, 0]
    assert Cb[0] == inf and Cb[1] == -inf and np.isnan(Cb[2]) and Cb[3] == 2.0 ** -133


def test_transpose_golden_worked_examples():
    cases = _golden_transposes()
    assert len(cases) == 3
    for c in cases:
        T = oracle.transpose(c["A"].reshape(c["rows"], c["cols"]))
        assert T.shape == (c["cols"], c["rows"]) and T.flags["C_CONTIGUOUS"]
        assert np.array_equal(T.ravel(), c["T"])


def test_transpose_brute_force_and_strided_views():
    rng = np.random.default_rng(5)
    for rows, cols in ((1, 1), (1, 7), (7, 1), (2, 3), (5, 5), (13, 4), (31, 33), (64, 65)):
        A = rng.standard_normal((rows, cols)).astype(np.float32)
        T = oracle.transpose(A)
        for i in range(rows):
            for j in range(cols):
                assert T[j, i] == A[i, j]
        # the same logical matrix seen through padded and column-major storage
        padded = np.full((rows, cols + 3), np.float32(np.nan)); padded[:, :cols] = A
        assert np.array_equal(oracle.transpose(padded[:, :cols]), T)
        assert np.array_equal(oracle.transpose(np.asfortranarray(A)), T)


def test_transpose_is_an_involution_and_matches_the_library_view():
    rng = np.random.default_rng(6)
    A = rng.standard_normal((37, 91)).astype(np.float32)
    bits = A.view(np.uint32)
    bits[0, 0], bits[1, 2], bits[3, 4], bits[5, 6] = 0x80000000, 0x7FC12345, 0xFFC00001, 0x00000001   # -0, NaNs with payload, denormal
    T = oracle.transpose(A)
    assert np.array_equal(oracle.transpose(T).view(np.uint32), bits)          # twice is the identity, bit for bit
    assert np.array_equal(T.view(np.uint32), np.ascontiguousarray(A.T).view(np.uint32))   # numpy's own transposition
    Q = rng.standard_normal((37, 37)).astype(np.float32)
    S = Q + Q.T                                                                # a symmetric matrix is its own transpose
    assert np.array_equal(oracle.transpose(S), S)
    eye = np.eye(9, dtype=np.float32)
    assert np.array_equal(oracle.transpose(eye), eye)


def test_transpose_ties_in_with_the_product_oracle():
    # (A B)^T = B^T A^T with the transposes taken by this oracle and the products by the other one: every sum
    # has the same terms in the same order, so the two sides agree bit for bit
    A, B = inputs.uniform_pm1(9, 1, 23, 17), inputs.uniform_pm1(9, 2, 17, 29)
    left, _ = oracle.gemm(A, B)
    right, _ = oracle.gemm(oracle.transpose(B), oracle.transpose(A))
    assert np.array_equal(left.T, right)


def test_transpose_detects_planted_mistakes():
    A = inputs.uniform_pm1(9, 3, 6, 6)
    T = oracle.transpose(A)
    assert not np.array_equal(T, A)                              # a plain copy is not a transpose
    assert not np.array_equal(T, A[::-1, ::-1])                  # nor is a reversal
    wrong = T.copy(); wrong[2, 3], wrong[3, 2] = T[3, 2], T[2, 3]
    assert not np.array_equal(wrong, T)
    assert oracle.transpose(np.zeros((0, 5), dtype=np.float32)).shape == (5, 0)
    assert oracle.transpose(np.zeros((4, 0), dtype=np.float32)).shape == (0, 4)
