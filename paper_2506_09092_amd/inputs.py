"""Seeded synthetic inputs for the GEMM validator and profiler.

The paper's Function Validator runs each kernel on randomly generated inputs
at several sizes (its Section 3.2 and the input-size table in its appendix)
without stating their distribution; the matrices below stand in for them.

This module only *produces operands and shape lists*.  It contains none of the
multiplication itself and is the one piece of code that both the GPU tests and
the CPU oracle's tests draw from.

Every value is a pure function of (seed, matrix_id, row, col): a 64-bit
counter is pushed through the SplitMix64 finaliser.  A matrix therefore holds
the same numbers whatever leading dimension it is later stored with.
"""
from __future__ import annotations

import math

import numpy as np

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)


def _splitmix64(x: np.ndarray) -> np.ndarray:
    """SplitMix64 output function (Steele, Lea, Flood 2014) on uint64 arrays."""
    x = x.astype(np.uint64, copy=True)
    with np.errstate(over="ignore"):
        x += np.uint64(0x9E3779B97F4A7C15)
        x ^= x >> np.uint64(30)
        x *= np.uint64(0xBF58476D1CE4E5B9)
        x ^= x >> np.uint64(27)
        x *= np.uint64(0x94D049BB133111EB)
        x ^= x >> np.uint64(31)
    return x


def _key(seed: int, matrix_id: int, stream: int) -> np.uint64:
    k = (seed * 0x100000001B3 + matrix_id * 0x1000193 + stream * 0x10001) & 0xFFFFFFFFFFFFFFFF
    return _splitmix64(np.array([k], dtype=np.uint64))[0]


def raw_bits(seed: int, matrix_id: int, rows: int, cols: int, stream: int = 0,
             r0: int = 0, r1: int | None = None) -> np.ndarray:
    """uint64 rows r0..r1-1 of a (rows, cols) matrix; entry (r, c) is a function of
    (seed, matrix_id, stream, r*cols + c) alone."""
    r1 = rows if r1 is None else r1
    idx = np.arange(r0 * cols, r1 * cols, dtype=np.uint64)
    with np.errstate(over="ignore"):
        idx = idx * np.uint64(0xD1342543DE82EF95) + _key(seed, matrix_id, stream)
    return _splitmix64(idx).reshape(r1 - r0, cols)


def _row_chunks(rows: int, cols: int):
    step = max(1, (1 << 22) // max(cols, 1))          # ~4M elements at a time bounds host memory
    for r0 in range(0, rows, step):
        yield r0, min(rows, r0 + step)


def uniform_pm1(seed: int, matrix_id: int, rows: int, cols: int) -> np.ndarray:
    """float32, multiples of 2^-23 in [-1, 1): (top 24 bits - 2^23) * 2^-23, exact in fp32."""
    out = np.empty((rows, cols), dtype=np.float32)
    for r0, r1 in _row_chunks(rows, cols):
        t = (raw_bits(seed, matrix_id, rows, cols, 0, r0, r1) >> np.uint64(40)).astype(np.int64)
        out[r0:r1] = ((t - (1 << 23)).astype(np.float64) * 2.0 ** -23).astype(np.float32)
    return out


def small_ints(seed: int, matrix_id: int, rows: int, cols: int) -> np.ndarray:
    """float32 holding integers uniform in {-4, ..., 4}."""
    out = np.empty((rows, cols), dtype=np.float32)
    for r0, r1 in _row_chunks(rows, cols):
        t = raw_bits(seed, matrix_id, rows, cols, 0, r0, r1) >> np.uint64(32)
        out[r0:r1] = (((t * np.uint64(9)) >> np.uint64(32)).astype(np.int64) - 4).astype(np.float32)
    return out


def _box_muller(b: np.ndarray) -> np.ndarray:
    """Standard normal (fp64) from the two 32-bit halves of each 64-bit draw."""
    u1 = ((b >> np.uint64(32)).astype(np.float64) + 1.0) * 2.0 ** -32      # (0, 1]
    u2 = (b & np.uint64(0xFFFFFFFF)).astype(np.float64) * 2.0 ** -32        # [0, 1)
    return np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * math.pi * u2)


def normal(seed: int, matrix_id: int, rows: int, cols: int) -> np.ndarray:
    """float32 standard normal (Box-Muller in fp64, rounded once to fp32)."""
    out = np.empty((rows, cols), dtype=np.float32)
    for r0, r1 in _row_chunks(rows, cols):
        out[r0:r1] = _box_muller(raw_bits(seed, matrix_id, rows, cols, 0, r0, r1)).astype(np.float32)
    return out


def any_bits_f32(seed: int, matrix_id: int, rows: int, cols: int) -> np.ndarray:
    """float32 whose 32 bits are the top half of the raw draw: every bit pattern can occur (NaNs with
    payloads, infinities, denormals, both zeros).  For operations that only move data."""
    out = np.empty((rows, cols), dtype=np.uint32)
    for r0, r1 in _row_chunks(rows, cols):
        out[r0:r1] = (raw_bits(seed, matrix_id, rows, cols, 0, r0, r1) >> np.uint64(32)).astype(np.uint32)
    return out.view(np.float32)


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round to bfloat16 (nearest, ties to even) and return the uint16 bit patterns.

    Finite inputs only.  fp64 input is first rounded to fp32; the double
    rounding is immaterial here and this routine is the single source of the
    bits that both the GPU and the oracle receive.
    """
    w = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = np.uint32(0x7FFF) + ((w >> np.uint32(16)) & np.uint32(1))
    return ((w + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to float32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_normal_scaled(seed: int, matrix_id: int, rows: int, cols: int, scale: float) -> np.ndarray:
    """bf16 bits of N(0,1) * scale (scaled in fp64, rounded once to bf16)."""
    out = np.empty((rows, cols), dtype=np.uint16)
    for r0, r1 in _row_chunks(rows, cols):
        out[r0:r1] = to_bf16_bits(_box_muller(raw_bits(seed, matrix_id, rows, cols, 0, r0, r1)) * scale)
    return out


def bf16_small_ints(seed: int, matrix_id: int, rows: int, cols: int) -> np.ndarray:
    """bf16 bits of integers uniform in {-4..4} (all exactly representable)."""
    return to_bf16_bits(small_ints(seed, matrix_id, rows, cols))


def embed(x: np.ndarray, ld: int, fill, offset: int = 0) -> np.ndarray:
    """Flat buffer of offset + rows*ld elements pre-filled with ``fill`` holding x at leading dimension ld.

    The padding (columns cols..ld-1 of each row and the ``offset`` leading
    elements) keeps the fill value, which serves as a canary: NaN for inputs,
    a recognisable sentinel for outputs.
    """
    rows, cols = x.shape
    assert ld >= cols
    buf = np.full(offset + rows * ld, fill, dtype=x.dtype)
    view = buf[offset:].reshape(rows, ld)
    view[:, :cols] = x
    return buf


# 16 shapes that every sweep contains: ones, primes, tile multiples +- 1.
FORCED_SWEEP_SHAPES = (
    (1, 1, 1), (1, 1, 4096), (4096, 4096, 1), (1, 4096, 4096), (4096, 1, 17), (17, 17, 17),
    (1000, 1000, 1000), (4097, 17, 1000), (1, 1000, 4097), (4097, 4097, 129), (257, 255, 129),
    (64, 64, 4097), (33, 65, 31), (1023, 1025, 1000), (128, 128, 128), (4095, 4097, 63),
)
_PADS = (1, 3, 8, 37)


def sweep_cases(seed: int = 3, total: int = 64):
    """The seeded shape sweep: 16 forced triples, then log-uniform draws in [1, 4096].

    Each case is a dict with M, N, K, the three leading dimensions and a
    base-pointer offset in elements.  Even-indexed cases use tight leading
    dimensions; odd-indexed ones pad each row by 1, 3, 8 or 37 elements.  The
    first eight random cases start every buffer one element in, so their base
    pointers are only 4-byte aligned.
    """
    n_rand = total - len(FORCED_SWEEP_SHAPES)
    bits = raw_bits(seed, 0xC0FFEE, max(n_rand, 1), 8)
    u = (bits >> np.uint64(11)).astype(np.float64) * 2.0 ** -53
    shapes = list(FORCED_SWEEP_SHAPES)
    for t in range(n_rand):
        shapes.append(tuple(int(min(4096, max(1, math.floor(2.0 ** (12.0 * u[t, d]))))) for d in range(3)))
    cases = []
    for idx, (M, N, K) in enumerate(shapes):
        if idx % 2 == 1:
            r = idx - len(FORCED_SWEEP_SHAPES)
            src = bits[r % max(n_rand, 1)] if r >= 0 else raw_bits(seed, 0xBEEF, 1, 8)[0] + np.uint64(idx)
            pa, pb, pc = (_PADS[int(src[3 + d] >> np.uint64(62))] for d in range(3))
        else:
            pa = pb = pc = 0
        off = 1 if len(FORCED_SWEEP_SHAPES) <= idx < len(FORCED_SWEEP_SHAPES) + 8 else 0
        cases.append(dict(index=idx, M=M, N=N, K=K, lda=K + pa, ldb=N + pb, ldc=N + pc, offset=off))
    return cases
