"""The seeded generators: determinism, stated value sets, shape-sweep composition."""
import numpy as np

from paper_2506_09092_amd import inputs


def test_values_depend_on_position_not_on_leading_dimension():
    a = inputs.uniform_pm1(3, 7, 9, 13)
    assert np.array_equal(a, inputs.uniform_pm1(3, 7, 9, 13))
    assert not np.array_equal(a, inputs.uniform_pm1(3, 8, 9, 13))
    assert not np.array_equal(a, inputs.uniform_pm1(4, 7, 9, 13))
    buf = inputs.embed(a, 20, np.float32(np.nan), offset=1)
    assert np.isnan(buf[0]) and np.array_equal(buf[1:].reshape(9, 20)[:, :13], a)
    assert np.all(np.isnan(buf[1:].reshape(9, 20)[:, 13:]))
    big = inputs.normal(2, 1, 3000, 2000)            # crosses the row-chunk boundary
    assert np.array_equal(big[2090:2110], inputs.normal(2, 1, 3000, 2000)[2090:2110])
    assert np.array_equal(inputs.raw_bits(2, 1, 3000, 2000, 0, 2097, 2099), inputs.raw_bits(2, 1, 3000, 2000)[2097:2099])


def test_distributions():
    u = inputs.uniform_pm1(0, 1, 256, 256)
    assert u.dtype == np.float32 and u.min() >= -1 and u.max() < 1
    assert np.all(u.astype(np.float64) * 2 ** 23 == np.round(u.astype(np.float64) * 2 ** 23))
    assert abs(u.mean()) < 0.01 and abs(u.std() - 3 ** -0.5) < 0.01
    i = inputs.small_ints(0, 2, 256, 256)
    vals, counts = np.unique(i, return_counts=True)
    assert vals.tolist() == list(range(-4, 5)) and counts.min() > 6500
    z = inputs.normal(2, 3, 512, 512)
    assert abs(z.mean()) < 0.01 and abs(z.std() - 1) < 0.01 and np.all(np.isfinite(z))


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.00390625, 1.005859375, 1.01171875, -2.5, 0.0, 3.140625], dtype=np.float32)
    # 1 + 2^-8 is a tie between 1.0 (even) and 1 + 2^-7; 1 + 3*2^-9 rounds up; 1 + 3*2^-8 ties to even (up)
    got = inputs.bf16_bits_to_f32(inputs.to_bf16_bits(x))
    assert got.tolist() == [1.0, 1.0, 1.0078125, 1.015625, -2.5, 0.0, 3.140625]
    ints = inputs.bf16_bits_to_f32(inputs.bf16_small_ints(0, 1, 64, 64))
    assert set(np.unique(ints).tolist()) == set(float(v) for v in range(-4, 5))
    b = inputs.bf16_normal_scaled(4, 1, 64, 1024, 1 / 32.0)
    assert abs(inputs.bf16_bits_to_f32(b).std() * 32 - 1) < 0.02


def test_sweep_composition():
    cases = inputs.sweep_cases(3, 64)
    assert len(cases) == 64 and cases == inputs.sweep_cases(3, 64)
    shapes = [(c["M"], c["N"], c["K"]) for c in cases]
    assert tuple(shapes[:16]) == inputs.FORCED_SWEEP_SHAPES
    dims = {d for s in shapes for d in s}
    assert {1, 17, 1000, 4097} <= dims
    for c in cases[16:]:
        assert all(1 <= c[d] <= 4096 for d in "MNK")
    for c in cases:
        assert c["lda"] >= c["K"] and c["ldb"] >= c["N"] and c["ldc"] >= c["N"]
        if c["index"] % 2 == 0:
            assert (c["lda"], c["ldb"], c["ldc"]) == (c["K"], c["N"], c["N"])
        else:
            assert c["lda"] - c["K"] in (1, 3, 8, 37)
    assert [c["offset"] for c in cases[16:24]] == [1] * 8 and sum(c["offset"] for c in cases) == 8
    small = sum(1 for s in shapes[16:] if min(s) <= 8)
    assert small >= 10          # log-uniform draws put real weight on tiny extents
