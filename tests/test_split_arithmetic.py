"""The arithmetic claim behind the split products (deferred rank-1024 updates on the bf16 matrix cores), checked on the
CPU with an emulation written from its definition: every float32 value is the exact sum of three bfloat16 pieces, each the
round-to-nearest-even of what the pieces before it leave; a product of two pieces is exact in float32; and the six piece
products with i + j <= 4 miss the exact product by at most 2^-23 of its magnitude (as long as nothing underflows)."""
import numpy as np


def _bf16_rne(x):
    """float32 array -> the nearest bfloat16 values (ties to even), returned as float32."""
    u = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) >> 16 << 16
    return (u & 0xFFFFFFFF).astype(np.uint32).view(np.float32)


def _split3(a):
    a = np.asarray(a, dtype=np.float32)
    p1 = _bf16_rne(a)
    r1 = a - p1                      # float32 subtraction: must be exact
    p2 = _bf16_rne(r1)
    r2 = r1 - p2
    p3 = _bf16_rne(r2)
    return p1, p2, p3, r1, r2


def _samples(rng, count, max_expo=60):
    mant = rng.normal(size=count)
    expo = rng.integers(-max_expo, max_expo, size=count)
    a = (mant * np.exp2(expo)).astype(np.float32)
    special = np.array([0.0, -0.0, 1.0, -1.0, 1.0 + 2.0 ** -23, 1.0 - 2.0 ** -24, 3.0000002, 255.99998, 2.0 ** -100,
                        0.1, -0.3, 16777215.0, 1.9999999, 65504.0, 1.0 + 2.0 ** -8, 1.0 + 2.0 ** -9, 1.0 + 3 * 2.0 ** -9], dtype=np.float32)
    return np.concatenate([a, special])


def test_three_bfloat16_pieces_sum_to_the_float32_value_exactly():
    rng = np.random.default_rng(2210)
    a = _samples(rng, 200000)
    p1, p2, p3, r1, r2 = _split3(a)
    a64 = a.astype(np.float64)
    assert np.array_equal(r1.astype(np.float64), a64 - p1.astype(np.float64))              # the remainders are exact
    assert np.array_equal(r2.astype(np.float64), r1.astype(np.float64) - p2.astype(np.float64))
    assert np.array_equal(p1.astype(np.float64) + p2.astype(np.float64) + p3.astype(np.float64), a64)
    for p in (p1, p2, p3):                                                                 # each piece is a bfloat16
        assert np.all((p.view(np.uint32) & 0xFFFF) == 0)
    nz = a != 0
    assert np.all(np.abs(p2[nz]) <= 2.0 ** -8 * np.abs(a64[nz])) and np.all(np.abs(p3[nz]) <= 2.0 ** -16 * np.abs(a64[nz]))


def test_six_piece_products_miss_the_product_by_at_most_2_to_minus_23():
    rng = np.random.default_rng(17323)
    # magnitudes between 2^-30 and 2^30: no piece product comes near the float32 underflow threshold, where "exact" ends
    a, b = _samples(rng, 100000, 30), _samples(rng, 100000, 30)[::-1].copy()
    A, B = _split3(a)[:3], _split3(b)[:3]
    kept = [(2, 0), (0, 2), (1, 1), (1, 0), (0, 1), (0, 0)]          # a3 b1, a1 b3, a2 b2, a2 b1, a1 b2, a1 b1
    total = np.zeros(a.shape, dtype=np.float64)
    for i, j in kept:
        prod32 = A[i] * B[j]                                          # float32 product of two bfloat16 values
        assert np.array_equal(prod32.astype(np.float64), A[i].astype(np.float64) * B[j].astype(np.float64))   # exact
        total += prod32.astype(np.float64)
    exact = a.astype(np.float64) * b.astype(np.float64)
    assert np.all(np.abs(total - exact) <= 2.0 ** -23 * np.abs(exact))
    # leaving out one of the kept products is visible at this bar (what the GPU tests' Frobenius figure catches)
    without = total - (A[1] * B[1]).astype(np.float64)
    assert np.mean(np.abs(without - exact) > 2.0 ** -23 * np.abs(exact)) > 0.5
