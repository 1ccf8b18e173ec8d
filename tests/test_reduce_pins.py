"""Pins for the reduce-scatter oracle (``oracle/reduce.py``): hand-derived IEEE-754 cases, exact integer
sums, the fp64 sum within the rounding bound, and properties that a wrong order, a dropped block or a
wrong rounding mode would break."""
import numpy as np
import pytest

import ficco_inputs as fi
from oracle import reduce as orr


def bits(x):
    """bf16 bits of values that are exactly representable (checked)."""
    x = np.asarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    assert np.all((u & 0xFFFF) == 0), "test value is not a bf16 number"
    return (u >> 16).astype(np.uint16)


def val(b):
    return (np.asarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def test_single_block_is_returned_unchanged():
    x = fi.make_partials(0, 1, 5, 16)
    assert np.array_equal(orr.rs_reduce([x[0]]), x[0])
    neg_zero = np.full((1, 8), 0x8000, dtype=np.uint16)
    assert np.array_equal(orr.rs_reduce([neg_zero]), neg_zero)          # -0 stays -0: the sum starts from x_0 itself


def test_small_integers_sum_exactly():
    rng = np.random.default_rng(1)
    blocks = [bits(rng.integers(-16, 17, size=(3, 8)).astype(np.float32)) for _ in range(8)]
    want = sum(val(b).astype(np.int64) for b in blocks)                  # |sum| <= 128: a bf16 number (8 significant bits)
    assert np.array_equal(val(orr.rs_reduce(blocks)).astype(np.int64), want)


def test_rounding_is_to_nearest_ties_to_even():
    # fp32 sums exact; bf16 spacing at 1 is 2^-7
    one, h = 1.0, 2.0 ** -8
    assert val(orr.rs_reduce([bits([[one]]), bits([[h]])]))[0, 0] == 1.0                       # 1 + 2^-8: tie, down to even
    assert val(orr.rs_reduce([bits([[one + 2 * h]]), bits([[h]])]))[0, 0] == 1.0 + 4 * h       # 1 + 3*2^-8: tie, up to even
    assert val(orr.rs_reduce([bits([[one]]), bits([[h]]), bits([[h / 2]])]))[0, 0] == 1.0 + 2 * h   # just above the tie: up
    assert val(orr.rs_reduce([bits([[-one]]), bits([[-h]])]))[0, 0] == -1.0


def test_addition_order_is_ascending_gpu_index():
    # 2^24 + 1 is not an fp32 number (tie, rounds to even 2^24), so the order of the additions shows
    big, one = 2.0 ** 24, 1.0
    assert val(orr.rs_reduce([bits([[big]]), bits([[one]]), bits([[-big]])]))[0, 0] == 0.0     # (2^24 + 1) - 2^24
    assert val(orr.rs_reduce([bits([[big]]), bits([[-big]]), bits([[one]])]))[0, 0] == 1.0     # (2^24 - 2^24) + 1
    assert val(orr.rs_reduce([bits([[one]]), bits([[big]]), bits([[-big]])]))[0, 0] == 0.0


def test_every_block_counts_once():
    x = fi.make_partials(2, 6, 4, 8)
    base = val(orr.rs_reduce(list(x))).astype(np.float64)
    for j in range(6):
        y = x.copy()
        y[j] = bits(np.zeros((4, 8), dtype=np.float32))
        without = orr.rs_reduce_f64(list(y))
        # dropping block j changes the result by block j (within the bf16 rounding of the result)
        assert np.allclose(base - without, val(x[j]).astype(np.float64), atol=2.0 ** -8 * (np.abs(base) + 1) + 1e-6)


@pytest.mark.parametrize("G,rows,N,seed", [(2, 3, 8, 0), (8, 16, 64, 1), (5, 7, 24, 2)])
def test_matches_fp64_sum_within_rounding(G, rows, N, seed):
    x = fi.make_partials(seed, G, rows, N)
    got = val(orr.rs_reduce(list(x))).astype(np.float64)
    ref = orr.rs_reduce_f64(list(x))
    # one bf16 rounding (2^-9 relative) plus G-1 fp32 roundings of partial sums
    bound = 2.0 ** -8 * np.abs(ref) + G * 2.0 ** -23 * np.sum(np.abs(val(x).astype(np.float64)), axis=0) + 1e-30
    assert np.all(np.abs(got - ref) <= bound)
    # brute force in exact integer arithmetic on a few elements: x = k * 2^-133 for every bf16 number
    from fractions import Fraction
    for (i, j) in [(0, 0), (rows - 1, N - 1), (rows // 2, N // 3)]:
        exact = sum(Fraction(float(val(x[g, i, j]))) for g in range(G))
        assert abs(Fraction(float(ref[i, j])) - exact) <= Fraction(1, 2 ** 40) * (abs(exact) + 1)


def test_nan_and_infinity_propagate():
    nan, inf = np.uint16(0x7FC0), np.uint16(0x7F80)
    one = bits([[1.0]])
    assert (orr.rs_reduce([one, np.array([[nan]], dtype=np.uint16)])[0, 0] & 0x7FFF) > 0x7F80
    assert orr.rs_reduce([one, np.array([[inf]], dtype=np.uint16)])[0, 0] == inf
    big = bits([[2.0 ** 127]])
    assert orr.rs_reduce([big, big])[0, 0] == inf                                               # fp32 overflow
