"""The carry-free split products of the inner-product and base-conversion kernels (moduli below 2^50), replayed with
Python integers: a product d * w with d held as two 25-bit halves and w as two 32-bit halves goes into four 64-bit
accumulators that are combined once.  Pins the recombination weights (2^0, 2^32, 2^25, 2^57) and that no accumulator
can pass 2^64 for as many terms as the kernels add (16 digits at most, 8 conversion sources) even at the largest
operands, including the digit words just below 2^51 that a lazy reduction could hand over."""
import numpy as np
import pytest

LOW25 = (1 << 25) - 1
M64 = (1 << 64) - 1


def split_sum(ds, ws):
    t00 = t01 = t10 = t11 = 0
    for d, w in zip(ds, ws):
        d0, d1 = d & LOW25, d >> 25
        w0, w1 = w & 0xFFFFFFFF, w >> 32
        t00 += d0 * w0
        t01 += d0 * w1
        t10 += d1 * w0
        t11 += d1 * w1
        assert max(t00, t01, t10, t11) <= M64, "a 64-bit accumulator would wrap"
    total = t00 + (t01 << 32) + (t10 << 25) + (t11 << 57)
    assert total < 1 << 128
    return total


@pytest.mark.parametrize("terms", [1, 6, 8, 16])
def test_split_products_equal_the_plain_sum(terms):
    rng = np.random.default_rng(terms)
    for _ in range(200):
        ds = [int(v) for v in rng.integers(0, 1 << 50, terms, dtype=np.uint64)]
        ws = [int(v) for v in rng.integers(0, 1 << 63, terms, dtype=np.uint64) * 2 + rng.integers(0, 2, terms, dtype=np.uint64)]
        assert split_sum(ds, ws) == sum(d * w for d, w in zip(ds, ws))


@pytest.mark.parametrize("dmax", [(1 << 50) - 1, (1 << 51) - 1])
def test_largest_operands_do_not_overflow(dmax):
    for terms in (8, 16):
        ds, ws = [dmax] * terms, [M64] * terms
        assert split_sum(ds, ws) == terms * dmax * M64
