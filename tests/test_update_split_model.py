"""The arithmetic the update kernel rests on, checked on the host in numpy: an fp32 element is the
exact sum of three bf16 pieces taken by repeated round-to-nearest-even (x1 = bf16(x),
x2 = bf16(x - x1), x3 = x - x1 - x2), the pieces shrink by 2^-8 each, and the three piece products
the kernel leaves out (a2 b3, a3 b2, a3 b3) are at most 2^-23 |a b| together.  The bf16 rounding
used here is the input generators' (blockgen.to_bf16_bits), not the kernel's code."""
import numpy as np

import blockgen as bg


def bf16(x):
    return bg.bf16_bits_to_f32(bg.to_bf16_bits(np.asarray(x, np.float32)))


def pieces(x):
    x = np.asarray(x, np.float32)
    x1 = bf16(x)
    r = (x - x1).astype(np.float32)          # exact: Sterbenz-type difference of x and its rounding
    x2 = bf16(r)
    x3 = (r - x2).astype(np.float32)
    return x1, x2, x3


def samples():
    rng = np.random.default_rng(5)
    normal = rng.standard_normal(400_000).astype(np.float32)
    wide = (rng.standard_normal(400_000) * np.exp2(rng.integers(-100, 100, 400_000))).astype(np.float32)
    bits = rng.integers(0, 2 ** 32, 400_000, dtype=np.uint64).astype(np.uint32).view(np.float32)
    bits = bits[np.isfinite(bits) & (np.abs(bits) < 3.0e38) & (np.abs(bits) > 1e-30)]
    awkward = np.array([0x3FFFFFFF, 0x3F800001, 0x3F80FFFF, 0x3F7FFFFF, 0x3FFF0001, 0x3F808080, 0x3F808000,
                        0x3F818000, 0x3F807FFF, 0x3F808001, 0x3FAAAAAA, 0x3FD55555, 0x00800000, 0x7F000000],
                       np.uint32).view(np.float32)
    return np.concatenate([normal, wide, bits, awkward, -awkward, np.zeros(1, np.float32)])


def test_three_bf16_pieces_sum_to_the_element_exactly():
    x = samples()
    x1, x2, x3 = pieces(x)
    assert np.array_equal(bf16(x3), x3)                                  # the third piece is a bf16 too
    total = x1.astype(np.float64) + x2.astype(np.float64) + x3.astype(np.float64)
    assert np.array_equal(total, x.astype(np.float64))
    ax = np.abs(x.astype(np.float64))
    assert (np.abs(x2) <= 2.0 ** -8 * ax).all() and (np.abs(x3) <= 2.0 ** -16 * ax).all()


def test_dropped_piece_products_are_below_the_stated_bound():
    x = samples()
    rng = np.random.default_rng(6)
    a, b = x, rng.permutation(x)
    a1, a2, a3 = (p.astype(np.float64) for p in pieces(a))
    b1, b2, b3 = (p.astype(np.float64) for p in pieces(b))
    kept = a1 * b3 + a3 * b1 + a2 * b2 + a1 * b2 + a2 * b1 + a1 * b1
    exact = a.astype(np.float64) * b.astype(np.float64)
    dropped = np.abs(exact - kept)
    assert np.array_equal(exact - kept, a2 * b3 + a3 * b2 + a3 * b3)
    assert (dropped <= 2.0 ** -23 * np.abs(exact)).all()
    nz = exact != 0
    assert (dropped[nz] / np.abs(exact[nz])).mean() < 2.0 ** -28
    # with two pieces per element the error would be far above fp32 rounding: the reason for three
    two = (a1 + a2) * (b1 + b2)
    assert (np.abs(exact - two)[nz] / np.abs(exact[nz])).max() > 2.0 ** -17


def test_an_element_beyond_the_largest_bf16_has_an_infinite_first_piece():
    big = np.array([3.4e38, -3.4e38], np.float32)
    assert np.isinf(bf16(big)).all()          # documented limit of the kernel: such an element gives NaN
    assert np.isfinite(bf16(np.array([3.38e38], np.float32))).all()
