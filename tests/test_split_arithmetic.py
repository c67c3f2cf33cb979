"""The arithmetic of the split contraction (csrc/circ_gemm_split.h), checked on the CPU with numpy.

The kernel writes every fp32 operand as the sum of three bfloat16 terms and takes six of the nine
partial products.  This file does not run the kernel (the GPU parity tests do); it pins the two claims
the kernel's error statement rests on, with bfloat16 rounding written out on the bit patterns:
the three terms reproduce an fp32 value to within 2^-24 of its magnitude (|x - h| <= 2^-8 |x|,
|x - h - m| <= 2^-16 |x|, |x - h - m - l| <= 2^-24 |x|), and the six products reproduce the product of
two fp32 values to within 2^-22 of its magnitude in the worst case (2^-23 from the two residuals,
2^-23 from the three products left out), 2^-24.5 over the random pairs here - one rounding of an fp32
product is 2^-24.
"""
import numpy as np


def bf16_round(x):
    """round-to-nearest-even of float32 values to bfloat16, returned as float32"""
    u = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32)


def split3(x):
    x = np.asarray(x, dtype=np.float32)
    h = bf16_round(x)
    r1 = x - h                      # exact in fp32: h shares the leading bits of x
    m = bf16_round(r1)
    r2 = r1 - m                     # exact as well
    l = bf16_round(r2)
    return h, m, l, r1, r2


def samples(n, seed):
    rng = np.random.default_rng(seed)
    mant = rng.uniform(1.0, 2.0, n) * rng.choice([-1.0, 1.0], n)
    expo = rng.integers(-30, 30, n)          # products and their lowest terms stay far from the ends of the fp32 range
    return (mant * np.exp2(expo)).astype(np.float32)


def test_three_terms_carry_24_bits():
    x = samples(200_000, 1)
    h, m, l, r1, r2 = split3(x)
    # the differences the kernel takes in fp32 are exact
    assert np.array_equal(r1.astype(np.float64), x.astype(np.float64) - h.astype(np.float64))
    assert np.array_equal(r2.astype(np.float64), r1.astype(np.float64) - m.astype(np.float64))
    rest = x.astype(np.float64) - (h.astype(np.float64) + m.astype(np.float64) + l.astype(np.float64))
    assert np.max(np.abs(rest) / np.abs(x.astype(np.float64))) <= 2.0 ** -24
    # every term is a bfloat16 value: the low 16 bits of its pattern are zero
    for t in (h, m, l):
        assert not np.any(t.view(np.uint32) & 0xFFFF)


def test_six_partial_products_match_an_fp32_product():
    a, b = samples(200_000, 2), samples(200_000, 3)
    ah, am, al, _, _ = split3(a)
    bh, bm, bl, _, _ = split3(b)
    f = lambda t: t.astype(np.float64)
    # products of two 8-bit significands are exact in fp32, so float64 sums them without error
    six = f(am) * f(bm) + f(al) * f(bh) + f(ah) * f(bl) + f(am) * f(bh) + f(ah) * f(bm) + f(ah) * f(bh)
    for x, y in ((am, bm), (al, bh), (ah, bl), (am, bh), (ah, bm), (ah, bh)):
        p32 = x * y                                  # float32 product
        assert np.array_equal(p32.astype(np.float64), f(x) * f(y))
    exact = f(a) * f(b)
    err = np.max(np.abs(six - exact) / np.abs(exact))
    print(f"six products: max relative error {err:.3e} (2^-24 = {2.0 ** -24:.3e})")
    assert err <= 2.0 ** -22
    # the three products left out: at most 2^-23 of the product
    left = f(am) * f(bl) + f(al) * f(bm) + f(al) * f(bl)
    assert np.max(np.abs(left) / np.abs(exact)) <= 2.0 ** -23


def test_a_dropped_product_is_caught():
    """The bound is tight enough to notice a missing term: without (m, m) the error is ~2^-16."""
    a, b = samples(50_000, 4), samples(50_000, 5)
    ah, am, al, _, _ = split3(a)
    bh, bm, bl, _, _ = split3(b)
    f = lambda t: t.astype(np.float64)
    five = f(al) * f(bh) + f(ah) * f(bl) + f(am) * f(bh) + f(ah) * f(bm) + f(ah) * f(bh)
    exact = f(a) * f(b)
    assert np.max(np.abs(five - exact) / np.abs(exact)) > 2.0 ** -20
