"""The integer arithmetic behind the fused kernel's path for groups of 4 and 8 query heads, checked in numpy: a folded
weight, scaled to an integer W with |W| <= 2^22, is split into three signed bytes by (W + 0x8080) ^ 0x8080, the int8
products with the biased symbols (symbol - 128) are exact, and adding 128 * sum(W) restores sum(W * symbol)."""
import numpy as np


def _digits(W):
    u = (W.astype(np.int64) + 0x8080) & 0xFFFFFFFF
    u ^= 0x8080
    return [((u >> (8 * j)) & 0xFF).astype(np.uint8).view(np.int8).astype(np.int64) for j in range(3)]


def test_three_signed_bytes_recombine_to_the_integer():
    rng = np.random.default_rng(7)
    W = np.concatenate([rng.integers(-(1 << 22), (1 << 22) + 1, size=200000),
                        np.array([0, 1, -1, 127, 128, -128, -129, 32767, 32768, -32768, -32769, 1 << 22, -(1 << 22),
                                  (1 << 22) - 1, 0x7F7F, 0x8080, -0x8080, -0x8081])])
    d0, d1, d2 = _digits(W)
    assert np.array_equal(d0 + 256 * d1 + 65536 * d2, W)
    assert d2.min() >= -65 and d2.max() <= 64       # the top digit of |W| <= 2^22 fits a signed byte with room


def test_biased_symbols_and_the_constant_term():
    rng = np.random.default_rng(8)
    for n_sym in (51, 128, 129, 256):
        W = rng.integers(-(1 << 22), 1 << 22, size=(8, 128))
        sym = rng.integers(0, n_sym, size=(128, 64))
        biased = (sym.astype(np.uint8) ^ 0x80).view(np.int8).astype(np.int64)   # what the decode table holds
        assert np.array_equal(biased, sym - 128)
        digit_sums = [d @ biased for d in _digits(W)]                            # exact in int32: |sum| <= 2^21
        assert max(np.abs(s).max() for s in digit_sums) < (1 << 31)
        joined = digit_sums[0] + 256 * digit_sums[1] + 65536 * digit_sums[2]
        assert np.array_equal(joined + 128 * W.sum(axis=1, keepdims=True), W @ sym)


def test_fp32_recombination_keeps_the_weights_precision():
    # the kernel joins the three int32 sums in fp32; against exact arithmetic the relative error stays near 2^-24
    rng = np.random.default_rng(9)
    W = rng.integers(-(1 << 22), 1 << 22, size=(8, 128))
    sym = rng.integers(0, 51, size=(128, 64))
    d = [x @ (sym - 128) for x in _digits(W)]
    f = np.float32
    joined = (f(d[2]) * f(256.0) + f(d[1])) * f(256.0) + f(d[0])
    exact = (W @ (sym - 128)).astype(np.float64)
    assert np.abs(joined.astype(np.float64) - exact).max() <= 2.0 ** -22 * np.abs(exact).max()


def test_rounding_inside_the_fma_and_digits_from_the_bit_pattern():
    """The kernel forms W = rint(a * b) as fma(a, b, 1.5 * 2^23): the sum is rounded at unit spacing, and the bit
    pattern of 1.5 * 2^23 + W is 0x4B400000 + W for every |W| <= 2^22 (also at W = 2^22, where the sum reaches 2^24).
    The signed byte digits then come straight from the bit pattern: (bits + (0x8080 - 0x4B400000)) ^ 0x8080."""
    rng = np.random.default_rng(10)
    W = np.concatenate([rng.integers(-(1 << 22), (1 << 22) + 1, size=200000),
                        np.array([0, 1, -1, (1 << 22), -(1 << 22), (1 << 22) - 1, 1 - (1 << 22), 32768, -32769])])
    magic = np.float32(12582912.0)
    assert magic.view(np.uint32) == 0x4B400000
    sums = (magic.astype(np.float64) + W).astype(np.float32)          # exact: integers below 2^25 at unit spacing
    assert np.array_equal(sums.astype(np.float64), 12582912.0 + W)
    bits = sums.view(np.uint32).astype(np.int64)
    assert np.array_equal(bits - 0x4B400000, W)
    digits = ((bits + (0x8080 - 0x4B400000)) & 0xFFFFFFFF) ^ 0x8080
    ref = ((W + 0x8080) & 0xFFFFFFFF) ^ 0x8080
    assert np.array_equal(digits & 0xFFFFFF, ref & 0xFFFFFF)          # bytes 0..2 are the three digits
    # a product that is not an integer is rounded to nearest, ties to even, by the single rounding of the fma
    a = rng.standard_normal(50000).astype(np.float32)
    b = (rng.standard_normal(50000) * 1e5).astype(np.float32)
    keep = np.abs(a.astype(np.float64) * b.astype(np.float64)) < (1 << 22)
    a, b = a[keep], b[keep]
    exact = a.astype(np.float64) * b.astype(np.float64)               # exact: 24 x 24 bit significands
    # (exact + magic) has at most 24 + 25 significant bits: exact in float64, so one rounding to float32 is the fma's
    fused = (exact + 12582912.0).astype(np.float32)
    assert np.array_equal(fused.view(np.uint32).astype(np.int64) - 0x4B400000, np.rint(exact).astype(np.int64))
