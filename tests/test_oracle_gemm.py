"""Pins of the oracle's prefill product (dequantise to bf16, then a dense product; paper:
kernel table).  Two independent routes to the expected values: exact rational arithmetic
with a bf16 rounding written out here, and the batch-1 W4A16 oracle for scales that make
the bf16 rounding exact."""
from fractions import Fraction

import numpy as np

import oracle


def half_bits(v):
    return np.array([v], np.float16).view(np.uint16)[0]


def bf16_rne_fraction(v):
    """Nearest bf16 (8 significant bits, ties to even) of a rational, as a Fraction."""
    if v == 0:
        return Fraction(0)
    sign = -1 if v < 0 else 1
    a = abs(v)
    e = 0
    while a >= 2:
        a /= 2
        e += 1
    while a < 1:
        a *= 2
        e -= 1
    scaled = a * 128                       # 1.xxxxxxx -> integer part has 8 bits
    lo = scaled.numerator // scaled.denominator
    rest = scaled - lo
    if rest > Fraction(1, 2) or (rest == Fraction(1, 2) and lo % 2 == 1):
        lo += 1
    return sign * Fraction(lo, 128) * Fraction(2) ** e


def test_tiny_product_against_exact_rational_arithmetic():
    rng = np.random.default_rng(5)
    N, K, M = 3, 64, 2
    codes = rng.integers(-8, 8, (N, K))
    sc = np.array([[0.3, 0.0123], [1.7, 0.051], [0.02, 3.3]], np.float16)       # not powers of two
    q = np.zeros((N, K // 2), np.uint8)
    for n in range(N):
        for g in range(K // 32):
            for j in range(16):
                lo, hi = codes[n, 32 * g + j] + 8, codes[n, 32 * g + 16 + j] + 8
                q[n, 16 * g + j] = lo | (hi << 4)
    x = rng.standard_normal((M, K)).astype(np.float32)
    xb = (x.view(np.uint32) >> 16).astype(np.uint16)                             # truncated: any bf16
    y = oracle.gemm_w4a16_dense(q, sc.view(np.uint16), xb)
    for m in range(M):
        for n in range(N):
            acc = Fraction(0)
            for k in range(K):
                w = bf16_rne_fraction(Fraction(int(codes[n, k])) * Fraction(float(sc[n, k // 32])))
                xv = Fraction(float((xb[m, k].astype(np.uint32) << 16).view(np.float32)))
                acc += w * xv
            assert abs(float(acc) - y[m, n]) <= 1e-12 * max(1.0, abs(float(acc)))
    # the rounding matters: with unrounded weights the result differs
    y_exact = oracle.gemv_w4a16(q, sc.view(np.uint16), xb)
    assert np.abs(y - y_exact).max() > 1e-6


def test_power_of_two_scales_reduce_to_the_batch_one_product():
    rng = np.random.default_rng(6)
    N, K, M = 40, 256, 5
    q = rng.integers(0, 256, (N, K // 2)).astype(np.uint8)                        # all codes, -8 too
    sc = (2.0 ** rng.integers(-9, 3, (N, K // 32))).astype(np.float16)
    xb = (rng.standard_normal((M, K)).astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)
    y = oracle.gemm_w4a16_dense(q, sc.view(np.uint16), xb)
    y1 = oracle.gemv_w4a16(q, sc.view(np.uint16), xb)      # code * scale is a bf16 number here
    assert np.allclose(y, y1, rtol=1e-13, atol=1e-13)
