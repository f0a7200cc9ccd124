"""Pins for the oracle's GEMM on fp32 operands (CPU only).

The kernel table of the paper lists FP32 beside BF16 and FP16 and says nothing else; the tree (App. C, App. D.1,
Theorem 1) is format-independent.  What needs a reading is a leaf's accumulation, because fp32 products are not exact
in fp32: the oracle takes one fused multiply-add per k in ascending k.  Pinned here against an exact-rational
implementation of that chain, hand values that tell a fused from an unfused product, int64 arithmetic, fp64 within
the tree's error bound, and Theorem 1.
"""
import math
from fractions import Fraction

import numpy as np
import pytest

from oracle import tbik_oracle as orc

U = 2.0 ** -24


def u32(a):
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


def round_to_f32(q: Fraction) -> np.float32:
    """Round-to-nearest-even of an exact rational to binary32 (normal range), in integer arithmetic."""
    if q == 0:
        return np.float32(0.0)
    sign = -1 if q < 0 else 1
    q = abs(q)
    e = q.numerator.bit_length() - q.denominator.bit_length()
    if Fraction(2) ** e > q:
        e -= 1                                           # 2^e <= q < 2^(e+1)
    assert -126 <= e <= 127
    scaled = q / Fraction(2) ** (e - 23)                 # in [2^23, 2^24)
    n, rem = divmod(scaled.numerator, scaled.denominator)
    twice = 2 * rem
    if twice > scaled.denominator or (twice == scaled.denominator and n % 2 == 1):
        n += 1
    return np.float32(sign * math.ldexp(n, e - 23))


def fma_chain(x, w):
    acc = np.float32(0.0)
    for a, b in zip(x, w):
        acc = round_to_f32(Fraction(float(a)) * Fraction(float(b)) + Fraction(float(acc)))
    return acc


def tree(vals):
    vals = list(vals)
    while len(vals) > 1:
        vals = [np.float32(vals[i] + vals[i + 1]) for i in range(0, len(vals), 2)]
    return vals[0]


def test_hand_value_fused_product():
    """x = w = 1 + 2^-12: the product 1 + 2^-11 + 2^-24 is not an fp32 number.  Chained onto -(1 + 2^-11) a fused
    multiply-add leaves 2^-24; a product rounded first (ties to even: 1 + 2^-11) would leave 0."""
    a = np.float32(1 + 2.0 ** -12)
    X = np.array([[-1.0, a] + [0.0] * 14], dtype=np.float32)
    W = np.array([[np.float32(1 + 2.0 ** -11)], [a]] + [[0.0]] * 14, dtype=np.float32)
    y = orc.gemm_f32(X, W, 16, 1)
    assert float(y[0, 0]) == 2.0 ** -24
    assert float(np.float32(np.float32(a * a) - np.float32(1 + 2.0 ** -11))) == 0.0


def test_order_inside_a_leaf_is_ascending_k():
    """(2^24, 1, -2^24, 1) * ones: ascending k gives fma(1, 1, 2^24) = 2^24 (tie to even), then 0, then 1;
    any other order of the four terms gives 0 or 2."""
    X = np.array([[2.0 ** 24, 1.0, -2.0 ** 24, 1.0] + [0.0] * 12], dtype=np.float32)
    W = np.ones((16, 1), dtype=np.float32)
    assert float(orc.gemm_f32(X, W, 16, 1)[0, 0]) == 1.0


@pytest.mark.parametrize("leaf,k_first,K", [(16, 1, 128), (32, 3, 384), (16, 5, 640)])
def test_against_exact_rational_fma_chains(leaf, k_first, K):
    rng = np.random.Generator(np.random.PCG64(K))
    M, N = 3, 4
    X = (rng.standard_normal((M, K)) * np.exp2(rng.integers(-6, 7, (M, K)))).astype(np.float32)
    W = (rng.standard_normal((K, N)) * np.exp2(rng.integers(-6, 7, (K, N)))).astype(np.float32)
    y = orc.gemm_f32(X, W, leaf, k_first)
    sl = leaf * k_first
    for m in range(M):
        for n in range(N):
            s = [fma_chain(X[m, j * sl:(j + 1) * sl], W[j * sl:(j + 1) * sl, n]) for j in range(K // sl)]
            assert u32(tree(s)) == u32(y[m, n]), (m, n)
            assert u32(orc.gemm_f32_element(X, W, m, n, leaf, k_first)) == u32(y[m, n])


def test_small_integers_against_int64():
    rng = np.random.Generator(np.random.PCG64(5))
    M, K, N = 7, 768, 9
    X = rng.integers(-64, 65, (M, K)).astype(np.float32)
    W = rng.integers(-64, 65, (K, N)).astype(np.float32)
    want = (X.astype(np.int64) @ W.astype(np.int64)).astype(np.float32)
    for P in (1, 2, 4):
        assert np.array_equal(orc.gemm_f32(X, W, 64, 3, orc.EVAL_SHARDED, P), want)


def test_fp64_within_the_tree_bound_and_theorem_1():
    rng = np.random.Generator(np.random.PCG64(6))
    M, K, N = 5, 2048, 6
    X = rng.standard_normal((M, K)).astype(np.float32)
    W = (rng.standard_normal((K, N)) * 0.02).astype(np.float32)
    leaf, g = 128, 1
    y = orc.gemm_f32(X, W, leaf, g)
    exact = X.astype(np.float64) @ W.astype(np.float64)
    A = np.abs(X).astype(np.float64) @ np.abs(W).astype(np.float64)
    depth = leaf * g + int(math.log2(K // (leaf * g)))
    assert np.all(np.abs(y - exact) <= depth * U * A * 1.01)
    for ev in (orc.EVAL_COUNTER,):
        assert np.array_equal(u32(orc.gemm_f32(X, W, leaf, g, ev)), u32(y))
    for P in (2, 4, 8, 16):
        yp, parts = orc.gemm_f32(X, W, leaf, g, orc.EVAL_SHARDED, P, want_partials=True)
        assert np.array_equal(u32(yp), u32(y)), P
        comb, _ = orc.tree_combine(parts)
        assert np.array_equal(u32(comb), u32(y))
    rows, cols = np.array([0, 4, 2]), np.array([5, 0, 3])
    assert np.array_equal(u32(orc.gemm_f32_elements(X, W, rows, cols, leaf, g)), u32(y[rows, cols]))
    # another leaf size is another order of roundings
    assert not np.array_equal(u32(orc.gemm_f32(X, W, 64, 1)), u32(y))


def test_values_representable_in_bf16_give_the_bf16_result():
    """With operands that are bf16 numbers every product is exact and the fused chain equals the 16-bit path."""
    from paper_2511_17826_amd import synthetic as syn
    Xb, Wb = syn.gemm_random(3, 4, 512, 8)
    y16, _ = orc.gemm(Xb, Wb, 64, 1)
    y32 = orc.gemm_f32(syn.bf16_bits_to_f32(Xb), syn.bf16_bits_to_f32(Wb), 64, 1)
    assert np.array_equal(u32(y16), u32(y32))


def test_illegal_trees_are_refused():
    X = np.zeros((1, 96), dtype=np.float32)
    W = np.zeros((96, 1), dtype=np.float32)
    with pytest.raises(ValueError):
        orc.gemm_f32(X, W, 32, 1)                      # 3 superleaves: not a power of two
