"""Pins for the oracle's 8-bit floating-point GEMM (CPU only).

The paper's outlook names quantised types as the next step; the method itself (Sec. 4.2, App. C, App. D.1, Theorem 1)
does not change: only the widening of an operand does, and a product of two 8-bit floats is still exact in fp32.
"""
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import tbik_oracle as orc
from paper_2511_17826_amd import synthetic as syn

SPEC = {"e4m3": (4, 3, 7), "e5m2": (5, 2, 15)}          # exponent bits, fraction bits, bias


def value_by_integers(b, fmt):
    """The pattern's value as an exact fraction, from the format's definition; None for NaN, +-inf as floats."""
    ebits, fbits, bias = SPEC[fmt]
    s, e, f = b >> 7, (b >> fbits) & ((1 << ebits) - 1), b & ((1 << fbits) - 1)
    if fmt == "e5m2" and e == 31:
        return None if f else (float("-inf") if s else float("inf"))
    if fmt == "e4m3" and e == 15 and f == 7:
        return None
    mant = f if e == 0 else f + (1 << fbits)
    v = Fraction(mant) * Fraction(2) ** (max(e, 1) - bias - fbits)
    return -v if s else v


@pytest.mark.parametrize("fmt", ["e4m3", "e5m2"])
def test_all_256_patterns_against_integer_arithmetic_and_a_library(fmt):
    got = orc.fp8_to_f32(np.arange(256, dtype=np.uint8), fmt)
    lib = syn.fp8_bits_to_f32(np.arange(256, dtype=np.uint8), fmt)          # torch's conversion
    for b in range(256):
        want = value_by_integers(b, fmt)
        if want is None:
            assert np.isnan(got[b]) and np.isnan(lib[b]), b
        elif isinstance(want, float):
            assert got[b] == want and lib[b] == want, b
        else:
            assert Fraction(float(got[b])) == want, (b, got[b], want)
            assert got[b] == lib[b], b
            assert np.signbit(got[b]) == bool(b >> 7), b                    # -0 keeps its sign


def test_hand_values():
    e4 = lambda b: float(orc.fp8_to_f32(np.uint8(b), "e4m3"))
    e5 = lambda b: float(orc.fp8_to_f32(np.uint8(b), "e5m2"))
    assert e4(0x38) == 1.0 and e4(0x7E) == 448.0 and e4(0x01) == 2.0 ** -9 and e4(0x08) == 2.0 ** -6 and e4(0xC0) == -2.0
    assert e5(0x3C) == 1.0 and e5(0x7B) == 57344.0 and e5(0x01) == 2.0 ** -16 and e5(0x04) == 2.0 ** -14 and e5(0xC0) == -2.0


@pytest.mark.parametrize("fmt", ["e4m3", "e5m2"])
def test_small_integers_are_exact_and_operands_are_not_transposed(fmt):
    """|x|, |w| <= 8 are numbers of both formats; every order gives the exact integer.  M != N != K catches a swapped
    index or a transposed operand."""
    Xb, Wb = syn.gemm_small_integers(5, 9, 512, 13, mag=8, fmt=fmt)
    y, ybf = orc.gemm_fp8(Xb, Wb, 128, 1, fmt=fmt)
    want = syn.from_storage(Xb, fmt).astype(np.int64) @ syn.from_storage(Wb, fmt).astype(np.int64)
    assert np.array_equal(y.astype(np.int64), want) and np.all(y == np.round(y))
    assert np.array_equal(syn.bf16_bits_to_f32(ybf), syn.bf16_bits_to_f32(syn.f32_to_bf16_bits(y)))


@pytest.mark.parametrize("fmt", ["e4m3", "e5m2"])
def test_theorem_1_and_the_three_evaluators(fmt):
    Xb, Wb = syn.gemm_random_fp8(7, 6, 2048, 10, fmt)
    whole, _ = orc.gemm_fp8(Xb, Wb, 128, 2, fmt=fmt)                        # 8 superleaves of 256
    counter, _ = orc.gemm_fp8(Xb, Wb, 128, 2, evaluator=orc.EVAL_COUNTER, fmt=fmt)
    assert np.array_equal(whole.view(np.uint32), counter.view(np.uint32))
    for P in (1, 2, 4, 8):
        y, _, parts = orc.gemm_fp8(Xb, Wb, 128, 2, evaluator=orc.EVAL_SHARDED, P=P, want_partials=True, fmt=fmt)
        assert np.array_equal(y.view(np.uint32), whole.view(np.uint32)), P
        # a shard's partial is the whole-K result of the shard on its own
        k = 2048 // P
        for p in (0, P - 1):
            own, _ = orc.gemm_fp8(Xb[:, p * k:(p + 1) * k], Wb[p * k:(p + 1) * k], 128, 2, fmt=fmt)
            assert np.array_equal(parts[p].view(np.uint32), own.view(np.uint32)), (P, p)


@pytest.mark.parametrize("fmt", ["e4m3", "e5m2"])
def test_equals_the_fp32_oracle_on_the_widened_operands(fmt):
    """Products of 8-bit floats are exact in fp32, so the chain "rounded sum of exact products" is the fused
    multiply-add chain of the fp32-operand oracle, a separately written and separately pinned function."""
    Xb, Wb = syn.gemm_random_fp8(8, 5, 1536, 7, fmt)
    y8, _ = orc.gemm_fp8(Xb, Wb, 256, 3, fmt=fmt)
    y32 = orc.gemm_f32(orc.fp8_to_f32(Xb, fmt), orc.fp8_to_f32(Wb, fmt), 256, 3)
    assert np.array_equal(y8.view(np.uint32), y32.view(np.uint32))


def test_one_superleaf_is_the_sequential_sum_and_fp64_bound():
    Xb, Wb = syn.gemm_random_fp8(9, 4, 512, 6, "e4m3")
    X, W = orc.fp8_to_f32(Xb), orc.fp8_to_f32(Wb)
    y, _ = orc.gemm_fp8(Xb, Wb, 512, 1)
    for m in range(4):
        for n in range(6):
            acc = np.float32(0)
            for k in range(512):
                acc = np.float32(acc + np.float32(X[m, k] * W[k, n]))
            assert y[m, n] == acc
    y8, _ = orc.gemm_fp8(Xb, Wb, 64, 1)                                     # 8 superleaves
    X64, W64 = X.astype(np.float64), W.astype(np.float64)
    A = np.abs(X64) @ np.abs(W64)
    assert np.all(np.abs(y8.astype(np.float64) - X64 @ W64) <= (64 + 3) * 2.0 ** -24 * A)


def test_tree_roundings_on_leaf_sparse_operands():
    """One non-zero product per superleaf: the superleaf sums are single exact products and the result is T of them,
    which the separately pinned tree operator gives."""
    Xb, Wb = syn.gemm_leaf_sparse(3, 5, 1024, 7, 128, exp_spread=3, fmt="e4m3")
    y, _ = orc.gemm_fp8(Xb, Wb, 128, 1)
    X, W = orc.fp8_to_f32(Xb), orc.fp8_to_f32(Wb)
    for m in range(5):
        for n in range(7):
            s = [np.float32(np.sum(X[m, j * 128:(j + 1) * 128].astype(np.float64) * W[j * 128:(j + 1) * 128, n])) for j in range(8)]
            assert y[m, n] == orc.T(s), (m, n)


def test_illegal_tree_parameters_are_refused():
    Xb, Wb = syn.gemm_random_fp8(1, 2, 384, 2, "e4m3")
    with pytest.raises(ValueError):
        orc.gemm_fp8(Xb, Wb, 128, 1)                                        # 3 superleaves
