"""Pins for the oracle's MXFP8 GEMM (8-bit E4M3 / E5M2 elements, one E8M0 scale per 32 consecutive k; CPU only).

The paper's outlook names quantised types; the method (Sec. 4.2, App. C, App. D.1, Theorem 1) is unchanged, and a
product of two scaled 8-bit floats is exact in fp32.  The element and scale decodings have exhaustive pins of their
own (the 8-bit and MXFP4 test files); here: the block structure, the transposed weight, the tree."""
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import tbik_oracle as orc
from paper_2511_17826_amd import synthetic as syn


def _exact_rows(bits, scales, fmt):
    """Every element as an exact fraction, from the library's decoding of the pattern and the scale byte as an integer
    power of two (nothing of the oracle's)."""
    t = torch.float8_e4m3fn if fmt == "e4m3" else torch.float8_e5m2
    el = torch.from_numpy(np.ascontiguousarray(bits)).view(t).to(torch.float64).numpy()
    return [[Fraction(float(el[r, k])) * Fraction(2) ** (int(scales[r, k // 32]) - 127) for k in range(bits.shape[1])]
            for r in range(bits.shape[0])]


@pytest.mark.parametrize("fmt", ["e4m3", "e5m2"])
def test_block_scales_and_transposed_weight_against_exact_fractions(fmt):
    """Small integers as elements and a different power of two per block of 32: every partial sum is a short dyadic
    number, so any correct evaluation gives the exact value.  M != N and per-row, per-block scales catch a transposed
    operand and a wrong block index; the reference is rational arithmetic on separately decoded operands."""
    rng = np.random.default_rng(11)
    M, N, K = 3, 5, 128
    Xv = rng.integers(-4, 5, size=(M, K)).astype(np.float32)
    Wv = rng.integers(-4, 5, size=(N, K)).astype(np.float32)
    Xq, Wq = syn.f32_to_fp8_bits(Xv, fmt), syn.f32_to_fp8_bits(Wv, fmt)
    Xs = rng.integers(120, 135, size=(M, K // 32)).astype(np.uint8)
    Ws = rng.integers(120, 135, size=(N, K // 32)).astype(np.uint8)
    y, ybf = orc.gemm_mxfp8(Xq, Xs, Wq, Ws, 32, 1, fmt=fmt)
    xr, wr = _exact_rows(Xq, Xs, fmt), _exact_rows(Wq, Ws, fmt)
    for m in range(M):
        for n in range(N):
            want = sum(a * b for a, b in zip(xr[m], wr[n]))
            assert Fraction(float(y[m, n])) == want, (m, n)
    assert np.array_equal(ybf, syn.f32_to_bf16_bits(y))
    deq = orc.mxfp8_dequant(Xq, Xs, fmt)
    assert all(Fraction(float(deq[m, k])) == xr[m][k] for m in range(M) for k in range(K))


@pytest.mark.parametrize("fmt", ["e4m3", "e5m2"])
def test_equals_the_fp32_oracle_on_dequantised_operands_and_the_unscaled_one_at_scale_one(fmt):
    """Exact products make the fused chain and the add chain coincide, so the separately pinned fp32-operand oracle on
    the dequantised matrices must give the same bits; with every scale 2^0 the separately pinned 8-bit oracle must."""
    Xq, Xs, Wq, Ws = syn.gemm_random_mxfp8(9, 4, 1536, 6, fmt=fmt, scale_spread=3)
    y, _ = orc.gemm_mxfp8(Xq, Xs, Wq, Ws, 256, 3, fmt=fmt)
    X, Wt = orc.mxfp8_dequant(Xq, Xs, fmt), orc.mxfp8_dequant(Wq, Ws, fmt)
    want = orc.gemm_f32(X, np.ascontiguousarray(Wt.T), 256, 3)
    assert np.array_equal(y.view(np.uint32), want.view(np.uint32))
    ones_x, ones_w = np.full_like(Xs, 127), np.full_like(Ws, 127)
    y1, b1 = orc.gemm_mxfp8(Xq, ones_x, Wq, ones_w, 256, 3, fmt=fmt)
    y8, b8 = orc.gemm_fp8(Xq, np.ascontiguousarray(Wq.T), 256, 3, fmt=fmt)
    assert np.array_equal(y1.view(np.uint32), y8.view(np.uint32)) and np.array_equal(b1, b8)
    # a power of two on every scale of X is a power of two on Y (no rounding changes, nothing leaves the range)
    y4, _ = orc.gemm_mxfp8(Xq, (Xs + 2).astype(np.uint8), Wq, Ws, 256, 3, fmt=fmt)
    assert np.array_equal(y4, y * np.float32(4.0))


def test_theorem_1_and_quantisation_recipe():
    Xq, Xs, Wq, Ws = syn.gemm_random_mxfp8(6, 5, 2048, 4, scale_spread=2)
    whole, _ = orc.gemm_mxfp8(Xq, Xs, Wq, Ws, 128, 2)
    for P in (2, 4, 8):
        y, _, parts = orc.gemm_mxfp8(Xq, Xs, Wq, Ws, 128, 2, evaluator=orc.EVAL_SHARDED, P=P, want_partials=True)
        assert np.array_equal(y.view(np.uint32), whole.view(np.uint32)), P
        k = 2048 // P
        own, _ = orc.gemm_mxfp8(Xq[:, :k], Xs[:, :k // 32], Wq[:, :k], Ws[:, :k // 32], 128, 2)
        assert np.array_equal(parts[0].view(np.uint32), own.view(np.uint32))
    for fmt, emax, ulp in (("e4m3", 8, 2.0 ** -4), ("e5m2", 15, 2.0 ** -3)):
        a = np.random.default_rng(1).standard_normal((3, 64)).astype(np.float32)
        q, s = syn.mxfp8_quantize(a, fmt)
        back = orc.mxfp8_dequant(q, s, fmt)
        top = np.repeat(orc.e8m0_to_f32(s), 32, axis=1) * 2.0 ** emax
        assert np.all(np.abs(back - a) <= top * ulp) and np.all(np.abs(back) <= top)
    with pytest.raises(ValueError):
        orc.gemm_mxfp8(Xq[:, :96], Xs[:, :3], Wq[:, :96], Ws[:, :3], 32, 1)                # three superleaves
