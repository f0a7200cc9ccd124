"""Pins for the oracle's MXFP4 GEMM (4-bit E2M1 elements, one E8M0 scale per 32 consecutive k; CPU only).

The paper's outlook names quantised types; the method (Sec. 4.2, App. C, App. D.1, Theorem 1) is unchanged, and a
product of two scaled 4-bit floats is exact in fp32."""
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import tbik_oracle as orc
from paper_2511_17826_amd import synthetic as syn


def test_all_16_element_patterns_and_all_scales():
    """E2M1 from its definition in integers: sign | e (2 bits, bias 1) | f (1 bit); e = 0 is subnormal.  The magnitudes
    are the format's published list 0, 0.5, 1, 1.5, 2, 3, 4, 6."""
    got = orc.fp4_to_f32(np.arange(16, dtype=np.uint8))
    for b in range(16):
        s, e, f = b >> 3, (b >> 1) & 3, b & 1
        mag = Fraction(f, 2) if e == 0 else Fraction(2 + f, 2) * Fraction(2) ** (e - 1)
        assert Fraction(float(got[b])) == (-mag if s else mag), b
        assert np.signbit(got[b]) == bool(s)
    assert got[:8].tolist() == [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]
    assert np.array_equal(orc.fp4_to_f32(np.arange(16, 32, dtype=np.uint8)), got)          # only the low nibble counts
    sc = orc.e8m0_to_f32(np.arange(256, dtype=np.uint8))
    lib = torch.arange(256, dtype=torch.uint8).view(torch.float8_e8m0fnu).to(torch.float32).numpy()   # a library's decoding
    assert np.isnan(sc[255]) and np.isnan(lib[255])
    assert np.array_equal(sc[:255], lib[:255])
    assert sc[127] == 1.0 and sc[0] == 2.0 ** -127 and sc[254] == 2.0 ** 127


def test_packing_low_nibble_first_and_block_scales():
    packed = np.array([[0x21, 0xF7] + [0] * 14 + [0x02] + [0] * 15], dtype=np.uint8)      # k0 = 0.5, k1 = 1, k2 = 6, k3 = -6; k32 = 1
    scales = np.array([[128, 126]], dtype=np.uint8)                                       # block 0: x2, block 1: x0.5
    v = orc.mxfp4_dequant(packed, scales)
    assert v[0, :4].tolist() == [1.0, 2.0, 12.0, -12.0] and v[0, 32] == 0.5 and np.count_nonzero(v) == 5


def test_gemm_against_integers_and_the_fp32_oracle_on_dequantised_operands():
    """Every element times its scale is a small dyadic number, so fp64 holds all partial sums of a superleaf exactly when
    the scales are equal; with spread scales the result must still equal the separately pinned fp32-operand oracle on
    the dequantised matrices (exact products make the fused chain and the add chain coincide).  M != N catches a
    transposed operand."""
    Xp, Xs, Wp, Ws = syn.gemm_random_mxfp4(3, 5, 512, 7)
    Xs[:] = 128
    Ws[:] = 128                                                                           # elements x 2: integers
    y, ybf = orc.gemm_mxfp4(Xp, Xs, Wp, Ws, 128, 1)
    X, Wt = orc.mxfp4_dequant(Xp, Xs), orc.mxfp4_dequant(Wp, Ws)
    assert np.array_equal(y.astype(np.int64), X.astype(np.int64) @ Wt.astype(np.int64).T)
    assert np.array_equal(ybf, syn.f32_to_bf16_bits(y))
    Xp, Xs, Wp, Ws = syn.gemm_random_mxfp4(4, 6, 1536, 9, scale_spread=3)
    y, _ = orc.gemm_mxfp4(Xp, Xs, Wp, Ws, 256, 3)
    X, Wt = orc.mxfp4_dequant(Xp, Xs), orc.mxfp4_dequant(Wp, Ws)
    want = orc.gemm_f32(X, np.ascontiguousarray(Wt.T), 256, 3)
    assert np.array_equal(y.view(np.uint32), want.view(np.uint32))


def test_theorem_1_and_quantisation_recipe():
    Xp, Xs, Wp, Ws = syn.gemm_random_mxfp4(5, 4, 2048, 6, scale_spread=2)
    whole, _ = orc.gemm_mxfp4(Xp, Xs, Wp, Ws, 128, 2)
    for P in (2, 4, 8):
        y, _, parts = orc.gemm_mxfp4(Xp, Xs, Wp, Ws, 128, 2, evaluator=orc.EVAL_SHARDED, P=P, want_partials=True)
        assert np.array_equal(y.view(np.uint32), whole.view(np.uint32)), P
        k = 2048 // P
        own, _ = orc.gemm_mxfp4(Xp[:, :k // 2], Xs[:, :k // 32], Wp[:, :k // 2], Ws[:, :k // 32], 128, 2)
        assert np.array_equal(parts[0].view(np.uint32), own.view(np.uint32))
    # the input recipe rounds to the nearest representable value of the block's scale
    a = np.random.default_rng(1).standard_normal((3, 64)).astype(np.float32)
    p, s = syn.mxfp4_quantize(a)
    back = orc.mxfp4_dequant(p, s)
    step = np.repeat(orc.e8m0_to_f32(s), 32, axis=1)
    assert np.all(np.abs(back - a) <= step) and np.all(np.abs(back) <= 6 * step)
    with pytest.raises(ValueError):
        orc.gemm_mxfp4(Xp[:, :48], Xs[:, :3], Wp[:, :48], Ws[:, :3], 32, 1)                # three superleaves
