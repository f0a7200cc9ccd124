"""Pins for the oracle's MXFP6 GEMM (6-bit E2M3 / E3M2 elements, 32 of them in 24 bytes, one E8M0 scale per block; CPU
only).

The paper's outlook names quantised types; the method (Sec. 4.2, App. C, App. D.1, Theorem 1) is unchanged, and a
product of two scaled 6-bit floats is exact in fp32."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import tbik_oracle as orc
from paper_2511_17826_amd import synthetic as syn

FMTS = ["e2m3", "e3m2"]


@pytest.mark.parametrize("fmt", FMTS)
def test_all_64_element_patterns(fmt):
    """The decoding from its definition in integers: sign | exponent | fraction, exponent 0 subnormal, no special
    values.  The largest magnitudes are the formats' published ones, 7.5 and 28; the smallest 0.125 and 0.0625."""
    ebits, fbits, bias = (2, 3, 1) if fmt == "e2m3" else (3, 2, 3)
    got = orc.fp6_to_f32(np.arange(64, dtype=np.uint8), fmt)
    for b in range(64):
        s, e, f = b >> 5, (b >> fbits) & ((1 << ebits) - 1), b & ((1 << fbits) - 1)
        mag = Fraction(f, 1 << fbits) * Fraction(2) ** (1 - bias) if e == 0 else Fraction(f + (1 << fbits), 1 << fbits) * Fraction(2) ** (e - bias)
        assert Fraction(float(got[b])) == (-mag if s else mag), b
        assert np.signbit(got[b]) == bool(s)
    assert float(got[31]) == (7.5 if fmt == "e2m3" else 28.0) and float(got[1]) == (0.125 if fmt == "e2m3" else 0.0625)
    assert np.array_equal(orc.fp6_to_f32(np.arange(64, 128, dtype=np.uint8), fmt), got)        # only the low six bits count
    assert np.array_equal(np.abs(got[:32]), syn.fp6_magnitudes(fmt))


def test_packing_is_one_little_endian_bit_stream():
    """Four elements in three bytes: element k in bits 6k .. 6k+5.  Patterns 1, 2, 3, 63 -> bits 000001 000010 000011
    111111 from the low end: byte 0 = 0x81, byte 1 = 0x30, byte 2 = 0xfc."""
    pat = np.zeros((1, 32), dtype=np.uint8)
    pat[0, :4] = [1, 2, 3, 63]
    packed = syn.fp6_pack(pat)
    assert packed.shape == (1, 24) and packed[0, :3].tolist() == [0x81, 0x30, 0xFC] and not packed[0, 3:].any()
    assert np.array_equal(orc.fp6_unpack(packed), pat)
    v = orc.mxfp6_dequant(packed, np.array([[128]], dtype=np.uint8), "e2m3")
    assert v[0, :4].tolist() == [0.25, 0.5, 0.75, -15.0] and np.count_nonzero(v) == 4


@pytest.mark.parametrize("fmt", FMTS)
def test_block_scales_and_transposed_weight_against_exact_fractions(fmt):
    """Random patterns (E3M2: those of magnitude 0.5 .. 3.5, multiples of 1/8 like all of E2M3) and a different power of
    two, 0.5 .. 2, per row and block: every partial sum is a multiple of 2^-8 below 2^15, so any correct evaluation
    gives the exact value, which rational arithmetic on the separately decoded operands must reproduce.  M != N catches
    a transposed operand, the per-block scales a wrong block index."""
    rng = np.random.default_rng(13)
    M, N, K = 3, 5, 128
    lo, hi = (0, 32) if fmt == "e2m3" else (8, 20)
    Xpat = (rng.integers(lo, hi, size=(M, K)) | (rng.integers(0, 2, size=(M, K)) << 5)).astype(np.uint8)
    Wpat = (rng.integers(lo, hi, size=(N, K)) | (rng.integers(0, 2, size=(N, K)) << 5)).astype(np.uint8)
    Xs = rng.integers(126, 129, size=(M, K // 32)).astype(np.uint8)
    Ws = rng.integers(126, 129, size=(N, K // 32)).astype(np.uint8)
    mags = syn.fp6_magnitudes(fmt)
    def exact(pat, sc):
        return [[Fraction(float(mags[p & 31])) * (-1 if p & 32 else 1) * Fraction(2) ** (int(sc[r, k // 32]) - 127) for k, p in enumerate(row)]
                for r, row in enumerate(pat)]
    xr, wr = exact(Xpat, Xs), exact(Wpat, Ws)
    y, ybf = orc.gemm_mxfp6(syn.fp6_pack(Xpat), Xs, syn.fp6_pack(Wpat), Ws, 32, 1, fmt=fmt)
    for m in range(M):
        for n in range(N):
            assert Fraction(float(y[m, n])) == sum(a * b for a, b in zip(xr[m], wr[n])), (m, n)
    assert np.array_equal(ybf, syn.f32_to_bf16_bits(y))


@pytest.mark.parametrize("fmt", FMTS)
def test_equals_the_fp32_oracle_on_dequantised_operands_theorem_1_and_the_recipe(fmt):
    Xp, Xs, Wp, Ws = syn.gemm_random_mxfp6(9, 4, 1536, 6, fmt=fmt, scale_spread=3)
    y, _ = orc.gemm_mxfp6(Xp, Xs, Wp, Ws, 256, 3, fmt=fmt)
    X, Wt = orc.mxfp6_dequant(Xp, Xs, fmt), orc.mxfp6_dequant(Wp, Ws, fmt)
    want = orc.gemm_f32(X, np.ascontiguousarray(Wt.T), 256, 3)
    assert np.array_equal(y.view(np.uint32), want.view(np.uint32))
    Xp, Xs, Wp, Ws = syn.gemm_random_mxfp6(6, 5, 2048, 4, fmt=fmt, scale_spread=2)
    whole, _ = orc.gemm_mxfp6(Xp, Xs, Wp, Ws, 128, 2, fmt=fmt)
    for P in (2, 4, 8):
        yp, _, parts = orc.gemm_mxfp6(Xp, Xs, Wp, Ws, 128, 2, evaluator=orc.EVAL_SHARDED, P=P, want_partials=True, fmt=fmt)
        assert np.array_equal(yp.view(np.uint32), whole.view(np.uint32)), P
        k = 2048 // P
        own, _ = orc.gemm_mxfp6(Xp[:, :3 * k // 4], Xs[:, :k // 32], Wp[:, :3 * k // 4], Ws[:, :k // 32], 128, 2, fmt=fmt)
        assert np.array_equal(parts[0].view(np.uint32), own.view(np.uint32))
    a = np.random.default_rng(1).standard_normal((3, 64)).astype(np.float32)
    q, s = syn.mxfp6_quantize(a, fmt)
    back = orc.mxfp6_dequant(q, s, fmt)
    step = np.repeat(orc.e8m0_to_f32(s), 32, axis=1)
    top = 7.5 if fmt == "e2m3" else 28.0
    assert np.all(np.abs(back) <= top * step) and np.all(np.abs(back - a) <= (0.25 if fmt == "e2m3" else 2.0) * step)
    with pytest.raises(ValueError):
        orc.gemm_mxfp6(Xp[:, :72], Xs[:, :3], Wp[:, :72], Ws[:, :3], 32, 1, fmt=fmt)           # three superleaves
