"""Pins for the oracle's fp16 (IEEE binary16) operand format (CPU only).

The paper's kernel table lists FP16 beside BF16 with the same block sizes, and the method itself
(Sec. 4.2, App. C, App. D.1) does not depend on the storage format: operands are widened exactly,
products and sums are fp32, the output is rounded once.  What is format-specific is the widening
and the final rounding, pinned here against numpy's float16 (an independent implementation of the
IEEE format), and the GEMM is pinned again with values that only binary16 can hold.
"""
import numpy as np
import pytest

from oracle import tbik_oracle as orc
from paper_2511_17826_amd import synthetic as syn

U = 2.0 ** -24


def u32(a):
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


# ----------------------------------------------------------------------------- the format itself

def test_widening_matches_numpy_on_every_pattern():
    h = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    mine = orc.f16_bits_to_f32(h)
    ref = h.view(np.float16).astype(np.float32)
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(mine), nan)
    assert np.array_equal(u32(mine[~nan]), u32(ref[~nan]))          # includes -0, subnormals, infinities


def _rounding_cases():
    h = np.arange(0x7C00, dtype=np.uint32).astype(np.uint16)        # every finite non-negative half
    v = h.view(np.float16).astype(np.float32)
    mid = (v[:-1].astype(np.float64) + v[1:].astype(np.float64)) / 2   # exact ties between neighbours (fit fp32)
    mid = mid.astype(np.float32)
    cases = [v, mid, np.nextafter(mid, np.float32(0)), np.nextafter(mid, np.float32(np.inf)),
             np.nextafter(v, np.float32(np.inf)), np.nextafter(v[1:], np.float32(0))]
    edge = np.array([65504.0, 65519.996, 65520.0, 65536.0, 1e38, np.inf, 2.0 ** -24, 2.0 ** -25,
                     np.nextafter(np.float32(2.0 ** -25), np.float32(1)), 2.0 ** -26, 1e-45, 0.0,
                     2.0 ** -14, np.nextafter(np.float32(2.0 ** -14), np.float32(0))], dtype=np.float32)
    cases.append(edge)
    rng = np.random.Generator(np.random.PCG64(11))
    bits = rng.integers(0, 2 ** 32, size=40000, dtype=np.uint64).astype(np.uint32)
    rnd = bits.view(np.float32)
    cases.append(rnd[np.isfinite(rnd)])
    cases.append((rng.standard_normal(20000) * np.exp2(rng.integers(-26, 17, size=20000))).astype(np.float32))
    pos = np.concatenate(cases)
    return np.concatenate([pos, -pos])


def test_rounding_matches_numpy_ties_subnormals_overflow():
    x = _rounding_cases()
    with np.errstate(over="ignore"):
        ref = x.astype(np.float16).view(np.uint16)
    mine = orc.f32_to_f16_bits(x)
    bad = np.nonzero(mine != ref)[0]
    assert bad.size == 0, [(float(x[i]), hex(mine[i]), hex(ref[i])) for i in bad[:5]]


def test_rounding_hand_values():
    """1 + 2^-11 is a tie between 1 and 1 + 2^-10: goes to the even one (1).  1 + 3*2^-11 ties up to 1 + 2^-9."""
    def f(v):
        return int(orc.f32_to_f16_bits(v).ravel()[0])

    assert (f(np.float32(1.0))) == 0x3C00
    assert (f(np.float32(1.0 + 2.0 ** -11))) == 0x3C00
    assert (f(np.float32(1.0 + 2.0 ** -11 + 2.0 ** -23))) == 0x3C01
    assert (f(np.float32(1.0 + 3 * 2.0 ** -11))) == 0x3C02
    assert (f(np.float32(-2.0))) == 0xC000
    assert (f(np.float32(65520.0))) == 0x7C00                    # tie at the top rounds to infinity
    assert (f(np.float32(2.0 ** -24))) == 0x0001                 # smallest subnormal
    assert (f(np.float32(2.0 ** -25))) == 0x0000                 # tie with zero: even
    assert (f(np.float32(np.nan))) & 0x7C00 == 0x7C00 and (f(np.float32(np.nan))) & 0x3FF != 0


# ----------------------------------------------------------------------------- the GEMM on fp16 operands

def test_same_bits_mean_different_numbers_in_the_two_formats():
    """0x3C00 is 1.0 as binary16 and 2^-7 as bf16; a product of two of them tells the formats apart."""
    K = 16
    X = np.zeros((1, K), dtype=np.uint16)
    W = np.zeros((K, 1), dtype=np.uint16)
    X[0, 3] = 0x3C00
    W[3, 0] = 0x3C00
    y16, _ = orc.gemm(X, W, 16, 1, fmt="fp16")
    ybf, _ = orc.gemm(X, W, 16, 1, fmt="bf16")
    assert float(y16[0, 0]) == 1.0 and float(ybf[0, 0]) == 2.0 ** -14


def test_products_of_eleven_bit_significands_are_exact():
    """(1 + 2^-10)^2 = 1 + 2^-9 + 2^-20 needs 21 bits: exact in fp32, and only reachable with binary16 operands.
    One such product per superleaf, four superleaves: T = ((p + p) + (p + p)) = 4p exactly."""
    leaf, ns = 32, 4
    K = leaf * ns
    a = np.float32(1.0 + 2.0 ** -10)
    X = np.zeros((2, K), dtype=np.float32)
    W = np.zeros((K, 2), dtype=np.float32)
    for j in range(ns):
        X[:, j * leaf + 7] = a
        W[j * leaf + 7, :] = a
    Xh, Wh = syn.f32_to_f16_bits(X), syn.f32_to_f16_bits(W)
    assert np.array_equal(syn.f16_bits_to_f32(Xh), X)
    for ev, P in [(orc.EVAL_RECURSIVE, 1), (orc.EVAL_COUNTER, 1), (orc.EVAL_SHARDED, 2), (orc.EVAL_SHARDED, 4)]:
        y32, y16 = orc.gemm(Xh, Wh, leaf, 1, ev, P, fmt="fp16")
        assert np.all(y32 == np.float32(4.0 * (1.0 + 2.0 ** -9 + 2.0 ** -20))), (ev, P)
        assert np.all(y16 == 0x4402)                                # 4 * (1 + 2^-9 + 2^-20) -> 4 * (1 + 2*2^-10)
    assert float(orc.gemm_element_alg1(Xh, Wh, 1, 1, leaf, 1, fmt="fp16")) == 4.0 * (1.0 + 2.0 ** -9 + 2.0 ** -20)
    assert float(orc.gemm_element(Xh, Wh, 0, 1, leaf, 1, fmt="fp16")) == 4.0 * (1.0 + 2.0 ** -9 + 2.0 ** -20)


def test_subnormal_operands_are_numbers_not_zeros():
    """2^-24 (smallest binary16 subnormal) times 2^10 is 2^-14 exactly."""
    K = 16
    X = np.zeros((1, K), dtype=np.uint16)
    W = np.zeros((K, 1), dtype=np.uint16)
    X[0, 0] = 0x0001
    W[0, 0] = 0x6400                                                # 1024.0
    y32, y16 = orc.gemm(X, W, 16, 1, fmt="fp16")
    assert float(y32[0, 0]) == 2.0 ** -14 and int(y16[0, 0]) == 0x0400


@pytest.mark.parametrize("leaf,k_first,K", [(16, 1, 256), (64, 3, 768), (32, 5, 1280)])
def test_small_integers_against_int64(leaf, k_first, K):
    X, W = syn.gemm_small_integers(5, 5, K, 33, fmt="fp16")
    exact = syn.f16_bits_to_f32(X).astype(np.int64) @ syn.f16_bits_to_f32(W).astype(np.int64)
    for ev, P in [(orc.EVAL_RECURSIVE, 1), (orc.EVAL_COUNTER, 1), (orc.EVAL_SHARDED, 2)]:
        y32, y16 = orc.gemm(X, W, leaf, k_first, ev, P, fmt="fp16")
        assert np.array_equal(y32.astype(np.int64), exact)
        with np.errstate(over="ignore"):
            assert np.array_equal(y16, exact.astype(np.float32).astype(np.float16).view(np.uint16))


def test_fp64_brute_force_within_the_tree_bound_and_theorem_1():
    M, K, N, leaf = 6, 1024, 40, 64
    X, W = syn.gemm_random(21, M, K, N, fmt="fp16")
    xf, wf = syn.f16_bits_to_f32(X).astype(np.float64), syn.f16_bits_to_f32(W).astype(np.float64)
    exact = xf @ wf
    mag = np.abs(xf) @ np.abs(wf)
    y32, y16 = orc.gemm(X, W, leaf, 1, fmt="fp16")
    depth = leaf + int(np.log2(K // leaf))                           # additions on the longest path
    assert np.all(np.abs(y32 - exact) <= depth * U * mag * 1.01)
    for P in (2, 4, 8, 16):
        ys, y16s, parts = orc.gemm(X, W, leaf, 1, orc.EVAL_SHARDED, P, want_partials=True, fmt="fp16")
        assert np.array_equal(u32(ys), u32(y32)) and np.array_equal(y16s, y16)
        yc, y16c = orc.tree_combine(parts, fmt="fp16")
        assert np.array_equal(u32(yc), u32(y32)) and np.array_equal(y16c, y16)
    with np.errstate(over="ignore"):
        assert np.array_equal(y16, y32.astype(np.float16).view(np.uint16))     # one RNE rounding of the fp32 value
    rows, cols = np.array([0, 3, 5]), np.array([1, 39, 17])
    assert np.array_equal(u32(orc.gemm_elements(X, W, rows, cols, leaf, 1, fmt="fp16")), u32(y32[rows, cols]))


def test_one_superleaf_is_the_sequential_sum():
    M, K, N = 3, 96, 5
    X, W = syn.gemm_random(22, M, K, N, fmt="fp16")
    xf, wf = syn.f16_bits_to_f32(X), syn.f16_bits_to_f32(W)
    y32, _ = orc.gemm(X, W, 32, 3, fmt="fp16")
    for m in range(M):
        for n in range(N):
            acc = np.float32(0)
            for k in range(K):
                acc = np.float32(acc + np.float32(xf[m, k] * wf[k, n]))
            assert u32(acc) == u32(y32[m, n])


# ----------------------------------------------------------------------------- RMSNorm and the fused tail on fp16 rows

def _h(v):
    return np.asarray(v, dtype=np.float16).view(np.uint16)


def test_rmsnorm_fp16_closed_forms():
    """x = 1, w = 1: ss = H exactly, y = fp16(1/sqrt(1 + eps)).  x = 4, eps = 0: (4 * 0.25) * w = w."""
    for H in (4096, 5120, 24):
        x, w = _h(np.ones((3, H))), _h(np.ones(H))
        y = orc.rmsnorm(x, w, 1e-6, fmt="fp16")
        r = np.float32(1.0) / np.sqrt(np.float32(1.0) + np.float32(1e-6), dtype=np.float32)
        assert np.all(y == _h(r))
        assert float(orc.sumsq16(x[0], fmt="fp16")) == float(H)
    H = 1024
    w = _h(np.linspace(0.5, 1.5, H))
    y = orc.rmsnorm(_h(np.full((2, H), 4.0)), w, 0.0, fmt="fp16")
    assert np.array_equal(y[0], w) and np.array_equal(y[1], w)


def test_rmsnorm_fp16_overflow_rounds_to_infinity_and_subnormals_count():
    """One element of 2 in a row of 64, weight 65504: y = (2 * sqrt(64)/2) * 65504 = 8 * 65504 -> +inf in fp16.
    A row of the smallest subnormal: squares are 2^-48 (exact in fp32), so the row normalises to 1."""
    H = 64
    x = np.zeros((1, H), dtype=np.float16)
    x[0, 5] = 2.0
    y = orc.rmsnorm(x.view(np.uint16), _h(np.full(H, 65504.0)), 0.0, fmt="fp16")
    assert y[0, 5] == 0x7C00 and np.all(np.delete(y[0], 5) == 0)
    tiny = np.full((1, H), 0x0001, dtype=np.uint16)
    assert float(orc.sumsq16(tiny[0], fmt="fp16")) == H * 2.0 ** -48
    y = orc.rmsnorm(tiny, _h(np.ones(H)), 0.0, fmt="fp16")
    assert np.all(y == 0x3C00)


@pytest.mark.parametrize("H", [4096, 5120, 100])
def test_rmsnorm_fp16_within_one_ulp_of_fp64(H):
    x, w = syn.rmsnorm_inputs(8, H, fmt="fp16")
    got = orc.rmsnorm(x, w, 1e-6, fmt="fp16").view(np.float16).astype(np.float64)
    X, Wt = x.view(np.float16).astype(np.float64), w.view(np.float16).astype(np.float64)
    ref = X / np.sqrt((X * X).mean(axis=1, keepdims=True) + 1e-6) * Wt
    ulp = np.maximum(np.abs(ref) * 2.0 ** -10, 2.0 ** -24)
    assert np.all(np.abs(got - ref) <= ulp)
    # the same bit patterns read as bf16 are other numbers and give other outputs
    assert not np.array_equal(orc.rmsnorm(x, w, 1e-6, fmt="bf16"), orc.rmsnorm(x, w, 1e-6, fmt="fp16"))


def test_fused_tail_fp16_hand_value_has_two_roundings():
    """T = 1 + 2^-11 + 2^-15 rounds to 1 + 2^-10 in fp16 (above the tie); adding R = 2^-11 gives a tie that goes to
    the even neighbour 1 + 2^-9.  One rounding of the whole sum would have given 1 + 2^-10.  The row of eight equal
    values then normalises to 1 (every fp32 sum of the squares is exact)."""
    H = 8
    parts = np.zeros((2, 1, H), dtype=np.float32)
    parts[0, 0, :] = 1.0
    parts[1, 0, :] = 2.0 ** -11 + 2.0 ** -15
    res = _h(np.full((1, H), 2.0 ** -11))
    hid, out = orc.combine_residual_rmsnorm(parts, res, _h(np.ones(H)), 0.0, fmt="fp16")
    assert np.all(hid == 0x3C02)
    assert np.all(out == 0x3C00)
    assert _h(np.float32(1.0 + 2.0 ** -11 + 2.0 ** -15 + 2.0 ** -11)) == 0x3C01


def test_fused_tail_fp16_is_the_three_steps():
    rng = np.random.Generator(np.random.PCG64(8))
    P, M, H = 4, 6, 200
    parts = rng.standard_normal((P, M, H), dtype=np.float32) * np.float32(0.5)
    res = syn.normal_bf16(rng, (M, H), 1.0, fmt="fp16")
    w = syn.normal_bf16(rng, (H,), 0.1, mean=1.0, fmt="fp16")
    hid, out = orc.combine_residual_rmsnorm(parts, res, w, 1e-6, fmt="fp16")
    y32, y16 = orc.tree_combine(parts, fmt="fp16")
    assert np.array_equal(y16, y32.astype(np.float16).view(np.uint16))
    h = (y16.view(np.float16).astype(np.float32) + res.view(np.float16).astype(np.float32)).astype(np.float16)
    assert np.array_equal(hid, h.view(np.uint16))
    assert np.array_equal(out, orc.rmsnorm(hid, w, 1e-6, fmt="fp16"))


# ----------------------------------------------------------------------------- attention on fp16 tensors

from test_oracle_attention import plain_attention_fp64  # noqa: E402


@pytest.mark.parametrize("causal,std", [(True, 1.0), (False, 1.0), (True, 4.0)])
def test_attention_fp16_plain_definition_within_the_rounding_bound(causal, std):
    """Error sources: p rounded to fp16 (2^-12 relative, or 2^-25 absolute on the subnormal grid), the output rounded
    to fp16 (2^-12 relative).  With std 4 the scores spread over tens of binades, so most weights of a row are
    subnormal or vanish; their absolute roundings sum to at most Lk * 2^-25 * max|v| / l <= 2^-13 here."""
    c = syn.attention_inputs(31, [70, 1, 200, 33], [70, 150, 200, 64], Hq=4, Hkv=2, D=32, std=std, fmt="fp16")
    O, O32 = orc.attention(c["Q"], c["K"], c["V"], c["cu_q"], c["cu_k"], c["scale"], causal, fmt="fp16")
    want, B = plain_attention_fp64(c, causal, fmt="fp16")
    got = O.view(np.float16).astype(np.float64)
    assert np.all(np.abs(O32 - want) <= 2.0 ** -11 * B + 2.0 ** -13)
    assert np.all(np.abs(got - want) <= 2.0 ** -11 * B + 2.0 ** -11 * np.abs(want) + 2.0 ** -13)
    assert np.array_equal(O, O32.astype(np.float16).view(np.uint16))         # one RNE rounding at the end
    if std == 1.0:
        assert np.sqrt(np.mean((O32 - want) ** 2)) <= 2.0 ** -14 * np.sqrt(np.mean(B ** 2))


def test_attention_fp16_weights_below_the_subnormal_grid_vanish():
    """Two keys in one tile, the second scoring about 35 binades lower: its weight 2^-35 is kept by bf16 and is 0 in
    fp16 (below half of 2^-24).  With v_0 = 1 and v_1 = 2^14 the fp16 result is exactly 1; bf16 operands give more."""
    D = 8
    Q = np.zeros((1, 1, D), dtype=np.float32)
    Q[0, 0, 0] = 8.0
    K = np.zeros((2, 1, D), dtype=np.float32)
    K[1, 0, 0] = -3.0                                                # s_1 = -24 * log2(e) = -34.6
    V = np.zeros((2, 1, D), dtype=np.float32)
    V[0], V[1] = 1.0, 2.0 ** 14
    for fmt, exact in (("fp16", True), ("bf16", False)):
        st = lambda a: syn.to_storage(a, fmt)
        O, O32 = orc.attention(st(Q), st(K), st(V), [0, 1], [0, 2], 1.0, False, fmt=fmt)
        assert (O32[0, 0, 0] == 1.0) == exact
        assert O32[0, 0, 0] < 1.0 + 2.0 ** -19
    # a weight of about 2^-17.3 is kept in fp16 too, on the grid of 2^-24: 103.08 * 2^-24 -> 103 * 2^-24
    K[1, 0, 0] = -1.5
    _, O32 = orc.attention(syn.to_storage(Q, "fp16"), syn.to_storage(K, "fp16"), syn.to_storage(V, "fp16"),
                           [0, 1], [0, 2], 1.0, False, fmt="fp16")
    p = np.exp2(np.float64(np.float32(-12.0) * np.float32(1.0 * 1.4426950408889634)))
    p16 = np.round(p * 2.0 ** 24) * 2.0 ** -24
    assert abs(O32[0, 0, 0] - (1.0 + p16 * 2.0 ** 14) / (1.0 + p)) <= 2.0 ** -22
    assert abs(p16 - p) * 2.0 ** 14 > 2.0 ** -16                     # an unrounded weight would miss the bound above


def test_attention_fp16_exact_cases_and_invariance():
    """One visible key returns its value; a decode step, a chunk and the prefill give the same bits."""
    L = 150
    c = syn.attention_inputs(36, [L], [L], Hq=4, Hkv=2, D=16, fmt="fp16")
    O, _ = orc.attention(c["Q"], c["K"], c["V"], c["cu_q"], c["cu_k"], c["scale"], True, fmt="fp16")
    for h in range(4):
        assert np.array_equal(O[0, h], c["V"][0, h // 2])
    for i in (0, 63, 64, 149):
        Od, _ = orc.attention(c["Q"][i:i + 1], c["K"][:i + 1], c["V"][:i + 1], [0, 1], [0, i + 1], c["scale"], True, fmt="fp16")
        assert np.array_equal(Od[0], O[i]), i
    Oc, _ = orc.attention(c["Q"][98:101], c["K"][:101], c["V"][:101], [0, 3], [0, 101], c["scale"], True, fmt="fp16")
    assert np.array_equal(Oc, O[98:101])
    assert not np.array_equal(O, orc.attention(c["Q"], c["K"], c["V"], c["cu_q"], c["cu_k"], c["scale"], True)[0])
