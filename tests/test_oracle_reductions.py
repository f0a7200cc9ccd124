"""Pins for the oracle's tree-ordered row reductions: TreeSum, RMSNorm, sum / max / log-softmax (CPU only).

App. B fixes what "batch invariant" means for these ops (each row reduced on its own,
in one fixed order); the order itself is the tree of App. C over 16-byte leaves.
"""
import math

import numpy as np
import pytest

from oracle import tbik_oracle as orc
from paper_2511_17826_amd import synthetic as syn


def u32(a):
    a = np.asarray(a, dtype=np.float32)
    return a.view(np.uint32) if a.ndim else np.uint32(a.reshape(1).view(np.uint32)[0])


def f32(b):
    return syn.bf16_bits_to_f32(b)


# ----------------------------------------------------------------------------- TreeSum

def test_treesum_hand_values():
    """leaf 2 over [1, 0 | 2^-24, 2^-24 | pad | pad]: leaves [1, 2^-23, 0, 0] -> (1 + 2^-23) + (0+0)."""
    t = 2.0 ** -24
    assert int(u32(orc.treesum([1, 0, t, t], 2))) == 0x3F800001
    # leaf 1: T over [1, 0, t, t] = (1+0) + (t+t) = 1 + 2^-23 ; leaf 4: sequential ((1+0)+t)+t = 1
    assert int(u32(orc.treesum([1, 0, t, t], 1))) == 0x3F800001
    assert int(u32(orc.treesum([1, 0, t, t], 4))) == 0x3F800000
    # ragged: 5 elements, leaf 2 -> leaves [1+0, t+t, t, pad] -> (1 + 2^-23) + (t + 0) = 1 + 3t -> tie -> even
    # 1 + 2^-23 + 2^-24 lies halfway between 1 + 2^-23 (odd mantissa) and 1 + 2^-22 (even) -> 1 + 2^-22
    assert int(u32(orc.treesum([1, 0, t, t, t], 2))) == 0x3F800002
    assert float(orc.treesum([], 4)) == 0.0


@pytest.mark.parametrize("n,leaf", [(1, 4), (7, 4), (64, 4), (1000, 8), (4096, 8), (5120, 8), (151936, 4)])
def test_treesum_equals_leafwise_cumsum_then_textbook_pairwise(n, leaf):
    rng = np.random.default_rng(n)
    v = (rng.standard_normal(n) * np.exp2(rng.integers(-6, 7, n))).astype(np.float32)
    nl = -(-n // leaf)
    n2 = 1 << max(0, (nl - 1).bit_length())
    pad = np.zeros(n2 * leaf, dtype=np.float32)
    pad[:n] = v
    leaves = np.cumsum(pad.reshape(n2, leaf), axis=1, dtype=np.float32)[:, -1]   # in-order fp32 adds
    while leaves.size > 1:
        leaves = (leaves[0::2] + leaves[1::2]).astype(np.float32)
    assert int(u32(orc.treesum(v, leaf))) == int(u32(leaves[0]))


def test_treesum_exact_on_integers_and_bounded_vs_fsum():
    rng = np.random.default_rng(2)
    v = rng.integers(-100, 100, 5000).astype(np.float32)
    assert float(orc.treesum(v, 4)) == float(v.astype(np.int64).sum())
    w = rng.standard_normal(151936).astype(np.float32)
    h = 3 + 16                                       # 3 in-leaf adds + tree of 2^16 padded leaves
    bound = h * 2.0 ** -24 * math.fsum(abs(float(x)) for x in w) * 1.01
    assert abs(float(orc.treesum(w, 4)) - math.fsum(float(x) for x in w)) <= bound


def test_treesum_sibling_swap_invariant_but_not_arbitrary_moves():
    """fp32 add commutes: swapping two sibling subtrees keeps the bits; a rotation by one element generally does not."""
    rng = np.random.default_rng(4)
    v = (rng.standard_normal(4096) * np.exp2(rng.integers(-8, 9, 4096))).astype(np.float32)
    base = int(u32(orc.treesum(v, 8)))
    swapped = v.copy()
    swapped[:2048], swapped[2048:] = v[2048:], v[:2048]          # swap the root's children
    assert int(u32(orc.treesum(swapped, 8))) == base
    sw2 = v.copy()
    sw2[0:8], sw2[8:16] = v[8:16], v[0:8]                        # swap two sibling leaves
    assert int(u32(orc.treesum(sw2, 8))) == base
    changed = sum(int(u32(orc.treesum(np.roll(v, s), 8))) != base for s in range(1, 9))
    assert changed >= 1


# ----------------------------------------------------------------------------- RMSNorm

def test_rmsnorm_closed_form_all_ones():
    """x = 1, w = 1: ss = H exactly, ms = 1, y = bf16(1/sqrt(1 + eps))."""
    for H in (4096, 5120, 24):
        x = syn.f32_to_bf16_bits(np.ones((3, H), dtype=np.float32))
        w = syn.f32_to_bf16_bits(np.ones(H, dtype=np.float32))
        y = orc.rmsnorm(x, w, 1e-6)
        r = np.float32(1.0) / np.sqrt(np.float32(1.0) + np.float32(1e-6), dtype=np.float32)
        assert np.all(y == syn.f32_to_bf16_bits(np.array([r]))[0])
        assert float(orc.sumsq_bf16(x[0])) == float(H)


def test_rmsnorm_power_of_two_rows_are_exact():
    """x_i = 2^a: squares and every partial sum are powers of two times integers -> exact; r = 2^-a exactly when eps = 0."""
    H = 1024
    x = syn.f32_to_bf16_bits(np.full((2, H), 4.0, dtype=np.float32))
    wv = np.linspace(0.5, 1.5, H).astype(np.float32)
    w = syn.f32_to_bf16_bits(wv)
    y = orc.rmsnorm(x, w, 0.0)
    assert np.array_equal(y[0], w) and np.array_equal(y[1], w)      # (4 * 0.25) * w = w, already bf16


@pytest.mark.parametrize("H", [4096, 5120, 100])
def test_rmsnorm_within_one_bf16_ulp_of_fp64(H):
    x, w = syn.rmsnorm_inputs(8, H)
    y = f32(orc.rmsnorm(x, w, 1e-6)).astype(np.float64)
    X, Wt = f32(x).astype(np.float64), f32(w).astype(np.float64)
    ref = X / np.sqrt((X * X).mean(axis=1, keepdims=True) + 1e-6) * Wt
    ulp = np.maximum(np.abs(ref), 2.0 ** -126) * 2.0 ** -7
    assert np.all(np.abs(y - ref) <= ulp)
    # sum of squares against exact arithmetic within the tree bound
    for r in range(8):
        exact = math.fsum(float(v) * float(v) for v in f32(x[r]))
        h = 7 + math.ceil(math.log2(-(-H // 8)))
        assert abs(float(orc.sumsq_bf16(x[r])) - exact) <= h * 2.0 ** -24 * exact * 1.01


def test_rmsnorm_rows_are_independent_of_batch():
    x, w = syn.rmsnorm_inputs(16, 4096)
    full = orc.rmsnorm(x, w)
    for M in (1, 5):
        assert np.array_equal(orc.rmsnorm(x[:M], w), full[:M])
    perm = np.random.default_rng(1).permutation(16)
    assert np.array_equal(orc.rmsnorm(x[perm], w), full[perm])


# ----------------------------------------------------------------------------- sum / max / log-softmax

def test_row_sum_and_max():
    rng = np.random.default_rng(9)
    x = rng.integers(-50, 50, (5, 1001)).astype(np.float32)
    assert np.array_equal(orc.row_sum(x), x.astype(np.int64).sum(axis=1).astype(np.float32))
    z = syn.logits_f32(3, 5000)
    assert np.array_equal(orc.row_max(z), z.max(axis=1))
    assert all(int(u32(orc.row_sum(z)[r])) == int(u32(orc.treesum(z[r], 4))) for r in range(3))


def test_logsoftmax_constant_row_is_minus_log_V():
    for V in (4, 1024, 151936):
        x = np.full((2, V), 1.25, dtype=np.float32)
        o = orc.row_logsoftmax(x)
        # exp(0) = 1 exactly, the tree sums V ones exactly, so o = 0 - logf(V)
        assert np.all(o == -np.float32(math.log(V))) or np.max(np.abs(o + math.log(V))) <= 1e-6


def test_logsoftmax_against_fp64_and_normalisation():
    x = syn.logits_f32(4, 151936)
    o = orc.row_logsoftmax(x).astype(np.float64)
    X = x.astype(np.float64)
    m = X.max(axis=1, keepdims=True)
    ref = (X - m) - np.log(np.exp(X - m).sum(axis=1, keepdims=True))
    assert np.max(np.abs(o - ref) / np.maximum(1.0, np.abs(ref))) <= 1e-5
    assert np.all(np.abs(np.exp(o).sum(axis=1) - 1.0) <= 1e-5)
    assert np.all(o.max(axis=1) <= 0.0)


def test_logsoftmax_shift_by_representable_constant():
    """Adding 8.0 to integer-valued logits changes neither x - max nor the result (exact subtraction)."""
    rng = np.random.default_rng(12)
    x = rng.integers(-20, 20, (3, 777)).astype(np.float32)
    a = orc.row_logsoftmax(x)
    b = orc.row_logsoftmax((x + np.float32(8.0)).astype(np.float32))
    assert np.array_equal(u32(a), u32(b))


def test_logsoftmax_rows_independent_of_batch():
    x = syn.logits_f32(6, 3001)
    full = orc.row_logsoftmax(x)
    assert np.array_equal(u32(orc.row_logsoftmax(x[2:3])), u32(full[2:3]))
    assert np.array_equal(u32(orc.row_logsoftmax(x[::-1].copy())), u32(full[::-1]))


def test_fused_tail_rounds_the_combined_value_before_the_residual_add():
    """Y = 1 + 2^-8 + 2^-12 rounds to bf16 1 + 2^-7; adding R = 2^-8 gives the tie 1 + 2^-7 + 2^-8, which goes to the
    even neighbour 1 + 2^-6 (0x3F82).  One rounding of Y + R = 1 + 2^-7 + 2^-12 would give 1 + 2^-7 (0x3F81) instead."""
    H = 8
    parts = np.zeros((2, 1, H), dtype=np.float32)
    parts[0, 0, :] = 1.0
    parts[1, 0, :] = 2.0 ** -8 + 2.0 ** -12
    res = np.full((1, H), 0x3B80, dtype=np.uint16)             # bf16 2^-8
    w = np.full((H,), 0x3F80, dtype=np.uint16)                 # bf16 1.0
    hid, out = orc.combine_residual_rmsnorm(parts, res, w, eps=0.0)
    assert np.all(hid == 0x3F82)
    # every element equal: x / sqrt(x^2) = 1 exactly or within one rounding; here ss/H = x^2 exactly, so 1.0
    assert np.all(out == 0x3F80)
    # the pieces are the public ones: same result as calling them one after the other
    _, ybf = orc.tree_combine(parts)
    assert np.all(ybf == 0x3F81)


# ----------------------------------------------------------------------------- gated activation (SiLU * up)

def _silu_mul_f64(gbits, ubits, fmt):
    g = syn.from_storage(gbits, fmt).astype(np.float64)
    u = syn.from_storage(ubits, fmt).astype(np.float64)
    return g / (1.0 + np.exp(-g)) * u


@pytest.mark.parametrize("fmt", ["bf16", "fp16"])
def test_silu_mul_matches_the_fp64_definition_within_one_step(fmt):
    """act = SiLU(gate) * up with SiLU(g) = g * sigmoid(g) (implementation appendix, "other kernels"): every output is
    one of the two 16-bit neighbours of the fp64 value, and all but a few are the nearest one."""
    rng = np.random.default_rng(11)
    g = syn.to_storage(rng.standard_normal((64, 1024), dtype=np.float32) * 3, fmt)
    u = syn.to_storage(rng.standard_normal((64, 1024), dtype=np.float32), fmt)
    got = syn.from_storage(orc.silu_mul(g, u, fmt), fmt).astype(np.float64)
    want = _silu_mul_f64(g, u, fmt)
    nearest = syn.from_storage(syn.to_storage(want.astype(np.float32), fmt), fmt).astype(np.float64)
    step = np.maximum(np.abs(nearest), 2.0 ** -14 if fmt == "fp16" else 2.0 ** -126) * (2.0 ** -10 if fmt == "fp16" else 2.0 ** -7)
    assert np.all(np.abs(got - want) <= step)
    assert np.mean(got != nearest) < 2e-3


def test_silu_mul_exact_cases():
    """Where the definition has an exact value.  g >= 32: e^-g < 2^-46, so 1 + e^-g rounds to 1 and SiLU(g) = g;
    g = 0 gives 0; g <= -104: e^104 overflows fp32, g / inf = -0; SiLU(-g) - SiLU(g) = -g ties the two branches."""
    b = lambda v: syn.f32_to_bf16_bits(np.asarray(v, dtype=np.float32))
    f = syn.bf16_bits_to_f32
    out = f(orc.silu_mul(b([[32, 64, 48, 0, 0, -104, -200]]), b([[3, -0.5, 1.5, 7, -7, 2, -2]])))
    assert out[0, :3].tolist() == [96.0, -32.0, 72.0]
    assert out[0, 3:].tolist() == [0.0] * 4
    # one hand value: g = 1, u = 1: 1 / (1 + e^-1) = 0.7310585786..., which bf16 rounds to 0.73046875 (0x3F3B)
    assert int(orc.silu_mul(b([[1.0]]), b([[1.0]]))[0, 0]) == 0x3F3B
    # the identity SiLU(g) - SiLU(-g) = g, on values where all three are bf16 numbers after rounding within a step
    g = b(np.linspace(0.125, 8, 64, dtype=np.float32)[None, :])
    one = b(np.ones((1, 64), dtype=np.float32))
    pos = f(orc.silu_mul(g, one)).astype(np.float64)
    neg = f(orc.silu_mul(g ^ np.uint16(0x8000), one)).astype(np.float64)
    assert np.all(np.abs((pos - neg) - f(g)) <= np.abs(f(g)) * 2.0 ** -7)


def test_silu_mul_takes_gate_first_and_up_second():
    """A swapped operand pair must fail: SiLU(2) * 0.5 != SiLU(0.5) * 2."""
    b = lambda v: syn.f32_to_bf16_bits(np.asarray(v, dtype=np.float32))
    a = syn.bf16_bits_to_f32(orc.silu_mul(b([[2.0]]), b([[0.5]])))[0, 0]
    assert abs(a - 2.0 / (1.0 + math.exp(-2.0)) * 0.5) < 2.0 ** -8
    assert abs(a - 0.5 / (1.0 + math.exp(-0.5)) * 2.0) > 0.1
