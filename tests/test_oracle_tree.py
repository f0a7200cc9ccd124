"""Pins for the oracle's tree operator, Alg. 1's counter loop and Alg. 2 (CPU only).

Each test checks the oracle against something fixed by the paper or by arithmetic:
hand-derived values (tests/golden/tree_pins.txt), the textbook level-by-level
pairwise sum, exact integer arithmetic, Theorem 1, and planted mistakes that the
pins must catch.
"""
import numpy as np
import pytest

from conftest import read_tree_pins
from oracle import tbik_oracle as orc

PINS = read_tree_pins()


def bits(x) -> int:
    return int(np.float32(x).view(np.uint32))


@pytest.mark.parametrize("name,leaves,t_bits,seq_bits", PINS, ids=[p[0] for p in PINS])
def test_hand_derived_values(name, leaves, t_bits, seq_bits):
    """App. C operator definition, worked by hand."""
    assert bits(orc.T(leaves)) == t_bits
    assert bits(orc.T_counter(leaves)) == t_bits          # Alg. 1's carry loop reaches the same bits
    assert bits(orc.T_python(leaves)) == t_bits           # independent transcription
    acc = np.float32(0.0)
    for v in leaves:                                       # the pin file's own "left to right" column
        acc = np.float32(acc + v)
    assert bits(acc) == seq_bits


def test_pins_tell_tree_from_other_orders():
    """The pins are sharp: sequential order, a wrong pairing and the exact sum all miss them."""
    four_a = dict((p[0], p) for p in PINS)["four_a"]
    four_b = dict((p[0], p) for p in PINS)["four_b"]
    eight_b = dict((p[0], p) for p in PINS)["eight_b"]
    assert four_a[2] != four_a[3]                           # tree != sequential
    k = four_b[1]
    wrong_pairing = np.float32(np.float32(k[0] + k[2]) + np.float32(k[1] + k[3]))
    assert bits(wrong_pairing) != four_b[2]
    exact = np.float32(sum(float(v) for v in eight_b[1]))  # correctly rounded exact sum
    assert bits(exact) not in (eight_b[2], eight_b[3])


def levelwise_pairwise(v: np.ndarray) -> np.float32:
    """Textbook pairwise summation, bottom-up: add neighbours, halve, repeat (vector fp32 adds)."""
    v = np.asarray(v, dtype=np.float32)
    while v.size > 1:
        v = (v[0::2] + v[1::2]).astype(np.float32)
    return v[0]


@pytest.mark.parametrize("n", [1, 2, 4, 8, 16, 64, 1024, 4096])
def test_T_is_textbook_pairwise_sum(n):
    rng = np.random.default_rng(n)
    for spread in (0, 6, 20):
        v = (rng.standard_normal(n) * np.exp2(rng.integers(-spread, spread + 1, n))).astype(np.float32)
        ref = levelwise_pairwise(v)
        assert bits(orc.T(v)) == bits(ref)
        assert bits(orc.T_counter(v)) == bits(ref)


def test_T_exact_on_integers():
    rng = np.random.default_rng(7)
    v = rng.integers(-1000, 1000, 512).astype(np.float32)
    assert float(orc.T(v)) == float(v.astype(np.int64).sum())
    assert float(orc.T_counter(v)) == float(v.astype(np.int64).sum())


def test_T_within_pairwise_error_bound_of_exact_sum():
    """|T(v) - sum(v)| <= log2(n) * u * sum|v| (+ higher order), u = 2^-24."""
    import math
    rng = np.random.default_rng(11)
    n = 2048
    v = rng.standard_normal(n).astype(np.float32)
    exact = math.fsum(float(x) for x in v)
    bound = 1.01 * math.log2(n) * 2.0 ** -24 * math.fsum(abs(float(x)) for x in v)
    assert abs(float(orc.T(v)) - exact) <= bound


def test_theorem1_on_raw_sequences():
    """T(k_1..k_N) == T(T(L_1)..T(L_C)) for every power-of-two C (Theorem 1)."""
    rng = np.random.default_rng(3)
    for n in (8, 16, 64):
        v = (rng.standard_normal(n) * np.exp2(rng.integers(-10, 11, n))).astype(np.float32)
        whole = bits(orc.T(v))
        C = 1
        while C <= n:
            per = n // C
            parts = [orc.T(v[c * per:(c + 1) * per]) for c in range(C)]
            assert bits(orc.T(parts)) == whole
            C *= 2


@pytest.mark.parametrize("W", [1, 2, 4, 8, 16])
def test_allreduce_is_T_and_every_rank_gets_it(W):
    """Alg. 2: after the broadcast phase all ranks hold T(x_0..x_{W-1}), elementwise."""
    rng = np.random.default_rng(W)
    n = 33
    x = (rng.standard_normal((W, n)) * np.exp2(rng.integers(-8, 9, (W, n)))).astype(np.float32)
    out = orc.allreduce(x)
    want = np.array([orc.T_python(x[:, i]) for i in range(n)], dtype=np.float32)
    for r in range(W):
        assert np.array_equal(out[r].view(np.uint32), want.view(np.uint32))


def test_allreduce_hand_value():
    """Ranks hold [1, 0, 2^-24, 2^-24]: level 0 gives (1+0), (2^-24+2^-24); level 1 gives 1 + 2^-23."""
    x = np.array([[1.0], [0.0], [2.0 ** -24], [2.0 ** -24]], dtype=np.float32)
    out = orc.allreduce(x)
    assert all(bits(out[r, 0]) == 0x3F800001 for r in range(4))
    # a ring / chain order (((x0+x1)+x2)+x3) would give 1.0
    chain = np.float32(np.float32(np.float32(x[0, 0] + x[1, 0]) + x[2, 0]) + x[3, 0])
    assert bits(chain) == 0x3F800000


def test_allreduce_rejects_non_power_of_two():
    from oracle.tbik_oracle import lib
    import ctypes as C
    a = np.zeros((3, 4), dtype=np.float32)
    assert lib().tbik_oracle_allreduce(a.ctypes.data_as(C.POINTER(C.c_float)), 3, 4) != 0


def test_tree_combine_matches_T_and_rounds_once():
    rng = np.random.default_rng(5)
    for P in (1, 2, 4, 8):
        parts = (rng.standard_normal((P, 6, 10)) * np.exp2(rng.integers(-6, 7, (P, 6, 10)))).astype(np.float32)
        y32, ybf = orc.tree_combine(parts)
        want = np.array([[orc.T_python(parts[:, i, j]) for j in range(10)] for i in range(6)], dtype=np.float32)
        assert np.array_equal(y32.view(np.uint32), want.view(np.uint32))
        # bf16 output = one RNE rounding of the fp32 root: nearest bf16, ties to even mantissa
        back = (ybf.astype(np.uint32) << 16).view(np.float32)
        up = ((ybf.astype(np.uint32) + 1) << 16).view(np.float32)
        dn = ((ybf.astype(np.uint32) - 1) << 16).view(np.float32)
        err = np.abs(back.astype(np.float64) - y32)
        assert np.all(err <= np.abs(up.astype(np.float64) - y32))
        assert np.all(err <= np.abs(dn.astype(np.float64) - y32))


def test_bf16_rounding_ties_to_even():
    # 1 + 2^-8 is exactly between bf16 neighbours 1.0 (even mantissa) and 1 + 2^-7 -> 1.0
    assert int(orc.f32_to_bf16_bits(np.float32(1.0 + 2.0 ** -8)).ravel()[0]) == 0x3F80
    # 1 + 3*2^-8 is between 1 + 2^-7 (odd mantissa) and 1 + 2^-6 (even) -> 1 + 2^-6
    assert int(orc.f32_to_bf16_bits(np.float32(1.0 + 3 * 2.0 ** -8)).ravel()[0]) == 0x3F82
    # just above a tie rounds up, just below rounds down
    assert int(orc.f32_to_bf16_bits(np.float32(1.0 + 2.0 ** -8 + 2.0 ** -20)).ravel()[0]) == 0x3F81
    assert int(orc.f32_to_bf16_bits(np.float32(1.0 + 2.0 ** -8 - 2.0 ** -20)).ravel()[0]) == 0x3F80
    assert int(orc.f32_to_bf16_bits(np.float32(-2.5)).ravel()[0]) == 0xC020
