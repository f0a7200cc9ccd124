"""Pins for the oracle's fixed-tile attention (CPU only).

The paper fixes the rule (a fixed tile size, one kernel for prefill and decode; Sec. 2.1: fp32 accumulation); the
streaming-softmax arithmetic is the oracle's stated reading.  It is pinned against what does not depend on that
reading: the plain definition softmax(q K^T * scale) V in fp64 within the rounding bound, cases with an exact
answer (one visible key, a dominant key, uniform weights over small integers), causality, and the invariances the
rule exists for (batch composition, prefill vs decode vs chunks).
"""
import numpy as np
import pytest

from oracle import tbik_oracle as orc
from paper_2511_17826_amd import synthetic as syn


def f32(b):
    return syn.bf16_bits_to_f32(b)


def plain_attention_fp64(c, causal=True, fmt="bf16"):
    """softmax(q K^T * scale) V per sequence and head, fp64, written from the definition.
    Returns (O, B) with B = sum_j p_j |v_j| / sum_j p_j, the magnitude the rounding bound is stated in."""
    Q, K, V = (syn.from_storage(c[n], fmt).astype(np.float64) for n in "QKV")
    Hq, Hkv = c["Hq"], c["Hkv"]
    O = np.zeros(Q.shape)
    B = np.zeros(Q.shape)
    for b in range(len(c["cu_q"]) - 1):
        q0, q1, k0, k1 = c["cu_q"][b], c["cu_q"][b + 1], c["cu_k"][b], c["cu_k"][b + 1]
        Lq, Lk = q1 - q0, k1 - k0
        for h in range(Hq):
            hk = h // (Hq // Hkv)
            S = Q[q0:q1, h] @ K[k0:k1, hk].T * c["scale"]
            if causal:
                i = np.arange(Lq)[:, None]
                j = np.arange(Lk)[None, :]
                S = np.where(j <= i + Lk - Lq, S, -np.inf)
            with np.errstate(invalid="ignore"):
                P = np.exp(S - np.max(S, axis=1, keepdims=True))
            P = np.nan_to_num(P)
            den = np.maximum(P.sum(axis=1, keepdims=True), 1e-300)
            O[q0:q1, h] = (P @ V[k0:k1, hk]) / den
            B[q0:q1, h] = (P @ np.abs(V[k0:k1, hk])) / den
    return O, B


@pytest.mark.parametrize("causal", [True, False])
def test_plain_definition_in_fp64_within_the_rounding_bound(causal):
    """Error sources: p rounded to bf16 (2^-9 relative per term), the output rounded to bf16 (2^-9 relative), fp32
    everywhere else (negligible beside them): |O - O_exact| <= 2^-8 * B + 2^-8 * |O_exact|."""
    c = syn.attention_inputs(31, [70, 1, 200, 33], [70, 150, 200, 64], Hq=4, Hkv=2, D=32)
    O, O32 = orc.attention(c["Q"], c["K"], c["V"], c["cu_q"], c["cu_k"], c["scale"], causal)
    want, B = plain_attention_fp64(c, causal)
    err = np.abs(f32(O).astype(np.float64) - want)
    assert np.all(err <= 2.0 ** -8 * B + 2.0 ** -8 * np.abs(want) + 1e-30)
    assert np.all(np.abs(O32 - want) <= 2.0 ** -8 * B)               # before the output rounding
    assert np.array_equal(O, syn.f32_to_bf16_bits(O32))              # one RNE rounding at the end
    # the typical error is far below the bound: the bf16 roundings of p are independent
    assert np.sqrt(np.mean((O32 - want) ** 2)) <= 2.0 ** -11 * np.sqrt(np.mean(B ** 2))


def test_one_visible_key_returns_its_value_exactly():
    """The first query of a causal prefill sees key 0 only: p = exp2(0) = 1, l = 1, O = v_0 bit for bit."""
    c = syn.attention_inputs(32, [5, 130], [5, 130], Hq=4, Hkv=2, D=16)
    O, _ = orc.attention(c["Q"], c["K"], c["V"], c["cu_q"], c["cu_k"], c["scale"], True)
    for b in range(2):
        q0, k0 = c["cu_q"][b], c["cu_k"][b]
        for h in range(4):
            assert np.array_equal(O[q0, h], c["V"][k0, h // 2])


def test_dominant_key_in_a_later_tile_wins_exactly():
    """Key 100 (second tile of 64) scores 2^10 above the rest: every other weight underflows to 0 in fp32, the
    running output of the first tile is scaled by exp2(-huge) = 0, and O = v_100 exactly."""
    D, Lk = 16, 150
    c = syn.attention_inputs(33, [1], [Lk], Hq=1, Hkv=1, D=D, std=0.25)
    q = np.zeros(D, dtype=np.float32)
    q[0] = 32.0
    K = f32(c["K"]).copy()
    K[:, 0, 0] = 0.0
    K[100, 0, 0] = 64.0                                              # q.k = 2048 for key 100, |q.k| small otherwise
    c["Q"][0, 0] = syn.f32_to_bf16_bits(q)
    c["K"] = syn.f32_to_bf16_bits(K)
    O, O32 = orc.attention(c["Q"], c["K"], c["V"], c["cu_q"], c["cu_k"], 1.0, True)
    assert np.array_equal(O[0, 0], c["V"][100, 0])
    assert np.array_equal(O32[0, 0], f32(c["V"][100, 0]))


@pytest.mark.parametrize("Lk", [64, 128, 256])
def test_uniform_weights_over_small_integers_give_the_exact_mean(Lk):
    """q = 0: every score is 0, every weight exp2(0) = 1, l = Lk (a power of two), o = sum of integers: exact."""
    D = 8
    rng = np.random.Generator(np.random.PCG64(34))
    V = rng.integers(-8, 9, size=(Lk, 1, D)).astype(np.float32)
    K = rng.standard_normal((Lk, 1, D)).astype(np.float32)
    Q = np.zeros((1, 1, D), dtype=np.float32)
    O, O32 = orc.attention(syn.f32_to_bf16_bits(Q), syn.f32_to_bf16_bits(K), syn.f32_to_bf16_bits(V),
                           [0, 1], [0, Lk], 0.5, True)
    want = V.sum(axis=0) / Lk
    assert np.array_equal(O32[0], want.astype(np.float32))
    assert np.array_equal(O[0], syn.f32_to_bf16_bits(want.astype(np.float32)))


def test_future_keys_do_not_matter():
    c = syn.attention_inputs(35, [90], [90], Hq=2, Hkv=1, D=16)
    O, _ = orc.attention(c["Q"], c["K"], c["V"], c["cu_q"], c["cu_k"], c["scale"], True)
    K2, V2 = c["K"].copy(), c["V"].copy()
    K2[50:] = syn.f32_to_bf16_bits(f32(K2[50:]) * -3 + 1)
    V2[50:] = syn.f32_to_bf16_bits(f32(V2[50:]) + 7)
    O2, _ = orc.attention(c["Q"], K2, V2, c["cu_q"], c["cu_k"], c["scale"], True)
    assert np.array_equal(O[:50], O2[:50]) and not np.array_equal(O[50:], O2[50:])
    O3, _ = orc.attention(c["Q"], K2, V2, c["cu_q"], c["cu_k"], c["scale"], False)         # without the mask they do
    assert not np.array_equal(O[:50], O3[:50])


def test_prefill_decode_chunks_and_batch_composition_give_the_same_bits():
    """Query i of a sequence, computed (a) in a prefill of the whole sequence, (b) as a decode step with i+1 keys,
    (c) in a chunk of queries i-2..i, (d) inside a batch with other sequences: one set of bits."""
    L = 150
    c = syn.attention_inputs(36, [L], [L], Hq=4, Hkv=2, D=16)
    O, _ = orc.attention(c["Q"], c["K"], c["V"], c["cu_q"], c["cu_k"], c["scale"], True)
    for i in (0, 63, 64, 100, 149):
        Od, _ = orc.attention(c["Q"][i:i + 1], c["K"][:i + 1], c["V"][:i + 1], [0, 1], [0, i + 1], c["scale"], True)
        assert np.array_equal(Od[0], O[i]), i
    Oc, _ = orc.attention(c["Q"][98:101], c["K"][:101], c["V"][:101], [0, 3], [0, 101], c["scale"], True)
    assert np.array_equal(Oc, O[98:101])
    other = syn.attention_inputs(37, [40, 7], [40, 90], Hq=4, Hkv=2, D=16)
    Qb = np.concatenate([other["Q"][:40], c["Q"], other["Q"][40:]])
    Kb = np.concatenate([other["K"][:40], c["K"], other["K"][40:]])
    Vb = np.concatenate([other["V"][:40], c["V"], other["V"][40:]])
    Ob, _ = orc.attention(Qb, Kb, Vb, [0, 40, 40 + L, 47 + L], [0, 40, 40 + L, 130 + L], c["scale"], True)
    assert np.array_equal(Ob[40:40 + L], O)


def test_the_tile_size_is_part_of_the_result():
    """Why the tile must be fixed: another tile size is another order of roundings -- close, but not the same bits."""
    c = syn.attention_inputs(38, [300], [300], Hq=2, Hkv=1, D=32)
    _, a = orc.attention(c["Q"], c["K"], c["V"], c["cu_q"], c["cu_k"], c["scale"], True, kv_tile=64)
    _, b = orc.attention(c["Q"], c["K"], c["V"], c["cu_q"], c["cu_k"], c["scale"], True, kv_tile=32)
    assert np.allclose(a, b, rtol=0, atol=2.0 ** -8)
    assert np.count_nonzero(a != b) > a.size // 10
    assert np.array_equal(a[:32], b[:32])                            # rows that fit one tile either way agree


def test_one_tile_is_the_two_pass_softmax():
    """With all visible keys in one tile the recurrence is the plain two-pass softmax in fp32 with bf16 weights."""
    c = syn.attention_inputs(39, [40], [40], Hq=1, Hkv=1, D=16)
    _, O32 = orc.attention(c["Q"], c["K"], c["V"], c["cu_q"], c["cu_k"], c["scale"], False, kv_tile=64)
    Q, K, V = f32(c["Q"])[:, 0], f32(c["K"])[:, 0], f32(c["V"])[:, 0]
    S = (Q.astype(np.float64) @ K.astype(np.float64).T).astype(np.float32) * np.float32(c["scale"] * 1.4426950408889634)
    P = np.exp2((S - S.max(axis=1, keepdims=True)).astype(np.float64))
    Pb = f32(syn.f32_to_bf16_bits(P.astype(np.float32))).astype(np.float64)
    want = (Pb @ V.astype(np.float64)) / P.sum(axis=1, keepdims=True)
    assert np.allclose(O32[:, 0], want, rtol=2e-5, atol=2e-6)


def test_queries_without_a_visible_key_give_zero():
    """More queries than keys under the causal rule (the first Lq - Lk queries precede every key)."""
    c = syn.attention_inputs(40, [6], [4], Hq=1, Hkv=1, D=8)
    O, _ = orc.attention(c["Q"], c["K"], c["V"], c["cu_q"], c["cu_k"], c["scale"], True)
    assert not O[:2].any() and np.array_equal(O[2, 0], c["V"][0, 0])


# ----------------------------------------------------------------------------- fixed splits of the key axis

def test_splits_fold_in_ascending_order_and_match_fp64():
    """Keys beyond one split (here 4 tiles of 16 = 64 keys per split, 300 keys): still the plain softmax within the
    rounding bound, and not the bits of the unsplit recurrence (the fold is another order of roundings)."""
    c = syn.attention_inputs(41, [300, 1, 40], [300, 290, 40], Hq=2, Hkv=1, D=16)
    O, O32 = orc.attention(c["Q"], c["K"], c["V"], c["cu_q"], c["cu_k"], c["scale"], True, kv_tile=16, kv_split=4)
    want, B = plain_attention_fp64(c, True)
    assert np.all(np.abs(O32 - want) <= 2.0 ** -8 * B)
    assert np.array_equal(O, syn.f32_to_bf16_bits(O32))
    _, U32 = orc.attention(c["Q"], c["K"], c["V"], c["cu_q"], c["cu_k"], c["scale"], True, kv_tile=16, kv_split=0)
    assert np.array_equal(O32[:64], U32[:64])                       # queries with at most one split of visible keys: same bits
    assert np.array_equal(O32[341:], U32[341:])                     # the 40-key sequence likewise
    assert np.count_nonzero(O32[64:300] != U32[64:300]) > 1000
    assert np.allclose(O32, U32, rtol=0, atol=2.0 ** -9)


def test_splits_by_hand_fold():
    """Two splits recomputed by two separate oracle calls and folded by the stated formula in numpy fp32."""
    D, T, S = 8, 16, 2                                              # 32 keys per split
    c = syn.attention_inputs(42, [1], [50], Hq=1, Hkv=1, D=D)
    _, O32 = orc.attention(c["Q"], c["K"], c["V"], [0, 1], [0, 50], c["scale"], False, kv_tile=T, kv_split=S)
    q = f32(c["Q"])[0, 0].astype(np.float32)
    cc = np.float32(np.float32(c["scale"]) * np.float32(1.44269504088896340736))
    states = []
    for lo, hi in ((0, 32), (32, 50)):
        K, V = f32(c["K"])[lo:hi, 0], f32(c["V"])[lo:hi, 0]
        m, l, o = np.float32(-np.inf), np.float32(0), np.zeros(D, dtype=np.float32)
        for t0 in range(0, hi - lo, T):
            s = []
            for j in range(t0, min(t0 + T, hi - lo)):
                dot = np.float32(0)
                for d in range(D):
                    dot = np.float32(dot + np.float32(q[d] * K[j, d]))
                s.append(np.float32(dot * cc))
            m2 = max(m, max(s))
            a = np.float32(np.exp2(np.float64(m - m2))) if np.isfinite(m) else np.float32(0)
            o = (o * a).astype(np.float32)
            ps = np.float32(0)
            for j, sj in zip(range(t0, t0 + len(s)), s):
                p = np.float32(np.exp2(np.float64(np.float32(sj - m2))))
                ps = np.float32(ps + p)
                pb = f32(syn.f32_to_bf16_bits(np.array([p], dtype=np.float32)))[0]
                o = (o + (pb * V[j]).astype(np.float32)).astype(np.float32)
            l = np.float32(np.float32(l * a) + ps)
            m = m2
        states.append((m, l, o))
    (m1, l1, o1), (m2, l2, o2) = states
    M = max(m1, m2)
    A, Bf = np.float32(np.exp2(np.float64(m1 - M))), np.float32(np.exp2(np.float64(m2 - M)))
    l = np.float32(np.float32(l1 * A) + np.float32(l2 * Bf))
    o = ((o1 * A).astype(np.float32) + (o2 * Bf).astype(np.float32)).astype(np.float32)
    assert np.allclose(O32[0, 0], o / l, rtol=3e-7, atol=1e-9)       # exp2 of libm vs numpy may differ in the last bit


def test_splits_keep_prefill_decode_and_batch_invariance():
    """With several splits: a query inside a prefill, as a decode step, in a chunk that starts inside a split, and in
    a batch with other sequences: one set of bits."""
    L = 200
    c = syn.attention_inputs(43, [L], [L], Hq=2, Hkv=1, D=16)
    kw = dict(kv_tile=16, kv_split=3)                               # 48 keys per split
    O, _ = orc.attention(c["Q"], c["K"], c["V"], c["cu_q"], c["cu_k"], c["scale"], True, **kw)
    for i in (0, 47, 48, 95, 96, 150, 199):
        Od, _ = orc.attention(c["Q"][i:i + 1], c["K"][:i + 1], c["V"][:i + 1], [0, 1], [0, i + 1], c["scale"], True, **kw)
        assert np.array_equal(Od[0], O[i]), i
    Oc, _ = orc.attention(c["Q"][70:130], c["K"][:130], c["V"][:130], [0, 60], [0, 130], c["scale"], True, **kw)
    assert np.array_equal(Oc, O[70:130])
    other = syn.attention_inputs(44, [30], [120], Hq=2, Hkv=1, D=16)
    Qb, Kb, Vb = (np.concatenate([other[n], c[n]]) for n in "QKV")
    Ob, _ = orc.attention(Qb, Kb, Vb, [0, 30, 30 + L], [0, 120, 120 + L], c["scale"], True, **kw)
    assert np.array_equal(Ob[30:], O)
    # the split size is part of the result, like the tile size
    O2, _ = orc.attention(c["Q"], c["K"], c["V"], c["cu_q"], c["cu_k"], c["scale"], True, kv_tile=16, kv_split=4)
    assert not np.array_equal(O2, O) and np.array_equal(O2[:48], O[:48])
