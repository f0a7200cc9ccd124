"""Pins for the oracle's tree-ordered GEMM (CPU only).

Sec. 3.3 (Y = XW with K split over ranks), Sec. 4.2 / App. D.1 (leaves, tree,
K_first), Theorem 1 (sharded == whole).  Every check compares the oracle with
something other than itself: hand values, int64 arithmetic, an fp64 dot product
with the summation-tree error bound, a sequential fp32 sum, a textbook pairwise
sum, or the paper's invariance claim.
"""
import numpy as np
import pytest

from conftest import read_tree_pins
from oracle import tbik_oracle as orc
from paper_2511_17826_amd import synthetic as syn

U = 2.0 ** -24  # unit roundoff of binary32


def u32(a):
    """fp32 bits; a scalar stays a scalar."""
    a = np.asarray(a, dtype=np.float32)
    return a.view(np.uint32) if a.ndim else np.uint32(a.reshape(1).view(np.uint32)[0])


def f32(bits16):
    return syn.bf16_bits_to_f32(bits16)


# ----------------------------------------------------------------------------- hand values

@pytest.mark.parametrize("leaf,k_first", [(16, 1), (64, 1), (32, 3)])
def test_hand_derived_tree_values_through_the_gemm(leaf, k_first):
    """Products 1 = 1*1 and 2^-24 = 2^-12 * 2^-12, one per superleaf, placed per the pin file:
    every superleaf sum is exact, so Y must equal the hand-derived T bits."""
    for name, leaves, t_bits, _ in read_tree_pins():
        ns = len(leaves)
        sl = leaf * k_first
        K = ns * sl
        X = np.zeros((2, K), dtype=np.float32)
        W = np.zeros((K, 3), dtype=np.float32)
        for j, v in enumerate(leaves):
            k = j * sl + (j * 5) % sl                 # anywhere inside superleaf j
            r = np.sqrt(np.float32(v))                # 1 -> 1, 2^-24 -> 2^-12, 0 -> 0
            X[:, k] = r
            W[k, :] = r
        Xb, Wb = syn.f32_to_bf16_bits(X), syn.f32_to_bf16_bits(W)
        assert np.array_equal(f32(Xb), X) and np.array_equal(f32(Wb), W)
        for ev, P in [(orc.EVAL_RECURSIVE, 1), (orc.EVAL_COUNTER, 1)] + [
                (orc.EVAL_SHARDED, p) for p in (1, 2, 4, 8) if p <= ns]:
            y32, ybf = orc.gemm(Xb, Wb, leaf, k_first, ev, P)
            assert np.all(u32(y32) == t_bits), (name, ev, P)
        assert int(u32(orc.gemm_element_alg1(Xb, Wb, 1, 2, leaf, k_first))) == t_bits


def test_shard_partials_hand_values():
    """four_a = [1, 0, 2^-24, 2^-24]: P=2 partials are [1, 2^-23]; P=4 partials are the leaves."""
    leaf = 16
    K = 4 * leaf
    X = np.zeros((1, K), dtype=np.float32)
    W = np.zeros((K, 1), dtype=np.float32)
    for j, v in enumerate([1.0, 0.0, 2.0 ** -24, 2.0 ** -24]):
        X[0, j * leaf + 3] = np.sqrt(v)
        W[j * leaf + 3, 0] = np.sqrt(v)
    Xb, Wb = syn.f32_to_bf16_bits(X), syn.f32_to_bf16_bits(W)
    _, _, p2 = orc.gemm(Xb, Wb, leaf, 1, orc.EVAL_SHARDED, 2, want_partials=True)
    assert [float(v) for v in p2[:, 0, 0]] == [1.0, 2.0 ** -23]
    _, _, p4 = orc.gemm(Xb, Wb, leaf, 1, orc.EVAL_SHARDED, 4, want_partials=True)
    assert [float(v) for v in p4[:, 0, 0]] == [1.0, 0.0, 2.0 ** -24, 2.0 ** -24]


# ----------------------------------------------------------------------------- Theorem 1 / invariance

def all_routes(Xb, Wb, leaf, g, Ps):
    outs = {("rec", 1): orc.gemm(Xb, Wb, leaf, g, orc.EVAL_RECURSIVE, 1),
            ("cnt", 1): orc.gemm(Xb, Wb, leaf, g, orc.EVAL_COUNTER, 1)}
    for P in Ps:
        outs[("shard", P)] = orc.gemm(Xb, Wb, leaf, g, orc.EVAL_SHARDED, P)
    return outs


def test_tiny_config_all_routes_bit_identical():
    """Tiny case (M=4, K=512, N=256, leaf 64): whole == counter == sharded P in {1,2,4,8}."""
    c = syn.gemm_tiny()
    outs = all_routes(c["X"], c["W"], c["leaf"], c["k_first"], (1, 2, 4, 8))
    ref32, refbf = outs[("rec", 1)]
    for key, (y32, ybf) in outs.items():
        assert np.array_equal(u32(y32), u32(ref32)), key
        assert np.array_equal(ybf, refbf), key


@pytest.mark.parametrize("K,leaf,g", [(768, 16, 3), (640, 16, 5), (1024, 64, 1), (1536, 256, 3), (800, 4, 25)])
def test_theorem1_with_k_first(K, leaf, g):
    Xb, Wb = syn.gemm_random(21, 5, K, 37)
    ns = K // (leaf * g)
    outs = all_routes(Xb, Wb, leaf, g, [p for p in (1, 2, 4, 8, 16) if p <= ns])
    ref32, _ = outs[("rec", 1)]
    for key, (y32, _) in outs.items():
        assert np.array_equal(u32(y32), u32(ref32)), key
    # Alg. 1 as one loop over tiles, and the plain single-element routine
    for (m, n) in [(0, 0), (4, 36), (2, 17)]:
        assert int(u32(orc.gemm_element_alg1(Xb, Wb, m, n, leaf, g))) == int(u32(ref32[m, n]))
        assert int(u32(orc.gemm_element(Xb, Wb, m, n, leaf, g))) == int(u32(ref32[m, n]))


def test_batch_invariance_and_row_permutation():
    """Row r of Y depends on row r of X only: any M, any position in the batch (App. B)."""
    Xb, Wb = syn.gemm_random(22, 16, 512, 64)
    full32, _ = orc.gemm(Xb, Wb, 32, 1)
    for M in (1, 3, 16):
        y32, _ = orc.gemm(Xb[:M], Wb, 32, 1)
        assert np.array_equal(u32(y32), u32(full32[:M]))
    perm = np.random.default_rng(0).permutation(16)
    y32, _ = orc.gemm(Xb[perm], Wb, 32, 1, orc.EVAL_SHARDED, 4)
    assert np.array_equal(u32(y32), u32(full32[perm]))


def test_tree_is_not_the_sequential_order_on_random_data():
    """Sanity of the whole point (Sec. 3.3): a chain over shards gives different bits than the tree."""
    c = syn.gemm_tiny()
    _, _, parts = orc.gemm(c["X"], c["W"], c["leaf"], 1, orc.EVAL_SHARDED, 8, want_partials=True)
    chain = parts[0].copy()
    for p in range(1, 8):
        chain = (chain + parts[p]).astype(np.float32)
    tree32, _ = orc.gemm(c["X"], c["W"], c["leaf"], 1)
    assert np.count_nonzero(u32(chain) != u32(tree32)) > 0


def test_illegal_parameters_are_rejected():
    Xb, Wb = syn.gemm_random(1, 2, 96, 4)
    with pytest.raises(ValueError):
        orc.gemm(Xb, Wb, 32, 1)                      # 3 superleaves: not a power of two
    with pytest.raises(ValueError):
        orc.gemm(Xb, Wb, 64, 1)                      # K not divisible
    Xb, Wb = syn.gemm_random(1, 2, 128, 4)
    with pytest.raises(ValueError):
        orc.gemm(Xb, Wb, 32, 1, orc.EVAL_SHARDED, 3)  # P not a power of two
    with pytest.raises(ValueError):
        orc.gemm(Xb, Wb, 32, 1, orc.EVAL_SHARDED, 8)  # P > number of superleaves


# ----------------------------------------------------------------------------- exact arithmetic

@pytest.mark.parametrize("M,K,N,leaf,g", [(7, 256, 33, 32, 1), (3, 768, 130, 64, 3), (1, 512, 5, 16, 1)])
def test_small_integer_inputs_equal_int64_matmul(M, K, N, leaf, g):
    """|x|,|w| <= 8: all partial sums < 2^24, so the result is the exact integer product (indexing pin)."""
    Xb, Wb = syn.gemm_small_integers(31, M, K, N)
    want = f32(Xb).astype(np.int64) @ f32(Wb).astype(np.int64)
    for ev, P in [(orc.EVAL_RECURSIVE, 1), (orc.EVAL_COUNTER, 1), (orc.EVAL_SHARDED, 2), (orc.EVAL_SHARDED, 4)]:
        y32, ybf = orc.gemm(Xb, Wb, leaf, g, ev, P)
        assert np.array_equal(y32.astype(np.int64), want)
        assert np.array_equal(y32, want.astype(np.float32))
    # a transposed or shifted operand would not survive this: X != X^T-like access, N != K
    rows, cols = syn.sample_elements(0, M, N, 4, 8)
    got = orc.gemm_elements(Xb, Wb, rows, cols, leaf, g)
    assert np.array_equal(got.astype(np.int64), want[rows, cols])


def test_leaf_sparse_inputs_equal_python_tree_of_exact_products():
    """One non-zero product per superleaf: superleaf sums are exact; the rest is T on 8 numbers."""
    K, sl = 8 * 48, 48
    Xb, Wb = syn.gemm_leaf_sparse(41, 3, K, 9, sl)
    y32, _ = orc.gemm(Xb, Wb, 16, 3)
    X, W = f32(Xb).astype(np.float64), f32(Wb).astype(np.float64)
    for m in range(3):
        for n in range(9):
            leaves = []
            for j in range(8):
                prods = X[m, j * sl:(j + 1) * sl] * W[j * sl:(j + 1) * sl, n]
                assert np.count_nonzero(prods) <= 1
                leaves.append(np.float32(prods.sum()))          # a single exact bf16*bf16 product
                assert float(leaves[-1]) == prods.sum()
            assert int(u32(y32[m, n])) == int(u32(orc.T_python(leaves)))


# ----------------------------------------------------------------------------- against fp64

def fp64_and_abs(Xb, Wb):
    X, W = f32(Xb).astype(np.float64), f32(Wb).astype(np.float64)
    return X @ W, np.abs(X) @ np.abs(W)


@pytest.mark.parametrize("cfg", ["tiny", "k768"])
def test_within_summation_tree_bound_of_fp64(cfg):
    """Products are exact, so only the h = (leaf*g - 1) + log2(n_s) additions on a path round:
    |y - y64| <= gamma_h * sum|x_k w_k|, gamma_h = h*u/(1 - h*u)."""
    if cfg == "tiny":
        c = syn.gemm_tiny()
        Xb, Wb, leaf, g = c["X"], c["W"], c["leaf"], c["k_first"]
    else:
        Xb, Wb = syn.gemm_random(51, 6, 768, 40)
        leaf, g = 32, 3
    K = Xb.shape[1]
    ns = K // (leaf * g)
    h = leaf * g - 1 + int(np.log2(ns)) + 1          # +1: the first add to +0 is exact but harmless
    gamma = h * U / (1 - h * U)
    y64, A = fp64_and_abs(Xb, Wb)
    y32, ybf = orc.gemm(Xb, Wb, leaf, g)
    err = np.abs(y32.astype(np.float64) - y64)
    assert np.all(err <= gamma * A)
    assert err.max() > 0                              # it is an fp32 computation, not fp64 in disguise
    # the stated GPU tolerance (1e-5 * A) leaves room above what the oracle itself does
    assert np.all(err <= 1e-5 * A)
    # the bf16 output is the rounding of the fp32 one (one rounding, not two)
    back = f32(ybf).astype(np.float64)
    assert np.all(np.abs(back - y32) <= np.abs(y32) * 2.0 ** -8)


def test_one_superleaf_is_the_sequential_fp32_dot():
    """leaf*k_first = K: no tree at all; y = sequential fp32 accumulation from +0 in ascending k."""
    Xb, Wb = syn.gemm_random(61, 3, 192, 7)
    X, W = f32(Xb), f32(Wb)
    for leaf, g in [(192, 1), (64, 3)]:
        y32, _ = orc.gemm(Xb, Wb, leaf, g)
        for m in range(3):
            for n in range(7):
                prods = (X[m] * W[:, n]).astype(np.float32)           # exact products
                seq = np.cumsum(prods, dtype=np.float32)[-1]          # numpy cumsum adds strictly in order
                assert int(u32(y32[m, n])) == int(u32(seq))


def test_leaf_one_is_textbook_pairwise_over_products():
    Xb, Wb = syn.gemm_random(62, 2, 64, 5)
    X, W = f32(Xb), f32(Wb)
    y32, _ = orc.gemm(Xb, Wb, 1, 1)
    for m in range(2):
        for n in range(5):
            v = (X[m] * W[:, n]).astype(np.float32)
            while v.size > 1:
                v = (v[0::2] + v[1::2]).astype(np.float32)
            assert int(u32(y32[m, n])) == int(u32(v[0]))


def test_transposed_or_shifted_operands_would_be_caught():
    """Planted mistakes (on the CPU): feeding W^T-like or k-shifted data changes the exact-integer result."""
    Xb, Wb = syn.gemm_small_integers(71, 4, 64, 64)
    want = f32(Xb).astype(np.int64) @ f32(Wb).astype(np.int64)
    y_t, _ = orc.gemm(Xb, np.ascontiguousarray(Wb.T), 16, 1)
    y_s, _ = orc.gemm(np.roll(Xb, 1, axis=1), Wb, 16, 1)
    assert not np.array_equal(y_t.astype(np.int64), want)
    assert not np.array_equal(y_s.astype(np.int64), want)


def test_row_sweep_equals_single_element_routine():
    """The whole-matrix routine (k outer, n inner) and the one-element routine give the same bits."""
    Xb, Wb = syn.gemm_random(81, 9, 1024, 300)
    y32, _ = orc.gemm(Xb, Wb, 64, 1)
    rows, cols = syn.sample_elements(5, 9, 300, 9, 40)
    got = orc.gemm_elements(Xb, Wb, rows, cols, 64, 1)
    assert np.array_equal(u32(got), u32(y32[rows, cols]))
    got = orc.gemm_elements(Xb, Wb, rows, cols, 64, 1, orc.EVAL_SHARDED, 8)
    assert np.array_equal(u32(got), u32(y32[rows, cols]))
