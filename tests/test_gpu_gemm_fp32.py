"""GPU parity and invariance tests of the tree-ordered GEMM on fp32 operands, through the C ABI.

The fp32 matrix instruction applies its two k-slots as two chained fused multiply-adds, which is the oracle's
definition of a leaf, so the bar is 0 bits against the oracle on every input -- random data with full significands,
wide exponent spreads and hand-built cancellations included -- for every kernel, every shard count and every batch.
"""
import numpy as np
import pytest
import torch

import gpu_util as gu
from conftest import read_tree_pins
from oracle import tbik_oracle as orc
from paper_2511_17826_amd import binding as tb
from paper_2511_17826_amd import synthetic as syn

pytestmark = pytest.mark.gpu

VARIANTS = [tb.VARIANT_REFERENCE, tb.VARIANT_T128, tb.VARIANT_T32]      # reference, 128-row tile, 32-row tile


@pytest.fixture(autouse=True)
def _reset_variant():
    yield
    tb.tbik_set_gemm_variant(tb.VARIANT_AUTO)


def run_all_routes(Xd, Wd, leaf, g, Ps, variants=VARIANTS):
    """{(variant, P): Y} through tbik_gemm_f32 (P == 0) and shard_partials_f32 + tree_combine (P >= 1)."""
    out = {}
    for v in variants:
        tb.tbik_set_gemm_variant(v)
        out[(v, 0)] = tb.tbik_gemm_f32(Xd, Wd, leaf, g)
        for P in Ps:
            parts = tb.tbik_gemm_shard_partials_f32(Xd, Wd, leaf, g, P)
            out[(v, P)] = tb.tbik_tree_combine(parts, out_dtype=torch.float32)
    tb.tbik_set_gemm_variant(tb.VARIANT_AUTO)
    torch.cuda.synchronize()
    return out


def test_hand_values_fused_product_and_order_inside_a_leaf():
    a = np.float32(1 + 2.0 ** -12)
    X = np.zeros((2, 64), dtype=np.float32)
    W = np.zeros((64, 8), dtype=np.float32)
    X[:, 0], X[:, 1] = -1.0, a
    W[0, :], W[1, :] = np.float32(1 + 2.0 ** -11), a
    for y in run_all_routes(gu.dev_f32(X), gu.dev_f32(W), 32, 1, [1, 2]).values():
        assert np.all(gu.host_f32(y) == np.float32(2.0 ** -24))           # a product rounded first would give 0
    X = np.zeros((1, 32), dtype=np.float32)
    X[0, :4] = [2.0 ** 24, 1.0, -2.0 ** 24, 1.0]
    W = np.ones((32, 4), dtype=np.float32)
    for y in run_all_routes(gu.dev_f32(X), gu.dev_f32(W), 32, 1, [1]).values():
        assert np.all(gu.host_f32(y) == 1.0)                              # ascending k; other orders give 0 or 2


@pytest.mark.parametrize("leaf,g", [(32, 1), (64, 3)])
def test_hand_derived_tree_values(leaf, g):
    """App. C worked by hand (tests/golden/tree_pins.txt): one exact product per superleaf."""
    for name, leaves, t_bits, _ in read_tree_pins():
        ns, sl = len(leaves), leaf * g
        K = ns * sl
        X = np.zeros((3, K), dtype=np.float32)
        W = np.zeros((K, 40), dtype=np.float32)
        for j, v in enumerate(leaves):
            k = j * sl + (j * 37) % sl
            X[:, k] = np.sqrt(np.float32(v))
            W[k, :] = np.sqrt(np.float32(v))
        outs = run_all_routes(gu.dev_f32(X), gu.dev_f32(W), leaf, g, [p for p in (1, 2, 4, 8) if p <= ns])
        for key, y in outs.items():
            assert np.all(gu.u32(gu.host_f32(y)) == t_bits), (name, key)


@pytest.mark.parametrize("M,K,N,leaf,g,spread", [(40, 1024, 136, 128, 1, 0), (130, 768, 260, 128, 3, 0), (7, 2048, 128, 64, 1, 12),
                                                 (257, 512, 72, 32, 1, 20), (33, 384, 520, 128, 3, 6), (5, 256, 12, 16, 1, 0)])
def test_bit_exact_against_the_oracle_every_route(M, K, N, leaf, g, spread):
    """Several tiles with ragged edges in M and N, superleaves of one to twelve K-steps, all shard counts; the last
    case has superleaves of 16 (not a multiple of the K-step) and runs on the reference kernel either way."""
    X, W = syn.gemm_random_f32(M + K, M, K, N, exp_spread=spread)
    want = orc.gemm_f32(X, W, leaf, g)
    ns = K // (leaf * g)
    outs = run_all_routes(gu.dev_f32(X), gu.dev_f32(W), leaf, g, [p for p in (1, 2, 4, 8, 16) if p <= ns])
    for key, y in outs.items():
        assert np.array_equal(gu.u32(gu.host_f32(y)), gu.u32(want)), key
    P = min(ns, 4)
    _, parts = orc.gemm_f32(X, W, leaf, g, orc.EVAL_SHARDED, P, want_partials=True)
    for v in VARIANTS:
        tb.tbik_set_gemm_variant(v)
        got = gu.host_f32(tb.tbik_gemm_shard_partials_f32(gu.dev_f32(X), gu.dev_f32(W), leaf, g, P))
        assert np.array_equal(gu.u32(got), gu.u32(parts)), v
        refp, refy = tb.tbik_gemm_reference_f32(gu.dev_f32(X), gu.dev_f32(W), leaf, g, 1)
        assert np.array_equal(gu.u32(gu.host_f32(refy)), gu.u32(want))


def test_subnormal_operands_and_results():
    """Products and sums in the subnormal range of fp32 are numbers, not zeros."""
    rng = np.random.Generator(np.random.PCG64(12))
    M, K, N = 9, 256, 40
    X = (rng.standard_normal((M, K)) * 2.0 ** -70).astype(np.float32)
    W = (rng.standard_normal((K, N)) * 2.0 ** -68).astype(np.float32)          # products around 2^-138: subnormal
    X[:, ::7] = (rng.standard_normal((M, len(range(0, K, 7)))) * 2.0 ** -130).astype(np.float32)   # subnormal operands
    W[::7, :] = (rng.standard_normal((len(range(0, K, 7)), N)) * 2.0 ** 3).astype(np.float32)
    want = orc.gemm_f32(X, W, 64, 1)
    assert np.count_nonzero(want) > want.size // 2 and np.max(np.abs(want)) < 2.0 ** -120
    for key, y in run_all_routes(gu.dev_f32(X), gu.dev_f32(W), 64, 1, [1, 4]).items():
        assert np.array_equal(gu.u32(gu.host_f32(y)), gu.u32(want)), key


def test_ragged_width_with_a_leading_dimension():
    """N = 130 inside rows of 136 floats (the last 16-byte chunk of a row is partly outside the matrix), output with
    its own leading dimension; M = 129 (one row in the second row of tiles)."""
    M, K, N, ld = 129, 512, 130, 136
    X, Wf = syn.gemm_random_f32(77, M, K, ld)
    Wd = gu.dev_f32(Wf)[:, :N]
    Y = torch.full((M, 140), -7.0, dtype=torch.float32, device="cuda:0")
    tb.tbik_gemm_f32(gu.dev_f32(X), Wd, 128, 1, out=Y[:, :N])
    want = orc.gemm_f32(X, np.ascontiguousarray(Wf[:, :N]), 128, 1)
    got = gu.host_f32(Y)
    assert np.array_equal(gu.u32(got[:, :N]), gu.u32(want)) and np.all(got[:, N:] == -7.0)


def test_batch_invariance_and_bf16_valued_operands_against_the_16_bit_oracle():
    K, N, leaf, g = 1536, 256, 128, 3
    X, W = syn.gemm_random_f32(5, 300, K, N)
    Xd, Wd = gu.dev_f32(X), gu.dev_f32(W)
    full = tb.tbik_gemm_f32(Xd, Wd, leaf, g)
    for M in (1, 2, 31, 33, 128, 129, 255):
        y = tb.tbik_gemm_f32(Xd[:M].contiguous(), Wd, leaf, g)
        assert torch.equal(y.view(torch.int32), full[:M].view(torch.int32)), M
    y = tb.tbik_gemm_f32(Xd[100:164].contiguous(), Wd, leaf, g)
    assert torch.equal(y.view(torch.int32), full[100:164].view(torch.int32))
    # operands that are bf16 numbers: every product is exact, so the fused chain is the plain sequential sum that the
    # oracle states for 16-bit operands -- bit for bit.  (The bf16 matrix instruction adds the 16 products of a step
    # in its own fixed order, so the bf16 entry point agrees with that sum within its stated tolerance only.)
    Xb, Wb = syn.gemm_random(9, 70, K, N)
    want16, _ = orc.gemm(Xb, Wb, leaf, g)
    y32 = tb.tbik_gemm_f32(gu.dev_f32(syn.bf16_bits_to_f32(Xb)), gu.dev_f32(syn.bf16_bits_to_f32(Wb)), leaf, g)
    assert np.array_equal(gu.u32(gu.host_f32(y32)), gu.u32(want16))


def test_paper_shape_sampled_parity_and_shard_invariance():
    """K = 6144, N = 2048 (the shape of the paper's kernel figure), leaf 128 (its FP32 block), K_first 3, 16 superleaves;
    M = 4096.  Sampled elements against the oracle; P in {1, 2, 4, 8, 16} and the whole-K call: one set of bits."""
    M, K, N, leaf, g = 4096, 6144, 2048, 128, 3
    X, W = syn.gemm_random_f32(21, M, K, N)
    Xd, Wd = gu.dev_f32(X), gu.dev_f32(W)
    y = tb.tbik_gemm_f32(Xd, Wd, leaf, g)
    rng = np.random.Generator(np.random.PCG64(22))
    rows = np.concatenate([rng.integers(0, M, 300), [0, M - 1, 127, 128]])
    cols = np.concatenate([rng.integers(0, N, 300), [0, N - 1, 127, 128]])
    want = orc.gemm_f32_elements(X, W, rows, cols, leaf, g)
    got = gu.host_f32(y)[rows, cols]
    assert np.array_equal(gu.u32(got), gu.u32(want))
    for P in (1, 2, 4, 8, 16):
        yp = tb.tbik_tree_combine(tb.tbik_gemm_shard_partials_f32(Xd, Wd, leaf, g, P), out_dtype=torch.float32)
        assert torch.equal(yp.view(torch.int32), y.view(torch.int32)), P
    exact = X[rows].astype(np.float64) @ W.astype(np.float64)
    exact = exact[np.arange(rows.size), cols]
    A = (np.abs(X[rows]).astype(np.float64) @ np.abs(W).astype(np.float64))[np.arange(rows.size), cols]
    assert np.all(np.abs(got - exact) <= 2e-6 * A)


def test_argument_validation_on_the_device():
    X = torch.zeros((4, 96), dtype=torch.float32, device="cuda:0")
    W = torch.zeros((96, 8), dtype=torch.float32, device="cuda:0")
    with pytest.raises(tb.TbikError) as e:
        tb.tbik_gemm_f32(X, W, 32, 1)                                    # three superleaves
    assert e.value.status == 2
    with pytest.raises(tb.TbikError) as e:
        tb.tbik_gemm_shard_partials_f32(X, W, 16, 3, 4)                  # more shards than superleaves
    assert e.value.status == 3
    W6 = torch.zeros((96, 6), dtype=torch.float32, device="cuda:0")      # rows of 24 bytes
    with pytest.raises(tb.TbikError) as e:
        tb.tbik_gemm_f32(X, W6, 32, 3)
    assert e.value.status == 5
