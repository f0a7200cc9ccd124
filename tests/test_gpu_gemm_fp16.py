"""GPU parity and invariance tests of the tree-ordered GEMM on fp16 (IEEE binary16) operands, through the C ABI.

Same bars as for bf16 operands: GPU vs GPU 0 bits; bit-exact against the oracle wherever every superleaf sum is
exact (hand values, leaf-sparse operands, small integers); fp32 outputs on random data within
1e-5 * sum|x w| of fp64 and within 2*(leaf*k_first+8)*2^-24 * sum|x w| of the oracle; fp16 outputs equal to the
round-to-nearest-even of the kernel's own fp32 value, and to fp16(oracle) except next to a rounding boundary.
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

VARIANTS = [tb.VARIANT_REFERENCE, tb.VARIANT_T128, tb.VARIANT_T32, tb.VARIANT_T64]


@pytest.fixture(autouse=True)
def _reset_variant():
    yield
    tb.tbik_set_gemm_variant(tb.VARIANT_AUTO)


def run_all_routes(Xd, Wd, leaf, g, Ps, variants=VARIANTS):
    """{(variant, P): fp32 Y} through tbik_gemm_f16 (P == 0) and shard_partials_f16 + tree_combine (P >= 1)."""
    out = {}
    for v in variants:
        tb.tbik_set_gemm_variant(v)
        out[(v, 0)] = tb.tbik_gemm_f16(Xd, Wd, leaf, g, out_dtype=torch.float32)
        for P in Ps:
            parts = tb.tbik_gemm_shard_partials_f16(Xd, Wd, leaf, g, P)
            out[(v, P)] = tb.tbik_tree_combine(parts, out_dtype=torch.float32)
    tb.tbik_set_gemm_variant(tb.VARIANT_AUTO)
    torch.cuda.synchronize()
    return out


@pytest.mark.parametrize("leaf,g", [(64, 1), (64, 3), (256, 1)])
def test_hand_derived_tree_values(leaf, g):
    """App. C worked by hand (tests/golden/tree_pins.txt): one exact product per superleaf."""
    for name, leaves, t_bits, _ in read_tree_pins():
        ns, sl = len(leaves), leaf * g
        K = ns * sl
        X = np.zeros((3, K), dtype=np.float32)
        W = np.zeros((K, 40), dtype=np.float32)
        for j, v in enumerate(leaves):
            k = j * sl + (j * 37) % sl
            X[:, k] = np.sqrt(np.float32(v))           # 1 or 2^-12: both binary16 normals
            W[k, :] = np.sqrt(np.float32(v))
        Xb, Wb = syn.f32_to_f16_bits(X), syn.f32_to_f16_bits(W)
        assert np.array_equal(syn.f16_bits_to_f32(Xb), X)
        outs = run_all_routes(gu.dev_f16(Xb), gu.dev_f16(Wb), leaf, g, [p for p in (1, 2, 4, 8) if p <= ns])
        for key, y in outs.items():
            assert np.all(gu.u32(gu.host_f32(y)) == t_bits), (name, key)


def test_eleven_bit_significands_subnormals_and_output_rounding():
    """Values that only binary16 holds.  Superleaf 0: (1 + 2^-10)^2 = 1 + 2^-9 + 2^-20 (21 significant bits, exact
    in fp32).  Superleaf 1: the smallest subnormal 2^-24 times 1024 = 2^-14.  The other two: 0.
    T = ((p0 + p1) + (0 + 0)); fp32: 1 + 2^-9 + 2^-14 + 2^-20; fp16 output: 1 + 2^-9 (0x3C02).
    Column 1 of W scales everything by 2^-16, which puts the fp16 output into the subnormal range:
    2^-16 * (1 + 2^-9 + ...) -> 2^-16 = 0x0100 after rounding on the 2^-24 grid."""
    leaf, ns = 64, 4
    K = leaf * ns
    X = np.zeros((2, K), dtype=np.uint16)
    W = np.zeros((K, 8), dtype=np.uint16)
    X[:, 5] = 0x3C01                 # 1 + 2^-10
    W[5, :] = 0x3C01
    X[:, leaf + 9] = 0x0001          # 2^-24
    W[leaf + 9, :] = 0x6400          # 1024
    W[5, 1] = int(syn.f32_to_f16_bits(np.array([(1 + 2.0 ** -10) * 2.0 ** -16]))[0])
    W[leaf + 9, 1] = int(syn.f32_to_f16_bits(np.array([2.0 ** -6]))[0])
    y_orc, y16_orc = orc.gemm(X, W, leaf, 1, fmt="fp16")
    assert float(y_orc[0, 0]) == 1 + 2.0 ** -9 + 2.0 ** -14 + 2.0 ** -20 and int(y16_orc[0, 0]) == 0x3C02
    assert int(y16_orc[0, 1]) == 0x0100
    Xd, Wd = gu.dev_f16(X), gu.dev_f16(W)
    for key, y in run_all_routes(Xd, Wd, leaf, 1, [1, 2, 4]).items():
        assert np.array_equal(gu.u32(gu.host_f32(y)), gu.u32(y_orc)), key
    for v in VARIANTS:
        tb.tbik_set_gemm_variant(v)
        y16 = tb.tbik_gemm_f16(Xd, Wd, leaf, 1, out_dtype=torch.float16)
        assert np.array_equal(gu.host_f16_bits(y16), y16_orc), v
        parts = tb.tbik_gemm_shard_partials_f16(Xd, Wd, leaf, 1, 2)
        assert np.array_equal(gu.host_f16_bits(tb.tbik_tree_combine(parts, out_dtype=torch.float16)), y16_orc), v


def test_output_rounding_ties_and_overflow_through_the_combine():
    """tbik_tree_combine with a binary16 output on hand-placed fp32 values: ties go to even, 65520 goes to infinity."""
    vals = np.array([1.0, 1 + 2.0 ** -11, 1 + 2.0 ** -11 + 2.0 ** -23, 1 + 3 * 2.0 ** -11, -2.0, 65504.0, 65519.99,
                     65520.0, 1e9, 2.0 ** -24, 2.0 ** -25, 1.5 * 2.0 ** -24, 2.0 ** -14, -(2.0 ** -14) * (1 - 2.0 ** -12),
                     0.0, 3.14159], dtype=np.float32)
    parts = np.stack([vals, np.zeros_like(vals)]).reshape(2, 2, 8)
    with np.errstate(over="ignore"):
        want = vals.astype(np.float16).view(np.uint16).reshape(2, 8)
    _, y16_orc = orc.tree_combine(parts, fmt="fp16")
    assert np.array_equal(y16_orc, want)
    y16 = tb.tbik_tree_combine(gu.dev_f32(parts), out_dtype=torch.float16)
    assert np.array_equal(gu.host_f16_bits(y16), want)
    y16 = tb.tbik_tree_combine(gu.dev_f32(parts[:, :, :7].copy()), out_dtype=torch.float16)     # scalar path (N % 4 != 0)
    assert np.array_equal(gu.host_f16_bits(y16), want[:, :7])


@pytest.mark.parametrize("M,K,N,leaf,g", [(77, 2048, 200, 64, 1), (130, 3072, 264, 64, 3), (300, 4096, 136, 256, 1)])
def test_leaf_sparse_bit_exact_against_oracle(M, K, N, leaf, g):
    """One non-zero product per superleaf: whatever happens inside a leaf is exact, so the tree must match bit for bit."""
    Xb, Wb = syn.gemm_leaf_sparse(400 + M, M, K, N, leaf * g, exp_spread=6, fmt="fp16")
    y_orc, y16_orc = orc.gemm(Xb, Wb, leaf, g, fmt="fp16")
    Xd, Wd = gu.dev_f16(Xb), gu.dev_f16(Wb)
    ns = K // (leaf * g)
    outs = run_all_routes(Xd, Wd, leaf, g, [p for p in (1, 2, 4, 8, 16) if p <= ns])
    for key, y in outs.items():
        assert np.array_equal(gu.u32(gu.host_f32(y)), gu.u32(y_orc)), key
    y16 = tb.tbik_gemm_f16(Xd, Wd, leaf, g, out_dtype=torch.float16)
    assert np.array_equal(gu.host_f16_bits(y16), y16_orc)


def test_deep_tree_and_64_shards():
    Xb, Wb = syn.gemm_leaf_sparse(500, 9, 16384, 72, 64, exp_spread=6, fmt="fp16")
    y_orc, _ = orc.gemm(Xb, Wb, 64, 1, fmt="fp16")
    outs = run_all_routes(gu.dev_f16(Xb), gu.dev_f16(Wb), 64, 1, [1, 16, 64])
    for key, y in outs.items():
        assert np.array_equal(gu.u32(gu.host_f32(y)), gu.u32(y_orc)), key


@pytest.mark.parametrize("M,K,N,leaf,g", [(70, 1024, 136, 64, 1), (33, 768, 264, 64, 3), (1, 512, 8, 64, 1),
                                          (129, 2048, 128, 128, 2)])
def test_small_integer_inputs_exact(M, K, N, leaf, g):
    """|x|,|w| <= 8: every order gives the exact integer, so this pins indexing, layout and ragged edges."""
    Xb, Wb = syn.gemm_small_integers(600 + M, M, K, N, fmt="fp16")
    want = (syn.f16_bits_to_f32(Xb).astype(np.int64) @ syn.f16_bits_to_f32(Wb).astype(np.int64)).astype(np.float32)
    ns = K // (leaf * g)
    outs = run_all_routes(gu.dev_f16(Xb), gu.dev_f16(Wb), leaf, g, [p for p in (1, 2, 4) if p <= ns])
    for key, y in outs.items():
        assert np.array_equal(gu.host_f32(y), want), key


def test_oproj_shape_invariance_and_sampled_parity():
    """The 8B-class o_proj shape with fp16 operands: one set of bits for every M, P, variant and repetition; sampled
    elements against the oracle and fp64 within the stated tolerances."""
    c = syn.gemm_oproj(4096, fmt="fp16")
    leaf, g, N = c["leaf"], c["k_first"], c["N"]
    Xd, Wd = gu.dev_f16(c["X"]), gu.dev_f16(c["W"])
    full = tb.tbik_gemm_f16(Xd, Wd, leaf, g, out_dtype=torch.float32)
    torch.cuda.synchronize()
    digests = {gu.digest(full)}
    for rep in range(2):
        for P in (1, 2, 4, 8):
            parts = tb.tbik_gemm_shard_partials_f16(Xd, Wd, leaf, g, P)
            digests.add(gu.digest(tb.tbik_tree_combine(parts, out_dtype=torch.float32)))
            del parts
        digests.add(gu.digest(tb.tbik_gemm_f16(Xd, Wd, leaf, g, out_dtype=torch.float32)))
    assert len(digests) == 1
    for M in (1, 16, 64, 256, 1024):
        for v in (tb.VARIANT_AUTO, tb.VARIANT_T128, tb.VARIANT_T32, tb.VARIANT_T64):
            tb.tbik_set_gemm_variant(v)
            y = tb.tbik_gemm_f16(Xd[:M], Wd, leaf, g, out_dtype=torch.float32)
            assert torch.equal(y.view(torch.int32), full[:M].view(torch.int32)), (M, v)
            parts = tb.tbik_gemm_shard_partials_f16(Xd[:M], Wd, leaf, g, 8)
            y = tb.tbik_tree_combine(parts, out_dtype=torch.float32)
            assert torch.equal(y.view(torch.int32), full[:M].view(torch.int32)), (M, v, "P8")
    tb.tbik_set_gemm_variant(tb.VARIANT_AUTO)
    y = tb.tbik_gemm_f16(Xd[1000:1001], Wd, leaf, g, out_dtype=torch.float32)
    assert torch.equal(y.view(torch.int32), full[1000:1001].view(torch.int32))
    parts, yref = tb.tbik_gemm_reference_f16(Xd[:160], Wd, leaf, g, 1)
    assert torch.equal(yref.view(torch.int32), full[:160].view(torch.int32))

    rows, cols = syn.sample_elements(12, 4096, N, 64, 256)
    y_orc = orc.gemm_elements(c["X"], c["W"], rows, cols, leaf, g, fmt="fp16")
    y64, A = gu.fp64_ref(c["X"], c["W"], rows, cols, fmt="fp16")
    y_gpu = gu.host_f32(full)[rows, cols]
    gu.check_fp32_against_fp64(y_gpu, y64, A)
    assert np.all(np.abs(y_gpu.astype(np.float64) - y_orc) <= 2 * (leaf * g + 8) * 2.0 ** -24 * A)
    y16 = gu.host_f16_bits(tb.tbik_gemm_f16(Xd, Wd, leaf, g, out_dtype=torch.float16))[rows, cols]
    n_exc = gu.check_bf16_against_oracle(y16, y_gpu, y_orc, fmt="fp16")
    assert n_exc <= max(2, y_gpu.size // 100), n_exc


def test_output_type_must_go_with_the_operand_format():
    Xd = torch.zeros((4, 64), dtype=torch.float16, device="cuda:0")
    Wd = torch.zeros((64, 8), dtype=torch.float16, device="cuda:0")
    with pytest.raises(tb.TbikError) as e:
        tb.tbik_gemm_f16(Xd, Wd, 64, 1, out_dtype=torch.bfloat16)
    assert e.value.status == 4
    with pytest.raises(tb.TbikError) as e:
        tb.tbik_gemm(Xd.view(torch.bfloat16), Wd.view(torch.bfloat16), 64, 1, out_dtype=torch.float16)
    assert e.value.status == 4
