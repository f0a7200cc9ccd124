"""GPU parity and invariance tests of the tree-ordered GEMM on 8-bit floating-point operands (OCP E4M3 and E5M2),
through the C ABI.  The oracle holds W as [K, N]; the library takes it transposed, [N, K].

Bars, as for 16-bit operands: GPU vs GPU 0 bits (reference kernel, tiled kernel, every shard count, any batch);
bit-exact against the oracle wherever every superleaf sum is exact (hand values, leaf-sparse operands, small integers);
fp32 outputs on random data within 1e-5 * sum|x w| of fp64 and within 2 (leaf k_first + 8) 2^-24 sum|x w| of the oracle
(the 64 products of one matrix instruction are added in the instruction's own order); bf16 outputs are the rounding of
the kernel's own fp32 value.
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
FMTS = ["e4m3", "e5m2"]


@pytest.fixture(autouse=True)
def _reset_variant():
    yield
    tb.tbik_set_gemm_variant(tb.VARIANT_AUTO)


def dev_u8(bits):
    return torch.from_numpy(np.ascontiguousarray(bits, dtype=np.uint8)).to("cuda:0")


def operands(Xb, Wb):
    """Device X [M, K] and the transposed weight [N, K]."""
    return dev_u8(Xb), dev_u8(np.ascontiguousarray(Wb.T))


def run_all_routes(Xd, Wt, leaf, g, Ps, fmt):
    """{(kernel, P): fp32 Y}: tbik_gemm_fp8 (P == 0) and shard partials + tree combine, on the tiled and the reference kernel."""
    out = {}
    for name, v in (("tiled", tb.VARIANT_AUTO), ("reference", tb.VARIANT_REFERENCE), ("tile128", tb.VARIANT_T128),
                    ("tile64", tb.VARIANT_T64), ("tile32", tb.VARIANT_T32)):
        tb.tbik_set_gemm_variant(v)
        out[(name, 0)] = tb.tbik_gemm_fp8(Xd, Wt, leaf, g, fmt, out_dtype=torch.float32)
        for P in Ps:
            parts = tb.tbik_gemm_shard_partials_fp8(Xd, Wt, leaf, g, P, fmt)
            out[(name, P)] = tb.tbik_tree_combine(parts, out_dtype=torch.float32)
    tb.tbik_set_gemm_variant(tb.VARIANT_AUTO)
    y, parts = tb.tbik_gemm_reference_fp8(Xd, Wt, leaf, g, 1, fmt)
    out[("reference_entry", 1)] = y
    torch.cuda.synchronize()
    return out


@pytest.mark.parametrize("fmt", FMTS)
@pytest.mark.parametrize("leaf,g", [(128, 1), (128, 3), (256, 1), (64, 2)])
def test_hand_derived_tree_values(fmt, leaf, g):
    """App. C worked by hand (tests/golden/tree_pins.txt): one exact product per superleaf.  The pins' leaf values are
    1 and 2^-12 and so on: powers of four have 8-bit square roots in both formats."""
    used = 0
    for name, leaves, t_bits, _ in read_tree_pins():
        ns, sl = len(leaves), leaf * g
        K = ns * sl
        X = np.zeros((3, K), dtype=np.float32)
        W = np.zeros((K, 40), dtype=np.float32)
        for j, v in enumerate(leaves):
            k = j * sl + (j * 37) % sl
            X[:, k] = np.sqrt(np.float32(v))
            W[k, :] = np.sqrt(np.float32(v))
        Xb, Wb = syn.to_storage(X, fmt), syn.to_storage(W, fmt)
        if not (np.array_equal(syn.from_storage(Xb, fmt), X) and np.array_equal(syn.from_storage(Wb, fmt), W)):
            continue                                   # a pin whose leaves this 8-bit format cannot hold
        outs = run_all_routes(*operands(Xb, Wb), leaf, g, [p for p in (1, 2, 4, 8) if p <= ns], fmt)
        for key, y in outs.items():
            assert np.all(gu.u32(gu.host_f32(y)) == t_bits), (name, key)
        used += 1
    assert used > 0 or fmt == "e4m3"       # E4M3's smallest product is 2^-18: the pins with 2^-24 leaves need E5M2


@pytest.mark.parametrize("fmt", FMTS)
@pytest.mark.parametrize("M,K,N,leaf,g", [(70, 1024, 136, 128, 1), (130, 1536, 264, 256, 3), (1, 2048, 128, 128, 2), (257, 512, 8, 64, 1)])
def test_small_integers_bit_exact_against_the_oracle(fmt, M, K, N, leaf, g):
    Xb, Wb = syn.gemm_small_integers(M + N, M, K, N, mag=8, fmt=fmt)
    want, want16 = orc.gemm_fp8(Xb, Wb, leaf, g, fmt=fmt)
    ns = K // (leaf * g)
    outs = run_all_routes(*operands(Xb, Wb), leaf, g, [p for p in (1, 2, 4, 8) if p <= ns], fmt)
    for key, y in outs.items():
        assert np.array_equal(gu.u32(gu.host_f32(y)), want.view(np.uint32)), key
    y16 = tb.tbik_gemm_fp8(*operands(Xb, Wb), leaf, g, fmt, out_dtype=torch.bfloat16)
    assert np.array_equal(gu.host_bf16_bits(y16), want16)


@pytest.mark.parametrize("fmt", FMTS)
@pytest.mark.parametrize("M,K,N,superleaf", [(200, 2048, 264, 128), (300, 4096, 128, 256), (33, 1024, 520, 128)])
def test_leaf_sparse_operands_show_the_tree_bit_exact(fmt, M, K, N, superleaf):
    """One non-zero product per superleaf with a wide exponent spread: only the tree's additions round."""
    Xb, Wb = syn.gemm_leaf_sparse(M, M, K, N, superleaf, exp_spread=3 if fmt == "e4m3" else 5, fmt=fmt)
    want, want16 = orc.gemm_fp8(Xb, Wb, superleaf, 1, fmt=fmt)
    ns = K // superleaf
    outs = run_all_routes(*operands(Xb, Wb), superleaf, 1, [p for p in (1, 2, 4, 8, 16) if p <= ns], fmt)
    for key, y in outs.items():
        assert np.array_equal(gu.u32(gu.host_f32(y)), want.view(np.uint32)), key
    y16 = tb.tbik_gemm_fp8(*operands(Xb, Wb), superleaf, 1, fmt, out_dtype=torch.bfloat16)
    assert np.array_equal(gu.host_bf16_bits(y16), want16)


@pytest.mark.parametrize("fmt", FMTS)
@pytest.mark.parametrize("M,K,N,leaf,g", [(300, 2048, 264, 128, 1), (128, 4096, 256, 256, 1), (40, 1536, 136, 128, 3)])
def test_random_operands_all_routes_one_result_within_tolerance_of_the_oracle(fmt, M, K, N, leaf, g):
    Xb, Wb = syn.gemm_random_fp8(M * 3 + N, M, K, N, fmt)
    ns = K // (leaf * g)
    outs = run_all_routes(*operands(Xb, Wb), leaf, g, [p for p in (1, 2, 4, 8) if p <= ns], fmt)
    ref = gu.host_f32(outs[("reference", 0)])
    for key, y in outs.items():
        assert np.array_equal(gu.u32(gu.host_f32(y)), gu.u32(ref)), key
    want, _ = orc.gemm_fp8(Xb, Wb, leaf, g, fmt=fmt)
    X64, W64 = orc.fp8_to_f32(Xb, fmt).astype(np.float64), orc.fp8_to_f32(Wb, fmt).astype(np.float64)
    A = np.abs(X64) @ np.abs(W64)
    assert np.all(np.abs(ref.astype(np.float64) - X64 @ W64) <= 1e-5 * A)
    assert np.all(np.abs(ref.astype(np.float64) - want) <= 2 * (leaf * g + 8) * 2.0 ** -24 * A)
    # bf16 output: the one rounding of the kernel's own fp32 value
    y16 = tb.tbik_gemm_fp8(*operands(Xb, Wb), leaf, g, fmt, out_dtype=torch.bfloat16)
    assert np.array_equal(gu.host_bf16_bits(y16), syn.f32_to_bf16_bits(ref))


@pytest.mark.parametrize("fmt", FMTS)
def test_batch_invariance_and_repetitions(fmt):
    """Row m depends on row m of X only: any subset of rows, alone or in another position, gives the same bits."""
    M, K, N, leaf = 384, 4096, 512, 256
    Xb, Wb = syn.gemm_random_fp8(21, M, K, N, fmt)
    Xd, Wt = operands(Xb, Wb)
    full = tb.tbik_gemm_fp8(Xd, Wt, leaf, 1, fmt, out_dtype=torch.float32)
    for rows in ([0], [383], list(range(100, 140)), list(range(5, 384, 7))):
        sub = tb.tbik_gemm_fp8(Xd[rows].contiguous(), Wt, leaf, 1, fmt, out_dtype=torch.float32)
        assert torch.equal(sub.view(torch.int32), full[rows].view(torch.int32)), rows[:3]
    d = gu.digest(full)
    for _ in range(5):
        assert gu.digest(tb.tbik_gemm_fp8(Xd, Wt, leaf, 1, fmt, out_dtype=torch.float32)) == d


def test_full_size_tiled_equals_reference_and_sampled_oracle():
    """o_proj shape of the benchmark (4096^3), E4M3: the tiled kernel and the reference kernel agree on every bit for
    P in {1, 8}; sampled elements against the oracle."""
    M = K = N = 4096
    leaf = 256
    Xb, Wb = syn.gemm_random_fp8(31, M, K, N, "e4m3")
    Xd, Wt = operands(Xb, Wb)
    y = tb.tbik_gemm_fp8(Xd, Wt, leaf, 1, "e4m3", out_dtype=torch.float32)
    y_ref, _ = tb.tbik_gemm_reference_fp8(Xd, Wt, leaf, 1, 1, "e4m3")
    assert torch.equal(y.view(torch.int32), y_ref.view(torch.int32))
    y8 = tb.tbik_tree_combine(tb.tbik_gemm_shard_partials_fp8(Xd, Wt, leaf, 1, 8, "e4m3"), out_dtype=torch.float32)
    assert torch.equal(y.view(torch.int32), y8.view(torch.int32))
    rows, cols = syn.sample_elements(6, M, N, 32, 64)
    got = gu.host_f32(y)[rows, cols]
    want = orc.gemm_fp8_elements(Xb, Wb, rows, cols, leaf, 1)
    X64, W64 = orc.fp8_to_f32(Xb).astype(np.float64), orc.fp8_to_f32(Wb).astype(np.float64)
    A = np.einsum("ik,ki->i", np.abs(X64[rows]), np.abs(W64[:, cols]))
    assert np.all(np.abs(got.astype(np.float64) - want) <= 2 * (leaf + 8) * 2.0 ** -24 * A)
    print("fp8 o_proj: elements equal to the oracle bit for bit: %d of %d" % (int(np.sum(gu.u32(got) == want.view(np.uint32))), got.size))


def test_argument_checks():
    X = torch.zeros((8, 512), dtype=torch.uint8, device="cuda:0")
    Wt = torch.zeros((16, 512), dtype=torch.uint8, device="cuda:0")
    with pytest.raises(tb.TbikError):
        tb.tbik_gemm_fp8(X, Wt, 96, 1)                      # superleaf not a multiple of 64
    with pytest.raises(tb.TbikError):
        tb.tbik_gemm_shard_partials_fp8(X, Wt, 128, 1, 8)   # more shards than superleaves
    with pytest.raises(tb.TbikError):
        tb.tbik_gemm_fp8(X, Wt, 128, 1, out_dtype=torch.float16)
    with pytest.raises(tb.TbikError):
        tb.tbik_gemm_fp8(X[:, 8:], Wt[:, 8:], 63, 1)        # misaligned operands / illegal leaf
    assert tb.tbik_gemm_fp8(X[:0], Wt, 128, 1).shape == (0, 16)
