"""GPU parity and invariance tests of the tree-ordered GEMM on MXFP8 operands (E4M3 / E5M2 elements, one E8M0 scale per
32 k), through the C ABI.

Bars as for the other formats: GPU vs GPU 0 bits (reference kernel, tiled kernel, every tile height, every shard count,
any batch); bit-exact against the oracle wherever every superleaf sum is exact (small-integer elements under equal
scales; one non-zero block per superleaf with its own scale); random operands: within 2 (leaf k_first + 8) 2^-24 sum|x w|
of the oracle plus 2^-13 sum|x w| for what the matrix instruction's fixed-point accumulate step drops when the 64
products of a step differ by many binades (observed: 3e-6 sum|x w| at scale spreads up to +-2, 1.2e-5 at +-4; the bar
is ten times that), and within 1e-4 sum|x w| of fp64; bf16 outputs are the rounding of the kernel's own fp32 value.
"""
import numpy as np
import pytest
import torch

import gpu_util as gu
from oracle import tbik_oracle as orc
from paper_2511_17826_amd import binding as tb
from paper_2511_17826_amd import synthetic as syn

pytestmark = pytest.mark.gpu
FMTS = ["e4m3", "e5m2"]


@pytest.fixture(autouse=True)
def _reset_variant():
    yield
    tb.tbik_set_gemm_variant(tb.VARIANT_AUTO)


def dev(*arrays):
    return [torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint8)).to("cuda:0") for a in arrays]


def run_all_routes(ops, leaf, g, Ps, fmt):
    """{(kernel, P): fp32 Y}: tbik_gemm_mxfp8 (P == 0) and shard partials + tree combine, tiled and reference kernels."""
    out = {}
    for name, v in (("tiled", tb.VARIANT_AUTO), ("reference", tb.VARIANT_REFERENCE), ("tile128", tb.VARIANT_T128),
                    ("tile64", tb.VARIANT_T64), ("tile32", tb.VARIANT_T32)):
        tb.tbik_set_gemm_variant(v)
        out[(name, 0)] = tb.tbik_gemm_mxfp8(*ops, leaf, g, fmt, out_dtype=torch.float32)
        for P in Ps:
            out[(name, P)] = tb.tbik_tree_combine(tb.tbik_gemm_shard_partials_mxfp8(*ops, leaf, g, P, fmt), out_dtype=torch.float32)
    tb.tbik_set_gemm_variant(tb.VARIANT_AUTO)
    out[("reference_entry", 1)] = tb.tbik_gemm_reference_mxfp8(*ops, leaf, g, 1, fmt)[0]
    torch.cuda.synchronize()
    return out


@pytest.mark.parametrize("fmt", FMTS)
@pytest.mark.parametrize("M,K,N,leaf,g", [(70, 1024, 136, 128, 1), (130, 1536, 264, 128, 3), (1, 2048, 128, 256, 2), (257, 512, 8, 64, 1)])
def test_small_integers_under_equal_scales_bit_exact_against_the_oracle(fmt, M, K, N, leaf, g):
    """Integer elements |v| <= 4 and one scale for all of X, one for all of W: every product is a multiple of a common
    power of two and the sums stay far below 2^24 of it, so any order gives the exact value.  Ragged M and N; superleaf
    64 runs on the reference kernel."""
    rng = np.random.default_rng(M + N)
    Xq = syn.f32_to_fp8_bits(rng.integers(-4, 5, size=(M, K)).astype(np.float32), fmt)
    Wq = syn.f32_to_fp8_bits(rng.integers(-4, 5, size=(N, K)).astype(np.float32), fmt)
    Xs = np.full((M, K // 32), 125, dtype=np.uint8)
    Ws = np.full((N, K // 32), 131, dtype=np.uint8)
    want, want16 = orc.gemm_mxfp8(Xq, Xs, Wq, Ws, leaf, g, fmt=fmt)
    ns = K // (leaf * g)
    outs = run_all_routes(dev(Xq, Xs, Wq, Ws), leaf, g, [p for p in (1, 2, 4, 8) if p <= ns], fmt)
    for key, y in outs.items():
        assert np.array_equal(gu.u32(gu.host_f32(y)), want.view(np.uint32)), key
    y16 = tb.tbik_gemm_mxfp8(*dev(Xq, Xs, Wq, Ws), leaf, g, fmt, out_dtype=torch.bfloat16)
    assert np.array_equal(gu.host_bf16_bits(y16), want16)


@pytest.mark.parametrize("fmt", FMTS)
@pytest.mark.parametrize("M,K,N,superleaf", [(200, 2048, 264, 256), (33, 4096, 136, 512)])
def test_one_block_per_superleaf_shows_scales_and_tree_bit_exact(fmt, M, K, N, superleaf):
    """In every superleaf one block of 32 k is non-zero (integer elements), with its own random scale per row and per
    column, spread over 2^+-10: the superleaf sums are exact sums of 32 same-scale products and only the tree's
    additions round.  This is where a wrong scale byte, a wrong block or a wrong lane would show."""
    rng = np.random.default_rng(M)
    Xv = rng.integers(-6, 7, size=(M, K)).astype(np.float32)
    Wq = syn.f32_to_fp8_bits(rng.integers(-6, 7, size=(N, K)).astype(np.float32), fmt)
    keep = np.zeros((M, K // 32), dtype=bool)
    for j in range(K // superleaf):
        keep[np.arange(M), j * (superleaf // 32) + rng.integers(0, superleaf // 32, size=M)] = True
    Xq = syn.f32_to_fp8_bits(np.where(np.repeat(keep, 32, axis=1), Xv, 0.0).astype(np.float32), fmt)
    Xs = (127 + rng.integers(-10, 11, size=(M, K // 32))).astype(np.uint8)
    Ws = (127 + rng.integers(-10, 11, size=(N, K // 32))).astype(np.uint8)
    want, _ = orc.gemm_mxfp8(Xq, Xs, Wq, Ws, superleaf, 1, fmt=fmt)
    ns = K // superleaf
    outs = run_all_routes(dev(Xq, Xs, Wq, Ws), superleaf, 1, [p for p in (1, 2, 4, 8) if p <= ns], fmt)
    for key, y in outs.items():
        assert np.array_equal(gu.u32(gu.host_f32(y)), want.view(np.uint32)), key


@pytest.mark.parametrize("fmt", FMTS)
@pytest.mark.parametrize("M,K,N,leaf,g,spread", [(300, 2048, 264, 256, 1, 0), (128, 4096, 256, 512, 1, 2), (40, 1536, 136, 128, 3, 4)])
def test_random_operands_all_routes_one_result_within_tolerance_of_the_oracle(fmt, M, K, N, leaf, g, spread):
    Xq, Xs, Wq, Ws = syn.gemm_random_mxfp8(M * 3 + N, M, K, N, fmt=fmt, scale_spread=spread)
    ns = K // (leaf * g)
    outs = run_all_routes(dev(Xq, Xs, Wq, Ws), leaf, g, [p for p in (1, 2, 4, 8) if p <= ns], fmt)
    ref = gu.host_f32(outs[("reference", 0)])
    for key, y in outs.items():
        assert np.array_equal(gu.u32(gu.host_f32(y)), gu.u32(ref)), key
    want, _ = orc.gemm_mxfp8(Xq, Xs, Wq, Ws, leaf, g, fmt=fmt)
    X64, W64 = orc.mxfp8_dequant(Xq, Xs, fmt).astype(np.float64), orc.mxfp8_dequant(Wq, Ws, fmt).astype(np.float64)
    A = np.abs(X64) @ np.abs(W64.T)
    assert np.all(np.abs(ref.astype(np.float64) - X64 @ W64.T) <= 1e-4 * A)
    assert np.all(np.abs(ref.astype(np.float64) - want) <= (2 * (leaf * g + 8) * 2.0 ** -24 + 2.0 ** -13) * A)
    print("mxfp8 %s spread %d: outputs equal to the oracle bit for bit: %.4f, largest |gpu - oracle| / sum|x w| = %.3g" % (
        fmt, spread, float(np.mean(gu.u32(ref) == want.view(np.uint32))), float(np.max(np.abs(ref.astype(np.float64) - want) / A))))
    y16 = tb.tbik_gemm_mxfp8(*dev(Xq, Xs, Wq, Ws), leaf, g, fmt, out_dtype=torch.bfloat16)
    assert np.array_equal(gu.host_bf16_bits(y16), syn.f32_to_bf16_bits(ref))


@pytest.mark.parametrize("fmt", FMTS)
def test_batch_invariance_and_repetitions(fmt):
    M, K, N, leaf = 384, 4096, 512, 256
    Xq, Xs, Wq, Ws = syn.gemm_random_mxfp8(21, M, K, N, fmt=fmt, scale_spread=1)
    X, XS, W, WS = dev(Xq, Xs, Wq, Ws)
    full = tb.tbik_gemm_mxfp8(X, XS, W, WS, leaf, 1, fmt, out_dtype=torch.float32)
    for rows in ([0], [383], list(range(100, 140)), list(range(5, 384, 7))):
        sub = tb.tbik_gemm_mxfp8(X[rows].contiguous(), XS[rows].contiguous(), W, WS, leaf, 1, fmt, out_dtype=torch.float32)
        assert torch.equal(sub.view(torch.int32), full[rows].view(torch.int32)), rows[:3]
    d = gu.digest(full)
    for _ in range(5):
        assert gu.digest(tb.tbik_gemm_mxfp8(X, XS, W, WS, leaf, 1, fmt, out_dtype=torch.float32)) == d


def test_full_size_tiled_equals_reference():
    """o_proj shape of the benchmark (4096^3): the tiled and the reference kernel agree on every bit, P in {1, 8}."""
    M = K = N = 4096
    Xq, Xs, Wq, Ws = syn.gemm_random_mxfp8(31, M, K, N)
    ops = dev(Xq, Xs, Wq, Ws)
    y = tb.tbik_gemm_mxfp8(*ops, 256, 1, out_dtype=torch.float32)
    y_ref, _ = tb.tbik_gemm_reference_mxfp8(*ops, 256, 1, 1)
    assert torch.equal(y.view(torch.int32), y_ref.view(torch.int32))
    y8 = tb.tbik_tree_combine(tb.tbik_gemm_shard_partials_mxfp8(*ops, 256, 1, 8), out_dtype=torch.float32)
    assert torch.equal(y.view(torch.int32), y8.view(torch.int32))


def test_scale_one_equals_the_unscaled_8_bit_gemm():
    """Every scale 2^0: the same bits as tbik_gemm_fp8 on the same (random) patterns -- the two kernels present a step of
    64 k to the instruction in the same, ascending arrangement."""
    Xq, Xs, Wq, Ws = syn.gemm_random_mxfp8(5, 200, 2048, 264)
    Xs[:] = 127
    Ws[:] = 127
    X, XS, W, WS = dev(Xq, Xs, Wq, Ws)
    a = tb.tbik_gemm_mxfp8(X, XS, W, WS, 256, 1, out_dtype=torch.float32)
    b = tb.tbik_gemm_fp8(X, W, 256, 1, out_dtype=torch.float32)
    assert torch.equal(a.view(torch.int32), b.view(torch.int32))


def test_argument_checks():
    X = torch.zeros((8, 256), dtype=torch.uint8, device="cuda:0")
    XS = torch.full((8, 8), 127, dtype=torch.uint8, device="cuda:0")
    W = torch.zeros((16, 256), dtype=torch.uint8, device="cuda:0")
    WS = torch.full((16, 8), 127, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(tb.TbikError):
        tb.tbik_gemm_mxfp8(X, XS, W, WS, 96, 1)                      # superleaf not a multiple of 64
    with pytest.raises(tb.TbikError):
        tb.tbik_gemm_shard_partials_mxfp8(X, XS, W, WS, 256, 1, 4)   # more shards than superleaves
    with pytest.raises(tb.TbikError):
        tb.tbik_gemm_mxfp8(X, XS, W, WS, 128, 1, out_dtype=torch.float16)
    assert tb.tbik_gemm_mxfp8(X[:0], XS[:0], W, WS, 128, 1).shape == (0, 16)
    assert float(tb.tbik_gemm_mxfp8(X, XS, W, WS, 128, 1, out_dtype=torch.float32).abs().max()) == 0.0
