"""The GPU's 8-, 6- and 4-bit GEMMs against the oracle's second in-leaf order (the measured accumulate step of the
matrix instruction for these formats): on RANDOM operands the comparison is a bit comparison.

Bar: every output bit-equal -- plain 8-bit operands (E4M3, E5M2) on every kernel and shard count, and the three
microscaling formats with their block scales."""
import numpy as np
import pytest
import torch

import gpu_util as gu
from oracle import tbik_oracle as orc
from paper_2511_17826_amd import binding as tb
from paper_2511_17826_amd import synthetic as syn

pytestmark = pytest.mark.gpu


def dev(*arrays):
    return [torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint8)).to("cuda:0") for a in arrays]


@pytest.mark.parametrize("fmt", ["e4m3", "e5m2"])
@pytest.mark.parametrize("M,K,N,leaf,g", [(70, 1024, 136, 128, 1), (130, 1536, 264, 128, 3), (33, 4096, 128, 256, 1)])
def test_plain_8_bit_random_operands_bit_exact(fmt, M, K, N, leaf, g):
    Xb, Wb = syn.gemm_random_fp8(M + K, M, K, N, fmt=fmt)
    want, want16 = orc.gemm_fp8_hw(Xb, Wb, leaf, g, fmt=fmt)
    Xd, Wt = dev(Xb, Wb.T)
    ns = K // (leaf * g)
    for v in (tb.VARIANT_AUTO, tb.VARIANT_REFERENCE, tb.VARIANT_T32):
        tb.tbik_set_gemm_variant(v)
        y = tb.tbik_gemm_fp8(Xd, Wt, leaf, g, fmt, out_dtype=torch.float32)
        assert np.array_equal(gu.u32(gu.host_f32(y)), want.view(np.uint32)), (v, fmt)
        for P in (p for p in (2, 8) if p <= ns):
            y = tb.tbik_tree_combine(tb.tbik_gemm_shard_partials_fp8(Xd, Wt, leaf, g, P, fmt), out_dtype=torch.float32)
            assert np.array_equal(gu.u32(gu.host_f32(y)), want.view(np.uint32)), (v, P, fmt)
    tb.tbik_set_gemm_variant(tb.VARIANT_AUTO)
    y16 = tb.tbik_gemm_fp8(Xd, Wt, leaf, g, fmt, out_dtype=torch.bfloat16)
    assert np.array_equal(gu.host_bf16_bits(y16), want16)


def _close(name, y, want, A):
    same = float(np.mean(gu.u32(y) == want.view(np.uint32)))
    worst = float(np.max(np.abs(y.astype(np.float64) - want) / A))
    print("%s: outputs equal to the instruction-level oracle bit for bit: %.5f, largest |gpu - oracle| / sum|x w| = %.3g" % (name, same, worst))
    assert same == 1.0 and worst == 0.0


@pytest.mark.parametrize("spread", [0, 3])
def test_microscaling_random_operands_bit_exact(spread):
    M, K, N, leaf = 130, 2048, 264, 256
    for fmt in ("e4m3", "e5m2"):
        Xq, Xs, Wq, Ws = syn.gemm_random_mxfp8(M + spread, M, K, N, fmt=fmt, scale_spread=spread)
        want, _ = orc.gemm_mxfp8_hw(Xq, Xs, Wq, Ws, leaf, 1, fmt=fmt)
        y = gu.host_f32(tb.tbik_gemm_mxfp8(*dev(Xq, Xs, Wq, Ws), leaf, 1, fmt, out_dtype=torch.float32))
        A = np.abs(orc.mxfp8_dequant(Xq, Xs, fmt).astype(np.float64)) @ np.abs(orc.mxfp8_dequant(Wq, Ws, fmt).astype(np.float64).T)
        _close("mxfp8 %s spread %d" % (fmt, spread), y, want, A)
    for fmt in ("e2m3", "e3m2"):
        Xp, Xs, Wp, Ws = syn.gemm_random_mxfp6(M + spread, M, K, N, fmt=fmt, scale_spread=spread)
        want, _ = orc.gemm_mxfp6_hw(Xp, Xs, Wp, Ws, leaf, 1, fmt=fmt)
        y = gu.host_f32(tb.tbik_gemm_mxfp6(*dev(Xp, Xs, Wp, Ws), leaf, 1, fmt, out_dtype=torch.float32))
        A = np.abs(orc.mxfp6_dequant(Xp, Xs, fmt).astype(np.float64)) @ np.abs(orc.mxfp6_dequant(Wp, Ws, fmt).astype(np.float64).T)
        _close("mxfp6 %s spread %d" % (fmt, spread), y, want, A)
    Xp, Xs, Wp, Ws = syn.gemm_random_mxfp4(M + spread, M, K, N, scale_spread=spread)
    want, _ = orc.gemm_mxfp4_hw(Xp, Xs, Wp, Ws, leaf, 1)
    y = gu.host_f32(tb.tbik_gemm_mxfp4(*dev(Xp, Xs, Wp, Ws), leaf, 1, out_dtype=torch.float32))
    A = np.abs(orc.mxfp4_dequant(Xp, Xs).astype(np.float64)) @ np.abs(orc.mxfp4_dequant(Wp, Ws).astype(np.float64).T)
    _close("mxfp4 spread %d" % spread, y, want, A)


def test_benchmark_shape_at_full_size_on_sampled_outputs():
    """4096^3 with leaf 256 (the benchmark's o_proj), plain 8-bit, MXFP8 and MXFP4 operands: a 48 x 40 sample of rows and
    columns of the full-size launch, bit for bit against the instruction-level oracle (which computes the sample as the
    product of the sampled rows of X with the sampled rows of the transposed weight)."""
    M = K = N = 4096
    rng = np.random.default_rng(17)
    rows, cols = np.sort(rng.choice(M, 48, replace=False)), np.sort(rng.choice(N, 40, replace=False))
    Xb, Wb = syn.gemm_random_fp8(41, M, K, N)
    y = gu.host_f32(tb.tbik_gemm_fp8(*dev(Xb, Wb.T), 256, 1, "e4m3", out_dtype=torch.float32))
    want, _ = orc.gemm_fp8_hw(Xb[rows], Wb[:, cols], 256, 1)
    assert np.array_equal(gu.u32(y[np.ix_(rows, cols)]), want.view(np.uint32))
    Xq, Xs, Wq, Ws = syn.gemm_random_mxfp8(42, M, K, N, scale_spread=2)
    y = gu.host_f32(tb.tbik_gemm_mxfp8(*dev(Xq, Xs, Wq, Ws), 256, 1, "e4m3", out_dtype=torch.float32))
    want, _ = orc.gemm_mxfp8_hw(Xq[rows], Xs[rows], Wq[cols], Ws[cols], 256, 1)
    assert np.array_equal(gu.u32(y[np.ix_(rows, cols)]), want.view(np.uint32))
    Xp, Xs, Wp, Ws = syn.gemm_random_mxfp4(43, M, K, N, scale_spread=2)
    y = gu.host_f32(tb.tbik_gemm_mxfp4(*dev(Xp, Xs, Wp, Ws), 256, 1, out_dtype=torch.float32))
    want, _ = orc.gemm_mxfp4_hw(Xp[rows], Xs[rows], Wp[cols], Ws[cols], 256, 1)
    assert np.array_equal(gu.u32(y[np.ix_(rows, cols)]), want.view(np.uint32))
