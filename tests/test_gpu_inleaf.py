"""GPU parity of the 16-bit tree GEMM, bit for bit on RANDOM operands, against the oracle's second in-leaf order (the
characterised accumulate step of the gfx950 matrix instruction; tests/test_oracle_inleaf.py pins the rule itself).

With the plain left-to-right oracle the comparison on random data needs a tolerance, because the matrix instruction adds
its products its own way.  With the instruction-level oracle nothing is left to tolerate: every kernel variant, every
shard count and every output format must reproduce it exactly.
"""
import numpy as np
import pytest
import torch

import gpu_util as gu
from oracle import tbik_oracle as orc
from paper_2511_17826_amd import binding as tb
from paper_2511_17826_amd import synthetic as syn

pytestmark = pytest.mark.gpu

API = {
    "bf16": (gu.dev_bf16, tb.tbik_gemm, tb.tbik_gemm_shard_partials, torch.bfloat16),
    "fp16": (gu.dev_f16, tb.tbik_gemm_f16, tb.tbik_gemm_shard_partials_f16, torch.float16),
}


@pytest.fixture(autouse=True)
def _reset_variant():
    yield
    tb.tbik_set_gemm_variant(tb.VARIANT_AUTO)


def no_subnormal_operands(bits_, fmt):
    v = np.abs(syn.from_storage(bits_, fmt))
    tiny = 2.0 ** -14 if fmt == "fp16" else 2.0 ** -126
    return not np.any((v > 0) & (v < tiny))


@pytest.mark.parametrize("fmt", ["bf16", "fp16"])
@pytest.mark.parametrize("M,K,N,leaf,g", [(200, 2048, 136, 128, 1), (70, 1536, 264, 256, 3), (33, 4096, 40, 256, 1)])
def test_whole_matrices_every_variant_and_shard_count(fmt, M, K, N, leaf, g):
    dev, gemm, partials, dt = API[fmt]
    Xb, Wb = syn.gemm_random(M + K, M, K, N, w_std=0.05, fmt=fmt)
    if fmt == "fp16":                       # N(0, 0.05) in binary16 brings subnormal operands along (below 2^-14)
        assert not no_subnormal_operands(Wb, fmt)
    want, want16 = orc.gemm_hw(Xb, Wb, leaf, g, fmt=fmt)
    Xd, Wd = dev(Xb), dev(Wb)
    ns = K // (leaf * g)
    for v in (tb.VARIANT_REFERENCE, tb.VARIANT_T128, tb.VARIANT_T64, tb.VARIANT_T32):
        tb.tbik_set_gemm_variant(v)
        y = gemm(Xd, Wd, leaf, g, out_dtype=torch.float32)
        assert np.array_equal(gu.u32(gu.host_f32(y)), want.view(np.uint32)), (v, "whole K")
        for P in (2, 8):
            if P <= ns:
                yp = tb.tbik_tree_combine(partials(Xd, Wd, leaf, g, P), out_dtype=torch.float32)
                assert np.array_equal(gu.u32(gu.host_f32(yp)), want.view(np.uint32)), (v, P)
    tb.tbik_set_gemm_variant(tb.VARIANT_AUTO)
    y16 = gemm(Xd, Wd, leaf, g, out_dtype=dt)
    assert np.array_equal(gu.host_bf16_bits(y16), want16)


@pytest.mark.parametrize("name", ["oproj", "downproj"])
def test_benchmark_shapes_at_full_size_on_sampled_outputs(name):
    """M = 4096 in the launch configuration bench.py times: 64 x 256 sampled outputs, 0 bits."""
    c = syn.gemm_oproj(4096) if name == "oproj" else syn.gemm_downproj(4096)
    Xd, Wd = gu.dev_bf16(c["X"]), gu.dev_bf16(c["W"])
    y = gu.host_f32(tb.tbik_gemm(Xd, Wd, c["leaf"], c["k_first"], out_dtype=torch.float32))
    rows, cols = syn.sample_elements(8, c["M"], c["N"], 64, 256)
    want = orc.gemm_hw_elements(c["X"], c["W"], rows, cols, c["leaf"], c["k_first"])
    assert np.array_equal(gu.u32(y[rows, cols]), want.view(np.uint32))
    y16 = gu.host_bf16_bits(tb.tbik_gemm(Xd, Wd, c["leaf"], c["k_first"], out_dtype=torch.bfloat16))
    assert np.array_equal(y16[rows, cols], syn.f32_to_bf16_bits(want))
    # and the plain in-leaf order differs from it on this data, within its stated tolerance (what the other tests bound)
    plain = orc.gemm_elements(c["X"], c["W"], rows, cols, c["leaf"], c["k_first"])
    print("%s: outputs where the plain in-leaf order gives other fp32 bits: %d of %d" % (name, int(np.sum(plain.view(np.uint32) != want.view(np.uint32))), want.size))
