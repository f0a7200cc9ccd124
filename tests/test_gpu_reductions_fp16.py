"""GPU parity: RMSNorm, the fused tail and the row reductions on fp16 (IEEE binary16) rows against the CPU oracle.

The arithmetic is the one of the bf16 calls (App. B, App. C, Alg. 2); only the widening and the final rounding are
format-specific.  Everything here is bit-exact.
"""
import numpy as np
import pytest
import torch

import gpu_util as gu
from oracle import tbik_oracle as orc
from paper_2511_17826_amd import binding as tb
from paper_2511_17826_amd import synthetic as syn

pytestmark = pytest.mark.gpu


def _h(v):
    return np.asarray(v, dtype=np.float16).view(np.uint16)


@pytest.mark.parametrize("H", [4096, 5120, 24, 1000, 8192, 16392])
def test_rmsnorm_fp16_bit_exact_and_batch_invariant(H):
    Mmax = 2048 if H in (4096, 5120) else 300
    x, w = syn.rmsnorm_inputs(Mmax, H, fmt="fp16")
    xd, wd = gu.dev_f16(x), gu.dev_f16(w)
    full = tb.tbik_rmsnorm_f16(xd, wd, 1e-6)
    n_check = min(Mmax, 512)
    assert np.array_equal(gu.host_f16_bits(full[:n_check]), orc.rmsnorm(x[:n_check], w, 1e-6, fmt="fp16"))
    assert np.array_equal(gu.host_f16_bits(full[-64:]), orc.rmsnorm(x[-64:], w, 1e-6, fmt="fp16"))
    for M in (1, 2, 3, 7, 64, 255, 1024):
        if M > Mmax:
            continue
        y = tb.tbik_rmsnorm_f16(xd[:M].contiguous(), wd, 1e-6)
        assert torch.equal(y.view(torch.int16), full[:M].view(torch.int16)), M
    y = tb.tbik_rmsnorm_f16(xd[100:164].contiguous(), wd, 1e-6)
    assert torch.equal(y.view(torch.int16), full[100:164].view(torch.int16))


def test_rmsnorm_fp16_special_values():
    """The closed form for a row of ones; overflow of the output gives +inf; subnormal inputs are numbers."""
    H = 4096
    y = gu.host_f16_bits(tb.tbik_rmsnorm_f16(gu.dev_f16(_h(np.ones((5, H)))), gu.dev_f16(_h(np.ones(H))), 1e-6))
    r = np.float32(1.0) / np.sqrt(np.float32(1.0) + np.float32(1e-6), dtype=np.float32)
    assert np.all(y == _h(r))
    H = 64
    x = np.zeros((1, H), dtype=np.float16)
    x[0, 5] = 2.0
    y = gu.host_f16_bits(tb.tbik_rmsnorm_f16(gu.dev_f16(x.view(np.uint16)), gu.dev_f16(_h(np.full(H, 65504.0))), 0.0))
    assert y[0, 5] == 0x7C00 and np.all(np.delete(y[0], 5) == 0)
    tiny = np.full((1, H), 0x0001, dtype=np.uint16)
    y = gu.host_f16_bits(tb.tbik_rmsnorm_f16(gu.dev_f16(tiny), gu.dev_f16(_h(np.ones(H))), 0.0))
    assert np.all(y == 0x3C00)


def test_rmsnorm_fp16_wide_exponent_rows():
    """Rows that mix subnormal and large entries, against the oracle."""
    rng = np.random.Generator(np.random.PCG64(77))
    M, H = 40, 2048
    v = rng.standard_normal((M, H), dtype=np.float32) * np.exp2(rng.integers(-22, 8, (M, H))).astype(np.float32)
    x = syn.to_storage(v, "fp16")
    w = syn.normal_bf16(rng, (H,), 0.1, mean=1.0, fmt="fp16")
    y = gu.host_f16_bits(tb.tbik_rmsnorm_f16(gu.dev_f16(x), gu.dev_f16(w), 1e-6))
    assert np.array_equal(y, orc.rmsnorm(x, w, 1e-6, fmt="fp16"))


@pytest.mark.parametrize("P,M,H", [(1, 5, 4096), (2, 33, 5120), (4, 64, 4096), (8, 7, 24), (16, 3, 1000), (8, 1100, 4096)])
def test_fused_tail_fp16_equals_the_three_steps_and_the_oracle(P, M, H):
    rng = np.random.Generator(np.random.PCG64(200 + P + H))
    parts = (rng.standard_normal((P, M, H), dtype=np.float32) * np.float32(1.0 / np.sqrt(P)))
    res_b = syn.normal_bf16(rng, (M, H), 1.0, fmt="fp16")
    w_b = syn.normal_bf16(rng, (H,), 0.1, mean=1.0, fmt="fp16")
    pd = torch.from_numpy(parts).to("cuda:0")
    rd, wd = gu.dev_f16(res_b), gu.dev_f16(w_b)

    hid, out = tb.tbik_combine_residual_rmsnorm_f16(pd, rd, wd, 1e-6)
    y = tb.tbik_tree_combine(pd, out_dtype=torch.float16)
    hid3 = (y.float() + rd.float()).to(torch.float16)                   # fp32 add, one RNE rounding
    out3 = tb.tbik_rmsnorm_f16(hid3, wd, 1e-6)
    assert torch.equal(hid.view(torch.int16), hid3.view(torch.int16))
    assert torch.equal(out.view(torch.int16), out3.view(torch.int16))

    if M * H <= 300000:
        hid_o, out_o = orc.combine_residual_rmsnorm(parts, res_b, w_b, 1e-6, fmt="fp16")
        assert np.array_equal(gu.host_f16_bits(hid), hid_o)
        assert np.array_equal(gu.host_f16_bits(out), out_o)

    inplace = rd.clone()
    hid2, out2 = tb.tbik_combine_residual_rmsnorm_f16(pd, inplace, wd, 1e-6, hidden=inplace)
    assert torch.equal(inplace.view(torch.int16), hid.view(torch.int16))
    assert torch.equal(out2.view(torch.int16), out.view(torch.int16))
    h1, o1 = tb.tbik_combine_residual_rmsnorm_f16(pd[:, M - 1:M].contiguous(), rd[M - 1:M].contiguous(), wd, 1e-6)
    assert torch.equal(o1.view(torch.int16), out[M - 1:M].view(torch.int16))


def test_fused_tail_fp16_hand_value():
    """Two roundings: fp16(1 + 2^-11 + 2^-15) = 1 + 2^-10, then fp16(that + 2^-11) ties to the even 1 + 2^-9."""
    H = 8
    parts = np.zeros((2, 1, H), dtype=np.float32)
    parts[0, 0, :] = 1.0
    parts[1, 0, :] = 2.0 ** -11 + 2.0 ** -15
    res = _h(np.full((1, H), 2.0 ** -11))
    hid, out = tb.tbik_combine_residual_rmsnorm_f16(torch.from_numpy(parts).to("cuda:0"), gu.dev_f16(res),
                                                    gu.dev_f16(_h(np.ones(H))), 0.0)
    assert np.all(gu.host_f16_bits(hid) == 0x3C02)
    assert np.all(gu.host_f16_bits(out) == 0x3C00)


@pytest.mark.parametrize("V", [8, 1024, 20000, 16384 + 8, 151936])
def test_row_reductions_on_fp16_rows(V):
    M = 5
    rng = np.random.Generator(np.random.PCG64(V))
    xb = syn.normal_bf16(rng, (M, V), 2.0, fmt="fp16")
    xb[1, : min(V, 64)] = rng.integers(0, 0x0400, min(V, 64)).astype(np.uint16)       # a run of subnormals
    xf = syn.f16_bits_to_f32(xb)
    xd = gu.dev_f16(xb)
    s = gu.host_f32(tb.tbik_row_reduce(xd, tb.TBIK_SUM))
    assert np.array_equal(gu.u32(s), gu.u32(orc.row_sum(xf, orc.LEAF_BF16)))
    mx = gu.host_f32(tb.tbik_row_reduce(xd, tb.TBIK_MAX))
    assert np.array_equal(gu.u32(mx), gu.u32(xf.max(axis=1)))
    o = gu.host_f32(tb.tbik_row_reduce(xd, tb.TBIK_LOGSOFTMAX))
    want = orc.row_logsoftmax(xf, orc.LEAF_BF16)
    assert np.max(np.abs(o - want) / np.maximum(1.0, np.abs(want))) <= 1e-5
    # a row alone gives the same bits as inside the batch
    o1 = gu.host_f32(tb.tbik_row_reduce(xd[3:4].contiguous(), tb.TBIK_LOGSOFTMAX))
    assert np.array_equal(gu.u32(o1[0]), gu.u32(o[3]))
