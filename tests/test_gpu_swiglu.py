"""The gated activation of the MLP block on the GPU: tbik_silu_mul against the oracle, and tbik_gemm_swiglu (the
[gate | up] GEMM that applies it before anything is stored) against "two tbik_gemm calls, then tbik_silu_mul", bit for bit,
on shapes that take each of its three routes: the 128 x 128 tile's epilogue, the combine of a K split, and the staged one.

Tolerance of the activation against the oracle (fp32 steps with libm's expf and a correctly rounded division): the
kernels use the hardware's exponential and reciprocal, about one fp32 ulp each, so the fp32 value before the final
rounding differs by a few fp32 ulps and the 16-bit result can fall on the other side of a rounding boundary: at most
one 16-bit step, in fewer than one element in a thousand (a boundary is hit with probability of about 2^-13 per ulp).
Results below 2^-100 in magnitude are compared by value only: for gate below about -87 the reciprocal leaves the normal
range and the kernel returns a zero where the oracle has a number below 1e-36.
"""
import numpy as np
import pytest
import torch

import gpu_util as gu
from oracle import tbik_oracle as orc
from paper_2511_17826_amd import binding as tb
from paper_2511_17826_amd import synthetic as syn

pytestmark = pytest.mark.gpu

DEV = {"bf16": gu.dev_bf16, "fp16": gu.dev_f16}
TORCH = {"bf16": torch.bfloat16, "fp16": torch.float16}


def bits(t):
    return gu.host_bf16_bits(t)


def assert_act_close(got_bits, want_bits, fmt, where):
    got = syn.from_storage(got_bits, fmt).astype(np.float64)
    want = syn.from_storage(want_bits, fmt).astype(np.float64)
    step = gu._bf16_spacing(want, fmt)
    assert np.all(np.abs(got - want) <= step + 2.0 ** -100), where
    differ = (got_bits != want_bits) & (np.abs(want) >= 2.0 ** -100)      # below: the flush of gate < -87, signed zeros
    assert np.mean(differ) <= 1e-3, (where, float(np.mean(differ)))


@pytest.mark.parametrize("fmt", ["bf16", "fp16"])
@pytest.mark.parametrize("M,I,pad", [(70, 1032, 0), (5, 37, 3), (1, 12288, 0), (300, 4096, 8)])
def test_silu_mul_against_the_oracle(fmt, M, I, pad):
    rng = np.random.default_rng(M * 7 + I)
    g = syn.to_storage(rng.standard_normal((M, I), dtype=np.float32) * 3, fmt)
    u = syn.to_storage(rng.standard_normal((M, I), dtype=np.float32), fmt)
    want = orc.silu_mul(g, u, fmt)
    # gate and up as the halves of one padded buffer (leading dimension 2 I + pad), and on their own
    buf = torch.zeros((M, 2 * I + pad), dtype=TORCH[fmt], device="cuda:0")
    buf[:, :I] = DEV[fmt](g)
    buf[:, I:2 * I] = DEV[fmt](u)
    a1 = tb.tbik_silu_mul(buf[:, :I], buf[:, I:2 * I])
    a2 = tb.tbik_silu_mul(DEV[fmt](g), DEV[fmt](u))
    torch.cuda.synchronize()
    assert np.array_equal(bits(a1), bits(a2))                 # vector and scalar paths, one definition
    assert_act_close(bits(a1), want, fmt, (fmt, M, I))


def test_silu_mul_exact_cases_and_batch_position():
    b = lambda v: gu.dev_bf16(syn.f32_to_bf16_bits(np.asarray(v, dtype=np.float32)))
    out = tb.tbik_silu_mul(b([[32, 64, 48, 0, 0, -104, -200, 1]]), b([[3, -0.5, 1.5, 7, -7, 2, -2, 1]])).float().cpu().numpy()
    assert out[0, :3].tolist() == [96.0, -32.0, 72.0]
    assert out[0, 3:7].tolist() == [0.0] * 4
    assert out[0, 7] == 0.73046875
    # a row's bits do not depend on the batch around it
    rng = np.random.default_rng(3)
    g = gu.dev_bf16(syn.to_storage(rng.standard_normal((64, 2048), dtype=np.float32) * 3))
    u = gu.dev_bf16(syn.to_storage(rng.standard_normal((64, 2048), dtype=np.float32)))
    full = tb.tbik_silu_mul(g, u)
    one = tb.tbik_silu_mul(g[17:18].contiguous(), u[17:18].contiguous())
    assert torch.equal(full[17:18].view(torch.int16), one.view(torch.int16))


def unfused(X, W_gu, leaf, g):
    I = W_gu.shape[1] // 2
    gemm = tb.tbik_gemm if X.dtype == torch.bfloat16 else tb.tbik_gemm_f16
    gate = gemm(X, W_gu[:, :I], leaf, g, out_dtype=X.dtype)
    up = gemm(X, W_gu[:, I:], leaf, g, out_dtype=X.dtype)
    return tb.tbik_silu_mul(gate, up), gate, up


# (M, I, K, leaf, k_first, route).  Routes: the epilogue needs a chip-filling number of 128-row tiles and no K split;
# few tiles split K; one round of 64-row tiles is neither.
ROUTES = [
    (1000, 1536, 1024, 128, 1, "epilogue"),        # 8 x 24 tiles, the last row tile ragged (104 rows)
    (1024, 1536, 1536, 128, 3, "epilogue"),        # full tiles only, k_first 3
    (40, 1024, 2048, 128, 1, "split"),
    (200, 512, 4096, 256, 1, "split"),
    (1000, 1024, 1024, 128, 1, "staged"),          # 16 x 16 tiles of 64 rows
    (1, 2048, 1024, 128, 1, "split"),
]


@pytest.mark.parametrize("M,I,K,leaf,g,route", ROUTES)
@pytest.mark.parametrize("fmt", ["bf16", "fp16"])
def test_gemm_swiglu_equals_two_gemms_then_the_activation(fmt, M, I, K, leaf, g, route):
    need = tb.gemm_swiglu_workspace_bytes(M, I, K, leaf, g)
    if route == "epilogue":
        assert need == 0
    elif route == "staged":
        assert 0 < need <= M * 2 * I * 2 + 256
    else:
        assert need >= 2 * M * 2 * I * 4
    Xb, Wb = syn.gemm_random(100 + M + I, M, K, 2 * I, fmt=fmt)
    X, W = DEV[fmt](Xb), DEV[fmt](Wb)
    act = tb.tbik_gemm_swiglu(X, W, leaf, g)
    want, _, _ = unfused(X, W, leaf, g)
    torch.cuda.synchronize()
    assert torch.equal(act.view(torch.int16), want.view(torch.int16)), (fmt, M, I, K, route)


@pytest.mark.parametrize("fmt", ["bf16", "fp16"])
def test_gemm_swiglu_against_the_oracle_on_exact_operands(fmt):
    """Leaf-sparse operands make gate and up exact whatever the order inside a leaf, so the oracle's GEMM gives the
    GPU's gate and up bit for bit and the activation is checked end to end, on a shape that takes the epilogue route
    (ragged last row tile) and on its first rows through the split route."""
    M, I, K, leaf = 900, 1536, 1024, 128
    Xb, Wb = syn.gemm_leaf_sparse(9, M, K, 2 * I, leaf, exp_spread=1 if fmt == "fp16" else 6, fmt=fmt)
    _, y16 = orc.gemm(Xb, Wb, leaf, 1, fmt=fmt)
    gate_b, up_b = np.ascontiguousarray(y16[:, :I]), np.ascontiguousarray(y16[:, I:])
    X, W = DEV[fmt](Xb), DEV[fmt](Wb)
    _, gate, up = unfused(X, W, leaf, 1)
    assert np.array_equal(bits(gate), gate_b) and np.array_equal(bits(up), up_b)
    want = orc.silu_mul(gate_b, up_b, fmt)
    act = tb.tbik_gemm_swiglu(X, W, leaf, 1)
    assert_act_close(bits(act), want, fmt, "epilogue")
    few = tb.tbik_gemm_swiglu(X[:24].contiguous(), W, leaf, 1)
    assert torch.equal(few.view(torch.int16), act[:24].view(torch.int16))       # M invariance across routes


def test_gemm_swiglu_full_size_rows_and_repetitions():
    """The 8B-class gate/up projection at the batch the benchmark times (M = 4096, K = 4096, I = 12288): one digest over
    three runs, and sampled rows equal what the same rows give on their own through the other routes."""
    M, I, K, leaf = 4096, 12288, 4096, 256
    g = torch.Generator(device="cuda:0")
    g.manual_seed(12)
    X = torch.randn((M, K), generator=g, device="cuda:0", dtype=torch.float32).to(torch.bfloat16)
    W = (torch.randn((K, 2 * I), generator=g, device="cuda:0", dtype=torch.float32) * 0.02).to(torch.bfloat16)
    assert tb.gemm_swiglu_workspace_bytes(M, I, K, leaf, 1) == 0
    act = tb.tbik_gemm_swiglu(X, W, leaf, 1)
    d = gu.digest(act)
    for _ in range(2):
        assert gu.digest(tb.tbik_gemm_swiglu(X, W, leaf, 1)) == d
    rows = [0, 1, 127, 128, 2047, 4095]
    sub = X[rows].contiguous()
    want, _, _ = unfused(sub, W, leaf, 1)
    assert torch.equal(act[rows].view(torch.int16), want.view(torch.int16))
    assert torch.equal(tb.tbik_gemm_swiglu(sub, W, leaf, 1).view(torch.int16), want.view(torch.int16))
    # the values are the activation of the products: fp64 on a few elements
    cols = [0, 5, 6143, 12287]
    Xs, Ws = sub.double(), W.double()
    gate64 = Xs @ Ws[:, cols]
    up64 = Xs @ Ws[:, [I + c for c in cols]]
    ref = (gate64 / (1 + torch.exp(-gate64)) * up64).cpu().numpy()
    got = act[rows][:, cols].double().cpu().numpy()
    assert np.all(np.abs(got - ref) <= 0.02 * np.abs(ref) + 2e-3)


def test_gemm_swiglu_argument_checks():
    X = torch.zeros((8, 256), dtype=torch.bfloat16, device="cuda:0")
    W = torch.zeros((256, 2 * 36), dtype=torch.bfloat16, device="cuda:0")
    with pytest.raises(tb.TbikError):
        tb.tbik_gemm_swiglu(X, W, 128, 1)                     # I = 36 is not a multiple of 8
    W = torch.zeros((256, 2 * 64), dtype=torch.bfloat16, device="cuda:0")
    need = tb.gemm_swiglu_workspace_bytes(8, 64, 256, 128, 1)
    assert need > 0
    small = torch.empty(256, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(tb.TbikError):
        tb.tbik_gemm_swiglu(X, W, 128, 1, workspace=small)
    assert tb.tbik_gemm_swiglu(X[:0], W, 128, 1).shape == (0, 64)
