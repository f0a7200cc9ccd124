"""GPU parity and invariance tests of the tree-ordered row reductions (through the C ABI).

Bars: RMSNorm, row sum and row max are bit-exact against the oracle (all their arithmetic is IEEE fp32
in a fixed order).  Log-softmax uses the device's exp/log, so it is checked within
|o_gpu - o_oracle| <= 1e-5 * max(1, |o|); GPU against GPU (any M, any row position) is always 0 bits.
"""
import numpy as np
import pytest
import torch

import gpu_util as gu
from oracle import tbik_oracle as orc
from paper_2511_17826_amd import binding as tb
from paper_2511_17826_amd import synthetic as syn

pytestmark = pytest.mark.gpu


# ----------------------------------------------------------------------------- RMSNorm

@pytest.mark.parametrize("H", [4096, 5120, 24, 1000, 8192])
def test_rmsnorm_bit_exact_and_batch_invariant(H):
    Mmax = 8192 if H in (4096, 5120) else 300
    x, w = syn.rmsnorm_inputs(Mmax, H)
    xd, wd = gu.dev_bf16(x), gu.dev_bf16(w)
    full = tb.tbik_rmsnorm(xd, wd, 1e-6)
    torch.cuda.synchronize()
    n_check = min(Mmax, 1024)
    want = orc.rmsnorm(x[:n_check], w, 1e-6)
    assert np.array_equal(gu.host_bf16_bits(full[:n_check]), want)
    want_tail = orc.rmsnorm(x[-64:], w, 1e-6)
    assert np.array_equal(gu.host_bf16_bits(full[-64:]), want_tail)
    for M in (1, 2, 3, 7, 16, 64, 255, 256, 1024, 4096, 8192):
        if M > Mmax:
            continue
        y = tb.tbik_rmsnorm(xd[:M].contiguous(), wd, 1e-6)
        assert torch.equal(y.view(torch.int16), full[:M].view(torch.int16)), M
    # shifted position: rows 100..163 run as their own batch
    if Mmax >= 200:
        y = tb.tbik_rmsnorm(xd[100:164].contiguous(), wd, 1e-6)
        assert torch.equal(y.view(torch.int16), full[100:164].view(torch.int16))


def test_rmsnorm_closed_form():
    H = 4096
    x = syn.f32_to_bf16_bits(np.ones((5, H), dtype=np.float32))
    w = syn.f32_to_bf16_bits(np.ones(H, dtype=np.float32))
    y = gu.host_bf16_bits(tb.tbik_rmsnorm(gu.dev_bf16(x), gu.dev_bf16(w), 1e-6))
    r = np.float32(1.0) / np.sqrt(np.float32(1.0) + np.float32(1e-6), dtype=np.float32)
    assert np.all(y == syn.f32_to_bf16_bits(np.array([r]))[0])


# ----------------------------------------------------------------------------- sum / max

@pytest.mark.parametrize("V", [4, 1024, 8192, 8196, 151936, 300000])
def test_row_sum_and_max_bit_exact(V):
    M = 9
    rng = np.random.default_rng(V)
    x = (rng.standard_normal((M, V)) * np.exp2(rng.integers(-6, 7, (M, V)))).astype(np.float32)
    xd = gu.dev_f32(x)
    s = gu.host_f32(tb.tbik_row_reduce(xd, tb.TBIK_SUM))
    assert np.array_equal(gu.u32(s), gu.u32(orc.row_sum(x, orc.LEAF_F32)))
    m = gu.host_f32(tb.tbik_row_reduce(xd, tb.TBIK_MAX))
    assert np.array_equal(m, x.max(axis=1))
    # batch invariance
    s1 = gu.host_f32(tb.tbik_row_reduce(xd[4:5].contiguous(), tb.TBIK_SUM))
    assert gu.u32(s1)[0] == gu.u32(s)[4]


def test_row_sum_bf16_input_bit_exact():
    M, V = 5, 20000
    xb = syn.normal_bf16(np.random.Generator(np.random.PCG64(1)), (M, V), 2.0)
    s = gu.host_f32(tb.tbik_row_reduce(gu.dev_bf16(xb), tb.TBIK_SUM))
    want = orc.row_sum(syn.bf16_bits_to_f32(xb), orc.LEAF_BF16)
    assert np.array_equal(gu.u32(s), gu.u32(want))


def test_row_sum_hand_value():
    """Leaves [1,0,0,0 | t,t,0,0 | ...]: (1) + (2^-23) at the first tree level = 1 + 2^-23; strict left-to-right gives 1."""
    t = 2.0 ** -24
    x = np.zeros((1, 16), dtype=np.float32)
    x[0, 0], x[0, 4], x[0, 5] = 1.0, t, t
    s = gu.host_f32(tb.tbik_row_reduce(gu.dev_f32(x), tb.TBIK_SUM))
    assert int(gu.u32(s)[0]) == 0x3F800001
    x2 = np.zeros((1, 16), dtype=np.float32)
    x2[0, 0], x2[0, 1], x2[0, 2] = 1.0, t, t        # same leaf: sequential inside the leaf -> ties -> 1.0
    s2 = gu.host_f32(tb.tbik_row_reduce(gu.dev_f32(x2), tb.TBIK_SUM))
    assert int(gu.u32(s2)[0]) == 0x3F800000


# ----------------------------------------------------------------------------- log-softmax

def test_logsoftmax_parity_and_invariance():
    V = 151936
    x = syn.logits_f32(64, V)
    xd = gu.dev_f32(x)
    full = tb.tbik_row_reduce(xd, tb.TBIK_LOGSOFTMAX)
    torch.cuda.synchronize()
    o = gu.host_f32(full)
    want = orc.row_logsoftmax(x[:16], orc.LEAF_F32)
    assert np.max(np.abs(o[:16] - want) / np.maximum(1.0, np.abs(want))) <= 1e-5
    assert np.all(np.abs(np.exp(o.astype(np.float64)).sum(axis=1) - 1.0) <= 1e-5)
    for (a, b) in [(0, 1), (5, 6), (0, 64), (17, 40)]:
        y = tb.tbik_row_reduce(xd[a:b].contiguous(), tb.TBIK_LOGSOFTMAX)
        assert torch.equal(y.view(torch.int32), full[a:b].view(torch.int32)), (a, b)
    # twice the same call: same bits
    again = tb.tbik_row_reduce(xd, tb.TBIK_LOGSOFTMAX)
    assert torch.equal(again.view(torch.int32), full.view(torch.int32))


def test_logsoftmax_constant_row_and_small_V():
    for V in (4, 1024, 4096):
        x = np.full((3, V), 1.25, dtype=np.float32)
        o = gu.host_f32(tb.tbik_row_reduce(gu.dev_f32(x), tb.TBIK_LOGSOFTMAX))
        assert np.max(np.abs(o + np.log(V))) <= 1e-5 * max(1.0, np.log(V))
    x = syn.logits_f32(7, 4096)
    o = gu.host_f32(tb.tbik_row_reduce(gu.dev_f32(x), tb.TBIK_LOGSOFTMAX))
    want = orc.row_logsoftmax(x)
    assert np.max(np.abs(o - want) / np.maximum(1.0, np.abs(want))) <= 1e-5


@pytest.mark.parametrize("V", [8192, 8196])
def test_logsoftmax_one_block_and_two_block_rows(V):
    """V = 8192 is the longest fp32 row that one block holds (read once, kept in registers); V = 8196 takes the
    general path with two blocks.  Both: oracle parity, sum of exp = 1, and a row's bits do not depend on the batch."""
    x = syn.logits_f32(9, V, seed=11)
    xd = gu.dev_f32(x)
    full = tb.tbik_row_reduce(xd, tb.TBIK_LOGSOFTMAX)
    o = gu.host_f32(full)
    want = orc.row_logsoftmax(x, orc.LEAF_F32)
    assert np.max(np.abs(o - want) / np.maximum(1.0, np.abs(want))) <= 1e-5
    assert np.all(np.abs(np.exp(o.astype(np.float64)).sum(axis=1) - 1.0) <= 1e-5)
    for (a, b) in [(0, 1), (8, 9), (3, 7)]:
        y = tb.tbik_row_reduce(xd[a:b].contiguous(), tb.TBIK_LOGSOFTMAX)
        assert torch.equal(y.view(torch.int32), full[a:b].view(torch.int32)), (a, b)


def test_logsoftmax_bounded_wait_runs_out_same_bits():
    """Long rows: the workgroups of a row wait for each other a bounded number of polls.  With the bound forced to 0
    from the host the waits run out and the workgroups finish their blocks alone, walking the row themselves: the bits
    must be those of the normal run (two implementations of the same arithmetic), and every kernel exits normally."""
    V = 151936
    x = syn.logits_f32(24, V, seed=5)
    xd = gu.dev_f32(x)
    normal = tb.tbik_row_reduce(xd, tb.TBIK_LOGSOFTMAX)
    torch.cuda.synchronize()
    prev = tb.tbik_set_row_wait_limit(0)
    try:
        forced = tb.tbik_row_reduce(xd, tb.TBIK_LOGSOFTMAX)
        torch.cuda.synchronize()
    finally:
        tb.tbik_set_row_wait_limit(prev)
    assert prev > 0
    assert torch.equal(forced.view(torch.int32), normal.view(torch.int32))
    xb = syn.normal_bf16(np.random.Generator(np.random.PCG64(2)), (6, 40000), 3.0)
    xbd = gu.dev_bf16(xb)
    normal = tb.tbik_row_reduce(xbd, tb.TBIK_LOGSOFTMAX)
    prev = tb.tbik_set_row_wait_limit(0)
    try:
        forced = tb.tbik_row_reduce(xbd, tb.TBIK_LOGSOFTMAX)
        torch.cuda.synchronize()
    finally:
        tb.tbik_set_row_wait_limit(prev)
    assert torch.equal(forced.view(torch.int32), normal.view(torch.int32))
    want = orc.row_logsoftmax(syn.bf16_bits_to_f32(xb), orc.LEAF_BF16)
    o = gu.host_f32(normal)
    assert np.max(np.abs(o - want) / np.maximum(1.0, np.abs(want))) <= 1e-5


@pytest.mark.parametrize("fmt,M,V", [("f32", 130, 151936), ("bf16", 450, 80008), ("fp16", 700, 40000)])
def test_logsoftmax_pipelined_launch_equals_row_by_row_and_survives_a_zero_wait(fmt, M, V):
    """Launches of two or more rounds of resident workgroups take the pipelined kernel (a workgroup walks several
    blocks, three of them in flight).  Its rows must have the bits of the same rows computed a few at a time (the
    one-block-per-workgroup kernel), must agree with the oracle, and with the wait bound forced to 0 from the host
    (every hand-off gets one look, most workgroups finish their blocks alone) the call must still end normally with
    the same bits."""
    rng = np.random.Generator(np.random.PCG64(M + V))
    if fmt == "f32":
        x = syn.logits_f32(M, V, seed=M)
        xd = gu.dev_f32(x)
        x32, leaf = x, orc.LEAF_F32
    else:
        xb = syn.to_storage(rng.standard_normal((M, V)).astype(np.float32) * 3.0, fmt)
        xd = gu.dev_bf16(xb) if fmt == "bf16" else gu.dev_f16(xb)
        x32, leaf = syn.from_storage(xb, fmt), orc.LEAF_BF16
    full = tb.tbik_row_reduce(xd, tb.TBIK_LOGSOFTMAX)
    torch.cuda.synchronize()
    for a in range(0, M, 37):
        b = min(M, a + 37)
        y = tb.tbik_row_reduce(xd[a:b].contiguous(), tb.TBIK_LOGSOFTMAX)
        assert torch.equal(y.view(torch.int32), full[a:b].view(torch.int32)), (a, b)
    rows = [0, M // 2, M - 1]
    want = orc.row_logsoftmax(x32[rows], leaf)
    got = gu.host_f32(full[rows])
    assert np.max(np.abs(got - want) / np.maximum(1.0, np.abs(want))) <= 1e-5
    prev = tb.tbik_set_row_wait_limit(0)
    try:
        forced = tb.tbik_row_reduce(xd, tb.TBIK_LOGSOFTMAX)
        torch.cuda.synchronize()
    finally:
        tb.tbik_set_row_wait_limit(prev)
    assert torch.equal(forced.view(torch.int32), full.view(torch.int32))


def test_logsoftmax_two_streams_at_once_same_bits():
    """Two pipelined launches on two streams compete for the compute units, so neither may have all its workgroups
    resident: hand-offs can then run out and workgroups finish blocks alone.  Whatever the interleaving, both calls
    must end and give the bits of the calls run one after the other."""
    V = 151936
    g = torch.Generator(device="cuda")
    g.manual_seed(11)
    xs = [torch.randn((192, V), generator=g, device="cuda") * 3.0 for _ in range(2)]
    need = int(tb.lib().tbik_row_reduce_workspace_bytes(192, V, tb.TBIK_LOGSOFTMAX))
    want = [tb.tbik_row_reduce(x, tb.TBIK_LOGSOFTMAX) for x in xs]
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream() for _ in range(2)]
    wss = [torch.empty(need, dtype=torch.uint8, device="cuda:0") for _ in range(2)]
    outs = [torch.empty_like(w) for w in want]
    for rep in range(3):
        for i in range(2):
            outs[i].fill_(float("nan"))
        torch.cuda.synchronize()
        for i in range(2):
            with torch.cuda.stream(streams[i]):
                tb.tbik_row_reduce(xs[i], tb.TBIK_LOGSOFTMAX, out=outs[i], workspace=wss[i])
        torch.cuda.synchronize()
        for i in range(2):
            assert torch.equal(outs[i].view(torch.int32), want[i].view(torch.int32)), (rep, i)


def test_logsoftmax_long_rows_repeatable_under_load():
    """The workgroups of a long row hand their maxima and sums to each other through memory, across chiplets: with
    all compute units busy (512 rows), repeated runs and runs on slices of the batch must keep giving the same bits."""
    V = 151936
    g = torch.Generator(device="cuda")
    g.manual_seed(7)
    x = torch.randn((512, V), generator=g, device="cuda") * 3.0
    full = tb.tbik_row_reduce(x, tb.TBIK_LOGSOFTMAX)
    for _ in range(25):
        again = tb.tbik_row_reduce(x, tb.TBIK_LOGSOFTMAX)
        assert torch.equal(again.view(torch.int32), full.view(torch.int32))
    for (a, b) in [(0, 1), (17, 40), (100, 300), (511, 512), (3, 260)]:
        for _ in range(3):
            y = tb.tbik_row_reduce(x[a:b].contiguous(), tb.TBIK_LOGSOFTMAX)
            assert torch.equal(y.view(torch.int32), full[a:b].view(torch.int32)), (a, b)


def test_logsoftmax_finds_no_stale_value_in_a_poisoned_workspace():
    """The published block maxima and sums sit in the caller's workspace, which keeps the last call's contents.  Every
    call first sets its slots to a "not yet" pattern, and a slot counts as written once it holds anything else -- so
    whatever the workspace held before must be gone by then.  Here that is, in turn, NaN (every byte 0xff) and a
    plausible finite number (every byte 0x42: 48.56), which as a stale block maximum or sum would change the result."""
    V = 151936
    x = gu.dev_f32(syn.logits_f32(256, V, seed=9))
    need = int(tb.lib().tbik_row_reduce_workspace_bytes(256, V, tb.TBIK_LOGSOFTMAX))
    ws = torch.empty(need, dtype=torch.uint8, device="cuda:0")
    want = tb.tbik_row_reduce(x, tb.TBIK_LOGSOFTMAX)
    out = torch.empty_like(want)
    for rep in range(20):
        ws.fill_(0xff if rep % 2 == 0 else 0x42)
        tb.tbik_row_reduce(x, tb.TBIK_LOGSOFTMAX, out=out, workspace=ws)
        assert not bool(torch.isnan(out).any()), rep
        assert torch.equal(out.view(torch.int32), want.view(torch.int32)), rep


def test_logsoftmax_512_rows_sampled():
    """The full 512 x 151936 case in the launch shape the benchmark times; rows sampled for the oracle."""
    V = 151936
    x = syn.logits_f32(512, V)
    xd = gu.dev_f32(x)
    o = tb.tbik_row_reduce(xd, tb.TBIK_LOGSOFTMAX)
    torch.cuda.synchronize()
    rows = [0, 63, 200, 511]
    want = orc.row_logsoftmax(x[rows])
    got = gu.host_f32(o[rows])
    assert np.max(np.abs(got - want) / np.maximum(1.0, np.abs(want))) <= 1e-5
    one = tb.tbik_row_reduce(xd[200:201].contiguous(), tb.TBIK_LOGSOFTMAX)
    assert torch.equal(one.view(torch.int32), o[200:201].view(torch.int32))


# ----------------------------------------------------------------------------- fused tail: combine + residual + RMSNorm

@pytest.mark.parametrize("P,M,H", [(1, 5, 4096), (2, 33, 5120), (4, 64, 4096), (8, 7, 24), (16, 3, 1000), (8, 130, 8192),
                                   (8, 1100, 4096), (8, 2100, 4096)])   # the last one: more than 192 MiB of partials, read with streaming loads
def test_fused_tail_equals_the_three_steps_and_the_oracle(P, M, H):
    """tbik_combine_residual_rmsnorm against (a) tbik_tree_combine -> bf16 add -> tbik_rmsnorm on the GPU and (b) the
    oracle's step-by-step definition: bit for bit, also when the hidden state is updated in place."""
    rng = np.random.Generator(np.random.PCG64(100 + P + H))
    parts = (rng.standard_normal((P, M, H), dtype=np.float32) * np.float32(1.0 / np.sqrt(P)))
    res_b = syn.normal_bf16(rng, (M, H), 1.0)
    w_b = syn.normal_bf16(rng, (H,), 0.1, mean=1.0)
    pd = torch.from_numpy(parts).to("cuda:0")
    rd, wd = gu.dev_bf16(res_b), gu.dev_bf16(w_b)

    hid, out = tb.tbik_combine_residual_rmsnorm(pd, rd, wd, 1e-6)
    y = tb.tbik_tree_combine(pd, out_dtype=torch.bfloat16)
    hid3 = (y.float() + rd.float()).to(torch.bfloat16)                  # fp32 add, one RNE rounding
    out3 = tb.tbik_rmsnorm(hid3, wd, 1e-6)
    assert torch.equal(hid.view(torch.int16), hid3.view(torch.int16))
    assert torch.equal(out.view(torch.int16), out3.view(torch.int16))

    if M * H <= 300000:
        hid_o, out_o = orc.combine_residual_rmsnorm(parts, res_b, w_b, 1e-6)
        assert np.array_equal(gu.host_bf16_bits(hid), hid_o)
        assert np.array_equal(gu.host_bf16_bits(out), out_o)

    inplace = rd.clone()
    hid2, out2 = tb.tbik_combine_residual_rmsnorm(pd, inplace, wd, 1e-6, hidden=inplace)
    assert hid2.data_ptr() == inplace.data_ptr()
    assert torch.equal(inplace.view(torch.int16), hid.view(torch.int16))
    assert torch.equal(out2.view(torch.int16), out.view(torch.int16))
    # a row alone gives the same bits
    h1, o1 = tb.tbik_combine_residual_rmsnorm(pd[:, M - 1:M].contiguous(), rd[M - 1:M].contiguous(), wd, 1e-6)
    assert torch.equal(o1.view(torch.int16), out[M - 1:M].view(torch.int16))


def test_fused_tail_hand_value():
    H = 8
    parts = np.zeros((2, 1, H), dtype=np.float32)
    parts[0, 0, :] = 1.0
    parts[1, 0, :] = 2.0 ** -8 + 2.0 ** -12
    res = np.full((1, H), 0x3B80, dtype=np.uint16)
    w = np.full((H,), 0x3F80, dtype=np.uint16)
    hid, out = tb.tbik_combine_residual_rmsnorm(torch.from_numpy(parts).to("cuda:0"), gu.dev_bf16(res), gu.dev_bf16(w), 0.0)
    assert np.all(gu.host_bf16_bits(hid) == 0x3F82)
    assert np.all(gu.host_bf16_bits(out) == 0x3F80)


@pytest.mark.parametrize("P", [1, 2, 4, 8, 16])
@pytest.mark.parametrize("n", [4096 * 33, 1001, 3])
def test_tree_allreduce_round_by_round_is_alg2(P, n):
    """App. D.2 taken literally: after the reduce and broadcast rounds every rank's buffer holds the oracle's all-reduced
    tensor bit for bit -- which is what tbik_tree_combine computes in one pass."""
    rng = np.random.default_rng(P * 1000 + n)
    bufs = (rng.standard_normal((P, n)) * np.exp2(rng.integers(-12, 13, size=(P, n)))).astype(np.float32)
    want = orc.allreduce(bufs)
    d = gu.dev_f32(bufs)
    combined = tb.tbik_tree_combine(d.view(P, 1, n).clone(), out_dtype=torch.float32) if P > 1 else d.clone().view(1, n)
    got = gu.host_f32(tb.tbik_tree_allreduce(d))
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    for r in range(P):
        assert np.array_equal(got[r].view(np.uint32), want[0].view(np.uint32)), r
    assert np.array_equal(gu.host_f32(combined).reshape(-1).view(np.uint32), want[0].view(np.uint32))
