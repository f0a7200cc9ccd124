"""GPU test of tbik_row_reduce_static: the row reductions on the library's own fixed scratch array, for callers that
cannot allocate.  Its results must be those of tbik_row_reduce bit for bit (same kernels, another scratch), call after
call on the one shared array -- the second call of each pair is smaller, so it finds the first call's leftovers in
the scratch -- and the log-softmax must also meet the oracle at the bar of the reductions test.
"""
import ctypes as C

import numpy as np
import pytest
import torch

import gpu_util as gu
from oracle import tbik_oracle as orc
from paper_2511_17826_amd import binding as tb

pytestmark = pytest.mark.gpu

STATIC_BYTES = 4 << 20


def logits(M, V, seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    return (rng.standard_normal((M, V)) * 3.0).astype(np.float32)


def call_static(xd, op, out):
    """Straight through the C ABI: device pointers and sizes only, no workspace, the caller's output buffer."""
    M, V = xd.shape
    st = tb.lib().tbik_row_reduce_static(xd.data_ptr(), tb.TBIK_F32, out.data_ptr(), op, M, V,
                                         torch.cuda.current_stream().cuda_stream)
    assert st == tb.OK, tb.lib().tbik_status_string(st)
    return out


@pytest.mark.parametrize("V", [151936, 4096])
def test_static_scratch_matches_workspace_entry_point_twice_in_a_row(V):
    # two calls in a row, the second with fewer rows (and other data): long rows take the cooperative kernel,
    # whose counters and published values live in the scratch
    for M, seed in ((37, 5), (3, 6)):
        x = logits(M, V, seed)
        xd = gu.dev_f32(x)
        for op in (tb.TBIK_LOGSOFTMAX, tb.TBIK_SUM, tb.TBIK_MAX):
            want = tb.tbik_row_reduce(xd, op)
            got = torch.full_like(want, float("nan"))
            before = torch.cuda.memory_allocated()
            call_static(xd, op, got)
            torch.cuda.synchronize()
            assert torch.cuda.memory_allocated() == before
            assert torch.equal(got.view(torch.int32), want.view(torch.int32)), (M, V, op)
        # and against the oracle, at the bars of the reductions test
        o = gu.host_f32(call_static(xd, tb.TBIK_LOGSOFTMAX, torch.empty((M, V), dtype=torch.float32, device="cuda:0")))
        ref = orc.row_logsoftmax(x, orc.LEAF_F32)
        assert np.all(np.abs(o - ref) <= 1e-5 * np.maximum(1.0, np.abs(ref)))
        s = gu.host_f32(call_static(xd, tb.TBIK_SUM, torch.empty(M, dtype=torch.float32, device="cuda:0")))
        assert np.array_equal(gu.u32(s), gu.u32(orc.row_sum(x, orc.LEAF_F32)))


def test_static_scratch_with_the_pipelined_launch_then_a_small_one():
    # 120 rows of 19 blocks are more than two rounds of resident workgroups: the pipelined log-softmax kernel, whose
    # slots and flags live in the scratch as well; then a small call on the same scratch
    V = 151936
    for M, seed in ((120, 8), (5, 9)):
        xd = gu.dev_f32(logits(M, V, seed))
        want = tb.tbik_row_reduce(xd, tb.TBIK_LOGSOFTMAX)
        got = torch.full_like(want, float("nan"))
        before = torch.cuda.memory_allocated()
        call_static(xd, tb.TBIK_LOGSOFTMAX, got)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert torch.equal(got.view(torch.int32), want.view(torch.int32)), M


def test_static_scratch_limit_and_setup_call():
    L = tb.lib()
    x = torch.zeros((1, 8), dtype=torch.float32, device="cuda:0")
    out = torch.zeros(8, dtype=torch.float32, device="cuda:0")
    # M == 0: set-up only
    assert L.tbik_row_reduce_static(x.data_ptr(), tb.TBIK_F32, out.data_ptr(), tb.TBIK_LOGSOFTMAX, 0, 8, None) == tb.OK
    # a shape whose scratch need exceeds the array is refused before anything runs (pointers are never touched)
    M, V = 20000, 151936
    assert L.tbik_row_reduce_workspace_bytes(M, V, tb.TBIK_LOGSOFTMAX) > STATIC_BYTES
    st = L.tbik_row_reduce_static(x.data_ptr(), tb.TBIK_F32, out.data_ptr(), tb.TBIK_LOGSOFTMAX, M, V, None)
    assert st == 6                      # TBIK_ERR_WORKSPACE
    assert L.tbik_row_reduce_static(None, tb.TBIK_F32, out.data_ptr(), tb.TBIK_SUM, 1, 8, None) == 1      # TBIK_ERR_NULL
    assert L.tbik_row_reduce_static(x.data_ptr(), tb.TBIK_F32, out.data_ptr(), tb.TBIK_SUM, 1, 6, None) == 2   # TBIK_ERR_SHAPE
