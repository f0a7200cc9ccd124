"""Every entry point inside a HIP graph: capture one pass of the hot path, replay it several times with eager work and
synchronisations in between, and compare every replay with the eager result bit for bit.  (The library enqueues only
kernels -- no memsets, no allocations -- so a captured call replays as the same kernels on the same buffers.)"""
import numpy as np
import pytest
import torch

import gpu_util as gu
from paper_2511_17826_amd import binding as tb
from paper_2511_17826_amd import synthetic as syn

pytestmark = pytest.mark.gpu


def test_hot_path_in_a_hip_graph_replays_bit_identically():
    M, K, N, leaf = 96, 1024, 8200, 64                    # N: two blocks per row for the log-softmax, ragged last tile
    Xb, Wb = syn.gemm_random(21, M, K, N)
    xn_b, wn_b = syn.rmsnorm_inputs(M, K, seed=9)
    X, W, Wn = gu.dev_bf16(Xb), gu.dev_bf16(Wb), gu.dev_bf16(wn_b)
    dev = X.device
    xn = torch.empty_like(X)
    y = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
    parts = torch.empty((4, M, N), dtype=torch.float32, device=dev)
    yf = torch.empty((M, N), dtype=torch.float32, device=dev)
    lsm = torch.empty((M, N), dtype=torch.float32, device=dev)
    rsum = torch.empty((M,), dtype=torch.float32, device=dev)
    ws_g = torch.empty(max(256, tb.gemm_workspace_bytes(M, N, K, leaf, 1)), dtype=torch.uint8, device=dev)
    ws_r = torch.empty(max(256, int(tb.lib().tbik_row_reduce_workspace_bytes(M, N, tb.TBIK_LOGSOFTMAX))), dtype=torch.uint8,
                       device=dev)

    def one_pass():
        tb.tbik_rmsnorm(X, Wn, 1e-6, out=xn)
        tb.tbik_gemm(xn, W, leaf, 1, out=y, workspace=ws_g)
        tb.tbik_gemm_shard_partials(xn, W, leaf, 1, 4, out=parts, workspace=ws_g)
        tb.tbik_tree_combine(parts, out=yf)
        tb.tbik_row_reduce(yf, tb.TBIK_LOGSOFTMAX, out=lsm, workspace=ws_r)
        tb.tbik_row_reduce(yf, tb.TBIK_SUM, out=rsum, workspace=ws_r)

    one_pass()
    torch.cuda.synchronize()
    want = [t.clone() for t in (xn, y, yf, lsm, rsum)]

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            one_pass()
    for rep in range(4):
        for t in (xn, y, yf, lsm, rsum):
            t.zero_()                                      # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip((xn, y, yf, lsm, rsum), want):
            assert torch.equal(got.view(torch.uint8), ref.view(torch.uint8)), rep
