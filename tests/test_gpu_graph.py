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


def test_fp32_gemm_fp16_tail_and_attention_in_a_hip_graph():
    """The later entry points (fp32 GEMM with its K split, fp16 fused tail, fp16 attention, attention over several splits
    of the key axis with its workspace) under capture and replay."""
    dev = "cuda:0"
    M, K, N = 70, 2048, 512
    Xf, Wf = syn.gemm_random_f32(31, M, K, N)
    X32, W32 = gu.dev_f32(Xf), gu.dev_f32(Wf)
    y32 = torch.empty((M, N), dtype=torch.float32, device=dev)
    parts = torch.empty((4, M, N), dtype=torch.float32, device=dev)
    ws = torch.empty(max(256, tb.gemm_workspace_bytes(M, N, K, 128, 1)), dtype=torch.uint8, device=dev)
    res_b, w_b = syn.rmsnorm_inputs(M, N, seed=5, fmt="fp16")
    res, wn = gu.dev_f16(res_b), gu.dev_f16(w_b)
    hid, nrm = torch.empty_like(res), torch.empty_like(res)
    a = syn.attention_inputs(32, [200, 1, 40], [200, 300, 90], Hq=8, Hkv=2, D=128, fmt="fp16")
    Q, Kk, V = gu.dev_f16(a["Q"]), gu.dev_f16(a["K"]), gu.dev_f16(a["V"])
    cu_q = torch.from_numpy(a["cu_q"]).to(dev)
    cu_k = torch.from_numpy(a["cu_k"]).to(dev)
    O = torch.empty_like(Q)
    # a decode step over three splits of the key axis (one workgroup per split, then the fold kernel; states in `ws_a`)
    al = syn.attention_inputs(33, [1], [9000], Hq=8, Hkv=2, D=128)
    Ql, Kl, Vl = gu.dev_bf16(al["Q"]), gu.dev_bf16(al["K"]), gu.dev_bf16(al["V"])
    cu_ql, cu_kl = torch.from_numpy(al["cu_q"]).to(dev), torch.from_numpy(al["cu_k"]).to(dev)
    Ol = torch.empty_like(Ql)
    ws_a = torch.empty(tb.attention_workspace_bytes(1, 1, 9000, 8, 2), dtype=torch.uint8, device=dev)

    def one_pass():
        tb.tbik_attention(Ql, Kl, Vl, cu_ql, cu_kl, 1, al["scale"], True, out=Ol, max_seqlen_k=9000, workspace=ws_a)
        tb.tbik_gemm_f32(X32, W32, 128, 1, out=y32, workspace=ws)
        tb.tbik_gemm_shard_partials_f32(X32, W32, 128, 1, 4, out=parts, workspace=ws)
        tb.tbik_combine_residual_rmsnorm_f16(parts, res, wn, 1e-6, hidden=hid, normed=nrm)
        tb.tbik_attention_f16(Q, Kk, V, cu_q, cu_k, 200, a["scale"], True, out=O, max_seqlen_k=300)   # given: reading it from the device would synchronise

    one_pass()
    torch.cuda.synchronize()
    outs = (y32, parts, hid, nrm, O, Ol)
    want = [t.clone() for t in outs]
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            one_pass()
    for rep in range(3):
        for t in outs + (ws_a,):
            t.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip(outs, want):
            assert torch.equal(got.view(torch.uint8), ref.view(torch.uint8)), rep


def test_8_bit_and_microscaling_gemms_in_a_hip_graph():
    """The 8-bit GEMM and the three microscaling ones (which re-tile their scales in a launch of their own from 128 rows
    on, into the caller's workspace) under capture and replay: a shape with the K cut and one without."""
    dev = "cuda:0"
    u8 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint8)).to(dev)
    cases = []
    for M, K, N, leaf in ((200, 2048, 264, 256), (40, 1024, 136, 128)):
        X8, Xs8, W8, Ws8 = [u8(a) for a in syn.gemm_random_mxfp8(M, M, K, N, scale_spread=1)]
        X6, Xs6, W6, Ws6 = [u8(a) for a in syn.gemm_random_mxfp6(M + 1, M, K, N, fmt="e3m2", scale_spread=1)]
        X4, Xs4, W4, Ws4 = [u8(a) for a in syn.gemm_random_mxfp4(M + 2, M, K, max(N, 256) if leaf == 256 else N, scale_spread=1)]
        outs = [torch.empty((M, W.shape[0]), dtype=torch.float32, device=dev) for W in (W8, W8, W6, W4)]
        ws = [torch.empty(max(256, n), dtype=torch.uint8, device=dev) for n in (
            tb.gemm_fp8_workspace_bytes(M, N, K, leaf, 1), tb.gemm_mxfp8_workspace_bytes(M, N, K, leaf, 1),
            tb.gemm_mxfp6_workspace_bytes(M, N, K, leaf, 1), tb.gemm_mxfp4_workspace_bytes(M, W4.shape[0], K, max(leaf, 256), 1))]
        cases.append((leaf, (X8, Xs8, W8, Ws8), (X6, Xs6, W6, Ws6), (X4, Xs4, W4, Ws4), outs, ws))

    def one_pass():
        for leaf, m8, m6, m4, outs, ws in cases:
            tb.tbik_gemm_fp8(m8[0], m8[2], leaf, 1, "e4m3", out=outs[0], workspace=ws[0])
            tb.tbik_gemm_mxfp8(*m8, leaf, 1, "e4m3", out=outs[1], workspace=ws[1])
            tb.tbik_gemm_mxfp6(*m6, leaf, 1, "e3m2", out=outs[2], workspace=ws[2])
            tb.tbik_gemm_mxfp4(*m4, max(leaf, 256), 1, out=outs[3], workspace=ws[3])

    one_pass()
    torch.cuda.synchronize()
    tensors = [t for c in cases for t in c[4]]
    want = [t.clone() for t in tensors]
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            one_pass()
    for rep in range(3):
        for t in tensors:
            t.zero_()
        for c in cases:
            for w in c[5]:
                w.fill_(0xA5)                              # the workspaces' old contents do not matter
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip(tensors, want):
            assert torch.equal(got.view(torch.uint8), ref.view(torch.uint8)), rep
