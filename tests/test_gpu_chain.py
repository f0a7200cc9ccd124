"""32B-class synthetic decoder-layer chain on one GPU: the final log-probabilities must be bit-identical for
P in {1,2,4,8} emulated shards of the two row-parallel layers (o_proj, down_proj).

RMSNorm -> QKV GEMM -> reference attention -> o_proj (tree GEMM, P shards) -> RMSNorm -> gate/up GEMM with SiLU*up ->
down_proj (tree GEMM, P shards) -> lm_head GEMM -> log-softmax, M = 512 tokens.  Column-parallel layers (qkv, gate, up,
lm_head) have no cross-shard sum, so they run as whole-K calls (Sec. 3.3).  leaf = 128 with k_first = 5 (K = 5120) and
25 (K = 25600) gives 8 superleaves, so P <= 8 is legal.  The attention here is a plain fp32 softmax(QK^T)V written with
torch ops: it is test scaffolding, computed once and fed to every P, not part of the library.

A second test runs the same layer with every reduction inside the library -- tbik_attention on the fused QKV buffer and
the fused tail after both row-parallel layers -- on two packed sequences, and checks the claim end to end: the final
log-probabilities of a token have the same bits for every shard count, with or without the other sequence in the
batch, and when the token is processed as a decode step against the cached keys and values.
"""
import numpy as np
import pytest
import torch

import gpu_util as gu
from oracle import tbik_oracle as orc
from paper_2511_17826_amd import binding as tb
from paper_2511_17826_amd import synthetic as syn

pytestmark = pytest.mark.gpu


def reference_attention(qkv: torch.Tensor) -> torch.Tensor:
    d = syn.CHAIN_DIMS
    T, hd, nq, nkv = qkv.shape[0], d["head_dim"], d["q_heads"], d["kv_heads"]
    q, k, v = qkv.float().split([nq * hd, nkv * hd, nkv * hd], dim=1)
    q = q.view(T, nq, hd).transpose(0, 1)
    k = k.view(T, nkv, hd).transpose(0, 1).repeat_interleave(nq // nkv, dim=0)
    v = v.view(T, nkv, hd).transpose(0, 1).repeat_interleave(nq // nkv, dim=0)
    s = torch.matmul(q, k.transpose(1, 2)) / hd ** 0.5
    s = s.masked_fill(torch.triu(torch.ones(T, T, dtype=torch.bool, device=qkv.device), 1), float("-inf"))
    o = torch.matmul(torch.softmax(s, dim=-1), v)
    return o.transpose(0, 1).reshape(T, nq * hd).to(torch.bfloat16).contiguous()


def row_parallel(x, w, leaf, g, P, out_dtype):
    if P == 1:
        return tb.tbik_gemm(x, w, leaf, g, out_dtype=out_dtype)
    return tb.tbik_tree_combine(tb.tbik_gemm_shard_partials(x, w, leaf, g, P), out_dtype=out_dtype)


def test_chain_logprobs_bit_identical_across_shard_counts():
    d = syn.CHAIN_DIMS
    leaf = d["leaf"]
    g_h = d["hidden"] // leaf // 8          # 5
    g_i = d["inter"] // leaf // 8           # 25
    t = syn.chain_tensors("cuda:0")
    n1 = tb.tbik_rmsnorm(t["x"], t["norm1"], 1e-6)
    qkv = tb.tbik_gemm(n1, t["w_qkv"], leaf, g_h)
    attn = reference_attention(qkv)
    w_gu = torch.cat([t["w_gate"], t["w_up"]], dim=1)          # [K, 2 I]: gate columns, then up columns

    digests, finals = {}, {}
    stages = {}
    for P in (1, 2, 4, 8):
        h1 = row_parallel(attn, t["w_o"], leaf, g_h, P, torch.bfloat16)
        n2 = tb.tbik_rmsnorm(h1, t["norm2"], 1e-6)
        act = tb.tbik_gemm_swiglu(n2, w_gu, leaf, g_h)
        if P == 1:      # the fused call is the two column-parallel GEMMs followed by the activation, bit for bit
            gate = tb.tbik_gemm(n2, t["w_gate"], leaf, g_h)
            up = tb.tbik_gemm(n2, t["w_up"], leaf, g_h)
            assert torch.equal(act.view(torch.int16), tb.tbik_silu_mul(gate, up).view(torch.int16))
            want = gate.float() / (1 + torch.exp(-gate.float())) * up.float()    # the definition, written out in fp32
            assert torch.all((act.float() - want).abs() <= want.abs() * 2.0 ** -7 + 1e-30)
            del gate, up, want
        h2 = row_parallel(act, t["w_down"], leaf, g_i, P, torch.bfloat16)
        logits = tb.tbik_gemm(h2, t["w_lm"], leaf, g_h, out_dtype=torch.float32)
        logp = tb.tbik_row_reduce(logits, tb.TBIK_LOGSOFTMAX)
        torch.cuda.synchronize()
        digests[P] = gu.digest(logp)
        if P == 1:
            stages = dict(h1=h1, act=act, h2=h2, logits=logits, logp=logp)
        else:
            assert torch.equal(h1.view(torch.int16), stages["h1"].view(torch.int16)), ("o_proj", P)
            assert torch.equal(h2.view(torch.int16), stages["h2"].view(torch.int16)), ("down_proj", P)
        del logits, logp
    assert len(set(digests.values())) == 1, digests

    # sampled oracle parity of the two row-parallel stages (fp32 route) and of the final log-softmax rows
    for name, x, w, g in [("o_proj", attn, t["w_o"], g_h), ("down_proj", stages["act"], t["w_down"], g_i)]:
        xb, wb = gu.host_bf16_bits(x), gu.host_bf16_bits(w)
        rows, cols = syn.sample_elements(5, x.shape[0], w.shape[1], 24, 48)
        y_gpu = gu.host_f32(row_parallel(x, w, leaf, g, 4, torch.float32))[rows, cols]
        y_orc = orc.gemm_elements(xb, wb, rows, cols, leaf, g)
        y64, A = gu.fp64_ref(xb, wb, rows, cols)
        gu.check_fp32_against_fp64(y_gpu, y64, A)
        assert np.all(np.abs(y_gpu.astype(np.float64) - y_orc) <= 2 * (leaf * g + 8) * 2.0 ** -24 * A), name
    lg = gu.host_f32(stages["logits"][[0, 255, 511]])
    want = orc.row_logsoftmax(lg)
    got = gu.host_f32(stages["logp"][[0, 255, 511]])
    assert np.max(np.abs(got - want) / np.maximum(1.0, np.abs(want))) <= 1e-5
    assert np.all(np.abs(np.exp(got.astype(np.float64)).sum(axis=1) - 1.0) <= 1e-5)


def _layer_logprobs(t, x, cu, max_q, P, kv_cache=None):
    """One decoder layer + lm_head on packed sequences, every reduction through the library:
    RMSNorm -> QKV GEMM -> tbik_attention on the fused QKV buffer -> o_proj shard partials -> fused tail (tree combine +
    residual + RMSNorm) -> gate/up GEMM with SiLU*up (tbik_gemm_swiglu) -> down_proj shard partials -> fused tail -> lm_head GEMM -> log-softmax.
    kv_cache = (K, V, cu_k): keys and values of the whole sequences (a decode step brings only its own queries)."""
    d = syn.CHAIN_DIMS
    leaf, hd, nq, nkv = d["leaf"], d["head_dim"], d["q_heads"], d["kv_heads"]
    g_h, g_i = d["hidden"] // leaf // 8, d["inter"] // leaf // 8
    T = x.shape[0]
    n1 = tb.tbik_rmsnorm(x, t["norm1"], 1e-6)
    qkv = tb.tbik_gemm(n1, t["w_qkv"], leaf, g_h)
    row = qkv.stride(0)
    Q = torch.as_strided(qkv, (T, nq, hd), (row, hd, 1), 0)
    K = torch.as_strided(qkv, (T, nkv, hd), (row, hd, 1), nq * hd)
    V = torch.as_strided(qkv, (T, nkv, hd), (row, hd, 1), (nq + nkv) * hd)
    cu_q = torch.from_numpy(np.asarray(cu, dtype=np.int32)).to("cuda:0")
    if kv_cache is None:
        attn = tb.tbik_attention(Q, K, V, cu_q, cu_q, max_q, hd ** -0.5, True)
    else:
        Kc, Vc, cu_k = kv_cache
        attn = tb.tbik_attention(Q, Kc, Vc, cu_q, torch.from_numpy(np.asarray(cu_k, dtype=np.int32)).to("cuda:0"), max_q,
                                 hd ** -0.5, True)
    attn = attn.view(T, nq * hd)
    h1, n2 = tb.tbik_combine_residual_rmsnorm(tb.tbik_gemm_shard_partials(attn, t["w_o"], leaf, g_h, P), x, t["norm2"], 1e-6)
    act = tb.tbik_gemm_swiglu(n2, t["w_gu"], leaf, g_h)       # position-wise after the GEMM: no reduction to order
    h2, n3 = tb.tbik_combine_residual_rmsnorm(tb.tbik_gemm_shard_partials(act, t["w_down"], leaf, g_i, P), h1, t["norm1"], 1e-6)
    logits = tb.tbik_gemm(n3, t["w_lm"], leaf, g_h, out_dtype=torch.float32)
    logp = tb.tbik_row_reduce(logits, tb.TBIK_LOGSOFTMAX)
    torch.cuda.synchronize()
    return logp, (K, V)


def test_layer_with_library_attention_is_invariant_to_batch_shards_and_call_shape():
    """The paper's claim end to end (Sec. 1: the same bits across batch sizes and tensor-parallel sizes; implementation
    appendix: prefill and decode through one attention kernel): two packed sequences of 300 and 212 tokens.
      (1) P in {1, 2, 4, 8}: one digest of the final log-probabilities;
      (2) each sequence run on its own gives the rows it has in the batch;
      (3) the last token of the second sequence run as a decode step (one query, keys and values from the cache of the
          batched run) gives the row it has in the batch."""
    t = syn.chain_tensors("cuda:0")
    t["w_gu"] = torch.cat([t.pop("w_gate"), t.pop("w_up")], dim=1)
    x = t["x"]
    cu = [0, 300, 512]
    full, (K, V) = _layer_logprobs(t, x, cu, 300, 1)
    for P in (2, 4, 8):
        other, _ = _layer_logprobs(t, x, cu, 300, P)
        assert torch.equal(other.view(torch.int32), full.view(torch.int32)), P
        del other
    a, _ = _layer_logprobs(t, x[:300].contiguous(), [0, 300], 300, 2)
    assert torch.equal(a.view(torch.int32), full[:300].view(torch.int32))
    b, _ = _layer_logprobs(t, x[300:].contiguous(), [0, 212], 212, 4)
    assert torch.equal(b.view(torch.int32), full[300:].view(torch.int32))
    del a, b
    step, _ = _layer_logprobs(t, x[511:512].contiguous(), [0, 1], 1, 8, kv_cache=(K[300:], V[300:], [0, 212]))
    assert torch.equal(step.view(torch.int32), full[511:512].view(torch.int32))
    # and the numbers are log-probabilities
    got = gu.host_f32(full[[0, 299, 511]])
    assert np.all(np.abs(np.exp(got.astype(np.float64)).sum(axis=1) - 1.0) <= 1e-5)
