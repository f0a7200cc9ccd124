"""GPU parity and invariance tests of the tree-ordered GEMM (all calls go through the C ABI).

Bars (stated up front):
  * GPU vs GPU (any M, row position, P, kernel variant, repetition): 0 bits.
  * Tree between superleaves: bit-exact against the oracle on inputs whose superleaf sums are exact
    (hand-derived pins, leaf-sparse operands, small integers).
  * fp32 outputs on random data: |y_gpu - y_fp64| <= 1e-5 * sum_k |x_k w_k| per element, and relative
    error <= 1e-3 where |y| >= 0.01 * sum|x w|; additionally |y_gpu - y_oracle| <= 2*gamma_{leaf*k_first}*sum|x w|
    (only the order inside a superleaf differs: the MFMA's own, against the oracle's strict left-to-right).
  * bf16 outputs: equal to bf16(oracle) except within |gpu-oracle| + 1 ulp of a rounding boundary.
"""
import numpy as np
import pytest
import torch

import gpu_util as gu
from conftest import read_tree_pins
from oracle import tbik_oracle as orc
from paper_2511_17826_amd import binding as tb
from paper_2511_17826_amd import synthetic as syn

pytestmark = pytest.mark.gpu

VARIANTS = [tb.VARIANT_REFERENCE, tb.VARIANT_T128, tb.VARIANT_T32, tb.VARIANT_T64]


@pytest.fixture(autouse=True)
def _reset_variant():
    yield
    tb.tbik_set_gemm_variant(tb.VARIANT_AUTO)


def run_all_routes(Xd, Wd, leaf, g, Ps, variants=VARIANTS):
    """{(variant, P): fp32 Y} through tbik_gemm (P == 0) and shard_partials + tree_combine (P >= 1)."""
    out = {}
    for v in variants:
        tb.tbik_set_gemm_variant(v)
        out[(v, 0)] = tb.tbik_gemm(Xd, Wd, leaf, g, out_dtype=torch.float32)
        for P in Ps:
            parts = tb.tbik_gemm_shard_partials(Xd, Wd, leaf, g, P)
            out[(v, P)] = tb.tbik_tree_combine(parts, out_dtype=torch.float32)
    tb.tbik_set_gemm_variant(tb.VARIANT_AUTO)
    torch.cuda.synchronize()
    return out


def assert_all_equal(outs):
    keys = list(outs)
    ref = outs[keys[0]]
    for k in keys[1:]:
        assert torch.equal(ref.view(torch.int32), outs[k].view(torch.int32)), (keys[0], k)


# ----------------------------------------------------------------------------- pins: the tree, bit-exact

@pytest.mark.parametrize("leaf,g", [(64, 1), (64, 3), (256, 1)])
def test_hand_derived_tree_values(leaf, g):
    """App. C worked by hand (tests/golden/tree_pins.txt): one exact product per superleaf."""
    for name, leaves, t_bits, _ in read_tree_pins():
        ns, sl = len(leaves), leaf * g
        K = ns * sl
        X = np.zeros((3, K), dtype=np.float32)
        W = np.zeros((K, 40), dtype=np.float32)
        for j, v in enumerate(leaves):
            k = j * sl + (j * 37) % sl
            X[:, k] = np.sqrt(np.float32(v))
            W[k, :] = np.sqrt(np.float32(v))
        Xd, Wd = gu.dev_bf16(syn.f32_to_bf16_bits(X)), gu.dev_bf16(syn.f32_to_bf16_bits(W))
        outs = run_all_routes(Xd, Wd, leaf, g, [p for p in (1, 2, 4, 8) if p <= ns])
        for key, y in outs.items():
            assert np.all(gu.u32(gu.host_f32(y)) == t_bits), (name, key)


@pytest.mark.parametrize("M,K,N,leaf,g", [(77, 2048, 200, 64, 1), (130, 3072, 264, 64, 3), (5, 1024, 8, 128, 1),
                                          (300, 4096, 136, 256, 1)])
def test_leaf_sparse_bit_exact_against_oracle(M, K, N, leaf, g):
    """One non-zero product per superleaf: whatever happens inside a leaf is exact, so the tree must match bit for bit."""
    Xb, Wb = syn.gemm_leaf_sparse(100 + M, M, K, N, leaf * g)
    y_orc, ybf_orc = orc.gemm(Xb, Wb, leaf, g)
    Xd, Wd = gu.dev_bf16(Xb), gu.dev_bf16(Wb)
    ns = K // (leaf * g)
    outs = run_all_routes(Xd, Wd, leaf, g, [p for p in (1, 2, 4, 8, 16) if p <= ns])
    for key, y in outs.items():
        assert np.array_equal(gu.u32(gu.host_f32(y)), gu.u32(y_orc)), key
    ybf = tb.tbik_gemm(Xd, Wd, leaf, g, out_dtype=torch.bfloat16)
    assert np.array_equal(gu.host_bf16_bits(ybf), ybf_orc)


@pytest.mark.parametrize("M,K,N,leaf,g,Ps", [(9, 16384, 72, 64, 1, (1, 16, 64)), (3, 65536, 40, 64, 1, (1, 2, 64)),
                                             (5, 8192, 24, 16, 1, (1, 8, 64))])
def test_deep_trees_and_many_shards(M, K, N, leaf, g, Ps):
    """256, 1024 and 512 superleaves (trees deeper than one kernel walks in registers: the K cut inside tbik_gemm and
    the reference kernel take over) and the largest shard count, on leaf-sparse inputs: bit-exact against the oracle."""
    Xb, Wb = syn.gemm_leaf_sparse(300 + M, M, K, N, leaf * g)
    y_orc, _ = orc.gemm(Xb, Wb, leaf, g)
    Xd, Wd = gu.dev_bf16(Xb), gu.dev_bf16(Wb)
    outs = run_all_routes(Xd, Wd, leaf, g, list(Ps))
    for key, y in outs.items():
        assert np.array_equal(gu.u32(gu.host_f32(y)), gu.u32(y_orc)), key


@pytest.mark.parametrize("M,K,N,leaf,g", [(70, 1024, 136, 64, 1), (33, 768, 264, 64, 3), (1, 512, 8, 64, 1),
                                          (129, 2048, 128, 128, 2)])
def test_small_integer_inputs_exact(M, K, N, leaf, g):
    """|x|,|w| <= 8: every order gives the exact integer, so this pins indexing, layout and ragged edges."""
    Xb, Wb = syn.gemm_small_integers(200 + M, M, K, N)
    want = (syn.bf16_bits_to_f32(Xb).astype(np.int64) @ syn.bf16_bits_to_f32(Wb).astype(np.int64)).astype(np.float32)
    Xd, Wd = gu.dev_bf16(Xb), gu.dev_bf16(Wb)
    ns = K // (leaf * g)
    outs = run_all_routes(Xd, Wd, leaf, g, [p for p in (1, 2, 4) if p <= ns])
    for key, y in outs.items():
        assert np.array_equal(gu.host_f32(y), want), key


def test_strided_operands_and_outputs():
    """Leading dimensions larger than the logical width (views into wider buffers)."""
    M, K, N, leaf = 40, 512, 72, 64
    Xb, Wb = syn.gemm_small_integers(7, M, K, N)
    want = (syn.bf16_bits_to_f32(Xb).astype(np.int64) @ syn.bf16_bits_to_f32(Wb).astype(np.int64)).astype(np.float32)
    Xw = torch.zeros((M, K + 64), dtype=torch.bfloat16, device="cuda:0")
    Ww = torch.zeros((K, N + 24), dtype=torch.bfloat16, device="cuda:0")
    Yw = torch.full((M, N + 9), -1.0, dtype=torch.float32, device="cuda:0")
    Xw[:, :K] = gu.dev_bf16(Xb)
    Ww[:, :N] = gu.dev_bf16(Wb)
    for v in VARIANTS:
        tb.tbik_set_gemm_variant(v)
        Yw.fill_(-1.0)
        tb.tbik_gemm(Xw[:, :K], Ww[:, :N], leaf, 1, out=Yw[:, :N])
        torch.cuda.synchronize()
        assert np.array_equal(gu.host_f32(Yw[:, :N]), want), v
        assert torch.all(Yw[:, N:] == -1.0)          # nothing written past N


def test_k_first_zero_is_the_odd_part():
    """k_first = 0 asks for the smallest legal K_first (App. D.1): K = 12288, leaf 256 -> 48 leaves -> 3."""
    c = syn.gemm_downproj(64)
    Xd, Wd = gu.dev_bf16(c["X"]), gu.dev_bf16(c["W"])
    a = tb.tbik_gemm(Xd, Wd, 256, 3, out_dtype=torch.float32)
    b = tb.tbik_gemm(Xd, Wd, 256, 0, out_dtype=torch.float32)
    assert torch.equal(a.view(torch.int32), b.view(torch.int32))
    pa = tb.tbik_gemm_shard_partials(Xd, Wd, 256, 0, 4)
    pb = tb.tbik_gemm_shard_partials(Xd, Wd, 256, 3, 4)
    assert torch.equal(pa.view(torch.int32), pb.view(torch.int32))


# ----------------------------------------------------------------------------- tiny config: full parity

def test_tiny_config_full_parity():
    """M=4, K=512, N=256, leaf 64 (8 leaves): P in {whole, 1, 2, 4, 8}, fp32 and bf16 outputs, every variant."""
    c = syn.gemm_tiny()
    Xd, Wd = gu.dev_bf16(c["X"]), gu.dev_bf16(c["W"])
    outs = run_all_routes(Xd, Wd, c["leaf"], 1, (1, 2, 4, 8))
    assert_all_equal(outs)
    y_gpu = gu.host_f32(outs[(VARIANTS[0], 0)])
    y_orc, _ = orc.gemm(c["X"], c["W"], c["leaf"], 1)
    y64, A = gu.fp64_ref(c["X"], c["W"])
    gu.check_fp32_against_fp64(y_gpu, y64, A)
    h = c["leaf"] + 8
    assert np.all(np.abs(y_gpu.astype(np.float64) - y_orc) <= 2 * h * 2.0 ** -24 * A)
    for v in VARIANTS:
        tb.tbik_set_gemm_variant(v)
        ybf = gu.host_bf16_bits(tb.tbik_gemm(Xd, Wd, c["leaf"], 1, out_dtype=torch.bfloat16))
        n_exc = gu.check_bf16_against_oracle(ybf, y_gpu, y_orc)
        assert n_exc <= max(2, y_gpu.size // 200)
        for P in (1, 2, 4, 8):
            parts = tb.tbik_gemm_shard_partials(Xd, Wd, c["leaf"], 1, P)
            assert np.array_equal(gu.host_bf16_bits(tb.tbik_tree_combine(parts, out_dtype=torch.bfloat16)), ybf)


def test_shard_partials_match_oracle_on_exact_inputs():
    """partials[p] themselves (what a rank would hold before the all-reduce), bit-exact on leaf-sparse data."""
    M, K, N, leaf = 9, 1024, 48, 64
    Xb, Wb = syn.gemm_leaf_sparse(5, M, K, N, leaf)
    Xd, Wd = gu.dev_bf16(Xb), gu.dev_bf16(Wb)
    for P in (1, 2, 4, 8, 16):
        _, _, want = orc.gemm(Xb, Wb, leaf, 1, orc.EVAL_SHARDED, P, want_partials=True)
        for v in VARIANTS:
            tb.tbik_set_gemm_variant(v)
            got = gu.host_f32(tb.tbik_gemm_shard_partials(Xd, Wd, leaf, 1, P))
            assert np.array_equal(gu.u32(got), gu.u32(want)), (P, v)


def test_tree_combine_alone_bit_exact():
    rng = np.random.default_rng(3)
    for P in (1, 2, 4, 8, 16, 32, 64):
        for (M, N) in [(7, 36), (3, 37), (64, 256)]:
            parts = (rng.standard_normal((P, M, N)) * np.exp2(rng.integers(-8, 9, (P, M, N)))).astype(np.float32)
            y32, ybf = orc.tree_combine(parts)
            d = gu.dev_f32(parts)
            assert np.array_equal(gu.u32(gu.host_f32(tb.tbik_tree_combine(d, out_dtype=torch.float32))), gu.u32(y32))
            assert np.array_equal(gu.host_bf16_bits(tb.tbik_tree_combine(d, out_dtype=torch.bfloat16)), ybf)


# ----------------------------------------------------------------------------- 8B-class shapes

def _big_case(name):
    if name == "oproj":
        return syn.gemm_oproj(4096), [1, 16, 64, 256, 1024, 4096]
    if name == "downproj":
        return syn.gemm_downproj(4096), [1, 64, 512, 4096]
    # a second 8B-class shape set (Sec. 4.1's Llama-3.1-8B / Mistral-7B): K = 14336 = 7 * 2^11 -> leaf 256, K_first 7
    return syn.gemm_downproj(4096, seed=5, K=14336, N=4096, leaf=256, k_first=7), [1, 64, 512, 4096]


@pytest.mark.parametrize("name", ["oproj", "downproj", "downproj_k14336"])
def test_8b_shapes_invariance_and_sampled_parity(name):
    """Row r of Y has the same bits for every M, every P in {1,2,4,8}, every kernel variant and every repetition;
    sampled elements match the oracle within the stated tolerance."""
    c, Ms = _big_case(name)
    leaf, g, K, N = c["leaf"], c["k_first"], c["K"], c["N"]
    Xd, Wd = gu.dev_bf16(c["X"]), gu.dev_bf16(c["W"])

    tb.tbik_set_gemm_variant(tb.VARIANT_AUTO)
    full = tb.tbik_gemm(Xd, Wd, leaf, g, out_dtype=torch.float32)
    torch.cuda.synchronize()
    digests = {gu.digest(full)}
    # every P, at full M, twice
    for rep in range(2):
        for P in (1, 2, 4, 8):
            parts = tb.tbik_gemm_shard_partials(Xd, Wd, leaf, g, P)
            digests.add(gu.digest(tb.tbik_tree_combine(parts, out_dtype=torch.float32)))
            del parts
        digests.add(gu.digest(tb.tbik_gemm(Xd, Wd, leaf, g, out_dtype=torch.float32)))
    assert len(digests) == 1                      # the analogue of "count of unique outputs = 1"
    # every M (prefix of the batch), default variant and forced variants, P in {whole, 8}
    for M in Ms:
        for v in ([tb.VARIANT_AUTO, tb.VARIANT_T128, tb.VARIANT_T32, tb.VARIANT_T64] if M <= 1024 else [tb.VARIANT_AUTO]):
            tb.tbik_set_gemm_variant(v)
            y = tb.tbik_gemm(Xd[:M], Wd, leaf, g, out_dtype=torch.float32)
            assert torch.equal(y.view(torch.int32), full[:M].view(torch.int32)), (M, v)
            parts = tb.tbik_gemm_shard_partials(Xd[:M], Wd, leaf, g, 8)
            y = tb.tbik_tree_combine(parts, out_dtype=torch.float32)
            assert torch.equal(y.view(torch.int32), full[:M].view(torch.int32)), (M, v, "P8")
    tb.tbik_set_gemm_variant(tb.VARIANT_AUTO)
    # row position: a permuted batch gives permuted rows; one row alone gives the same bits
    perm = torch.randperm(512, generator=torch.Generator().manual_seed(0)).to("cuda:0")
    y = tb.tbik_gemm(Xd[:512][perm].contiguous(), Wd, leaf, g, out_dtype=torch.float32)
    assert torch.equal(y.view(torch.int32), full[:512][perm].view(torch.int32))
    y = tb.tbik_gemm(Xd[1000:1001], Wd, leaf, g, out_dtype=torch.float32)
    assert torch.equal(y.view(torch.int32), full[1000:1001].view(torch.int32))
    # the reference kernel (different schedule altogether) on a slab of rows
    parts, yref = tb.tbik_gemm_reference(Xd[:160], Wd, leaf, g, 1)
    assert torch.equal(yref.view(torch.int32), full[:160].view(torch.int32))

    # sampled parity against the oracle and fp64
    rows, cols = syn.sample_elements(11, 4096, N, 64, 256)
    y_orc = orc.gemm_elements(c["X"], c["W"], rows, cols, leaf, g)
    y64, A = gu.fp64_ref(c["X"], c["W"], rows, cols)
    y_gpu = gu.host_f32(full)[rows, cols]
    gu.check_fp32_against_fp64(y_gpu, y64, A)
    assert np.all(np.abs(y_gpu.astype(np.float64) - y_orc) <= 2 * (leaf * g + 8) * 2.0 ** -24 * A)
    ybf = gu.host_bf16_bits(tb.tbik_gemm(Xd, Wd, leaf, g, out_dtype=torch.bfloat16))[rows, cols]
    n_exc = gu.check_bf16_against_oracle(ybf, y_gpu, y_orc)
    print("bf16 outputs that differ from bf16(oracle) across a rounding boundary: %d of %d (%s)" % (n_exc, y_gpu.size, name))
    # ten times the fraction measured on this data (1, 5 and 12 of 15936: the longer the superleaf, the further the MFMA's
    # order inside it drifts from the oracle's left-to-right sum, and the more often a rounding boundary falls in between)
    assert n_exc <= {"oproj": 10, "downproj": 50, "downproj_k14336": 120}[name], n_exc


def test_small_m_full_parity_oproj():
    """M = 64 of the o_proj shape, every element against the oracle."""
    c = syn.gemm_oproj(64)
    Xd, Wd = gu.dev_bf16(c["X"]), gu.dev_bf16(c["W"])
    y_gpu = gu.host_f32(tb.tbik_gemm(Xd, Wd, c["leaf"], 1, out_dtype=torch.float32))
    y_orc, _ = orc.gemm(c["X"], c["W"], c["leaf"], 1)
    y64, A = gu.fp64_ref(c["X"], c["W"])
    gu.check_fp32_against_fp64(y_gpu, y64, A)
    assert np.all(np.abs(y_gpu.astype(np.float64) - y_orc) <= 2 * (c["leaf"] + 8) * 2.0 ** -24 * A)
    ybf = gu.host_bf16_bits(tb.tbik_gemm(Xd, Wd, c["leaf"], 1, out_dtype=torch.bfloat16))
    n_exc = gu.check_bf16_against_oracle(ybf, y_gpu, y_orc)
    print("bf16 outputs that differ from bf16(oracle) across a rounding boundary: %d of %d (o_proj M = 64)" % (n_exc, y_gpu.size))
    assert n_exc <= 400                           # measured: 39 of 262144


def test_small_m_full_parity_downproj():
    """M = 64 of the down_proj shape (superleaves of 768), every element against the oracle."""
    c = syn.gemm_downproj(64)
    leaf, g = c["leaf"], c["k_first"]
    Xd, Wd = gu.dev_bf16(c["X"]), gu.dev_bf16(c["W"])
    y_gpu = gu.host_f32(tb.tbik_gemm(Xd, Wd, leaf, g, out_dtype=torch.float32))
    y_orc, _ = orc.gemm(c["X"], c["W"], leaf, g)
    y64, A = gu.fp64_ref(c["X"], c["W"])
    gu.check_fp32_against_fp64(y_gpu, y64, A)
    assert np.all(np.abs(y_gpu.astype(np.float64) - y_orc) <= 2 * (leaf * g + 8) * 2.0 ** -24 * A)
    ybf = gu.host_bf16_bits(tb.tbik_gemm(Xd, Wd, leaf, g, out_dtype=torch.bfloat16))
    n_exc = gu.check_bf16_against_oracle(ybf, y_gpu, y_orc)
    print("bf16 outputs that differ from bf16(oracle) across a rounding boundary: %d of %d (down_proj M = 64)" % (n_exc, y_gpu.size))
    assert n_exc <= 1000                          # sampled at M = 4096: 5 of 15936


def test_twenty_repetitions_give_one_output():
    """The race detector: the tuned kernel keeps its own count of loads and stores in flight and reuses live LDS as the
    output patch, so a race would show as a flipped bit now and then.  Twenty back-to-back calls of tbik_gemm and of
    shard_partials(P = 8) + tree_combine at the full o_proj shape must all give the first call's bits."""
    c = syn.gemm_oproj(4096)
    leaf, g = c["leaf"], c["k_first"]
    Xd, Wd = gu.dev_bf16(c["X"]), gu.dev_bf16(c["W"])
    first = tb.tbik_gemm(Xd, Wd, leaf, g, out_dtype=torch.bfloat16).clone()
    parts = torch.empty((8, 4096, c["N"]), dtype=torch.float32, device="cuda:0")
    y = torch.empty_like(first)
    for rep in range(20):
        tb.tbik_gemm(Xd, Wd, leaf, g, out=y)
        assert torch.equal(y.view(torch.int16), first.view(torch.int16)), ("tbik_gemm", rep)
        tb.tbik_gemm_shard_partials(Xd, Wd, leaf, g, 8, out=parts)
        tb.tbik_tree_combine(parts, out=y)
        assert torch.equal(y.view(torch.int16), first.view(torch.int16)), ("shard_partials(8) + tree_combine", rep)


def test_large_batch_and_ragged_width():
    """M = 40000 rows (313 row tiles, the last one ragged) and N = 4104 (one ragged column tile): a row's bits do not
    depend on the batch it sits in, and sampled elements match the oracle."""
    M, K, N, leaf = 40000, 2048, 4104, 256
    Xb, Wb = syn.gemm_random(77, M, K, N)
    Xd, Wd = gu.dev_bf16(Xb), gu.dev_bf16(Wb)
    full = tb.tbik_gemm(Xd, Wd, leaf, 1, out_dtype=torch.float32)
    for lo, hi in ((0, 1), (39999, 40000), (12345, 12345 + 77), (39936, 40000)):
        part = tb.tbik_gemm(Xd[lo:hi], Wd, leaf, 1, out_dtype=torch.float32)
        assert torch.equal(part.view(torch.int32), full[lo:hi].view(torch.int32)), (lo, hi)
    parts = tb.tbik_gemm_shard_partials(Xd, Wd, leaf, 1, 4)
    assert torch.equal(tb.tbik_tree_combine(parts, out_dtype=torch.float32).view(torch.int32), full.view(torch.int32))
    del parts
    rng = np.random.Generator(np.random.PCG64(78))
    rows = np.concatenate([rng.integers(0, M, size=500), [0, M - 1, M - 1]])
    cols = np.concatenate([rng.integers(0, N, size=500), [0, N - 1, 4096]])
    y_orc = orc.gemm_elements(Xb, Wb, rows, cols, leaf, 1)
    y64, A = gu.fp64_ref(Xb, Wb, rows, cols)
    y_gpu = gu.host_f32(full)[rows, cols]
    gu.check_fp32_against_fp64(y_gpu, y64, A)
    assert np.all(np.abs(y_gpu.astype(np.float64) - y_orc) <= 2 * (leaf + 8) * 2.0 ** -24 * A)


def test_baseline_gemm_is_not_shard_invariant():
    """Context for the method (Sec. 3.3): with an ordinary GEMM, summing per-shard results differs in bits
    from the whole-K result, while the tree route does not."""
    c = syn.gemm_oproj(256)
    Xd, Wd = gu.dev_bf16(c["X"]), gu.dev_bf16(c["W"])
    whole = torch.matmul(Xd.float(), Wd.float())
    K = c["K"]
    split = sum(torch.matmul(Xd[:, i * K // 4:(i + 1) * K // 4].float(), Wd[i * K // 4:(i + 1) * K // 4].float())
                for i in range(4))
    assert not torch.equal(whole.view(torch.int32), split.view(torch.int32))
