"""The C-ABI library loads, exports every function declared in include/tbik.h, and rejects bad
arguments before touching the device (CPU only: no kernel is launched here)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    from paper_2511_17826_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2511_17826_amd import build
        build.build()
    return binding.lib()


def declared_functions():
    src = open(os.path.join(ROOT, "include", "tbik.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    names = re.findall(r"\b(tbik_[a-z0-9_]+)\s*\(", src)
    return sorted(set(names))


def test_every_declared_symbol_is_exported_and_bound(L):
    from paper_2511_17826_amd import binding
    names = declared_functions()
    assert {"tbik_gemm", "tbik_gemm_shard_partials", "tbik_tree_combine", "tbik_rmsnorm", "tbik_row_reduce"} <= set(names)
    for n in names:
        assert hasattr(L, n), n
        assert n in binding.SIGNATURES, "binding lacks a signature for " + n


def test_status_strings_and_version(L):
    assert L.tbik_status_string(0) == b"ok"
    assert all(L.tbik_status_string(i) for i in range(0, 10))
    assert L.tbik_version().startswith(b"tbik")
    assert L.tbik_variant_name(0) == b"auto" and L.tbik_variant_name(99) is None


def test_workspace_sizes_are_pure_and_zero_for_illegal_shapes(L):
    assert L.tbik_gemm_workspace_bytes(4, 256, 512, 64, 1) == L.tbik_gemm_workspace_bytes(4, 256, 512, 64, 1)
    assert L.tbik_gemm_workspace_bytes(4, 256, 500, 64, 1) == 0
    assert L.tbik_row_reduce_workspace_bytes(512, 151936, 2) >= 2 * 512 * 19 * 4
    assert L.tbik_row_reduce_workspace_bytes(4, 100, 7) == 0


GOOD = 0x1000  # a fake, aligned, non-null "device pointer": validation must fail before it is ever used


def gemm(L, **kw):
    a = dict(X=GOOD, ldx=512, W=GOOD, ldw=256, Y=GOOD, ldy=256, dt=1, M=4, N=256, K=512, leaf=64, g=1, ws=None, wsb=0)
    a.update(kw)
    return L.tbik_gemm(a["X"], a["ldx"], a["W"], a["ldw"], a["Y"], a["ldy"], a["dt"], a["M"], a["N"], a["K"],
                       a["leaf"], a["g"], a["ws"], a["wsb"], None)


def test_gemm_argument_validation(L):
    assert gemm(L, M=0) == 0 and gemm(L, N=0) == 0                    # empty problem: OK, nothing launched
    assert gemm(L, X=None) == 1 and gemm(L, W=None) == 1 and gemm(L, Y=None) == 1
    assert gemm(L, K=500) == 2                                         # K not a multiple of the superleaf
    assert gemm(L, K=384, ldx=384) == 2                                # 6 superleaves: not a power of two
    assert gemm(L, leaf=8, g=1, K=512) == 2                            # superleaf not a multiple of 16
    assert gemm(L, K=384, ldx=384, g=0, M=0) == 0                      # k_first 0 = odd part of 6 leaves = 3: two superleaves
    assert gemm(L, K=500, g=0) == 2 and gemm(L, g=-1) == 2             # k_first 0 needs K % leaf == 0; negative is illegal
    assert L.tbik_gemm_workspace_bytes(4, 256, 384, 64, 0) == L.tbik_gemm_workspace_bytes(4, 256, 384, 64, 3)
    assert gemm(L, M=-1) == 2 and gemm(L, leaf=0) == 2
    assert gemm(L, ldx=504) == 2 and gemm(L, ldy=100) == 2             # leading dimension too small
    assert gemm(L, dt=5) == 4
    assert gemm(L, X=GOOD + 2) == 5 and gemm(L, ldw=260) == 5          # misaligned pointer / leading dimension


def test_fp16_entry_points_validate_like_the_bf16_ones(L):
    def g16(**kw):
        a = dict(X=GOOD, ldx=512, W=GOOD, ldw=256, Y=GOOD, ldy=256, dt=2, M=0, N=256, K=512, leaf=64, g=1)
        a.update(kw)
        return L.tbik_gemm_f16(a["X"], a["ldx"], a["W"], a["ldw"], a["Y"], a["ldy"], a["dt"], a["M"], a["N"], a["K"],
                               a["leaf"], a["g"], None, 0, None)
    assert g16() == 0 and g16(dt=0) == 0
    assert g16(dt=1) == 4                                              # bf16 output does not go with fp16 operands
    assert gemm(L, dt=2) == 4                                          # nor fp16 output with bf16 operands
    assert g16(M=4, X=None) == 1 and g16(K=500) == 2 and g16(M=4, X=GOOD + 2) == 5
    sp = L.tbik_gemm_shard_partials_f16
    assert sp(GOOD, 512, GOOD, 256, GOOD, 4, 256, 512, 64, 1, 3, None, 0, None) == 3
    assert sp(GOOD, 512, GOOD, 256, None, 4, 256, 512, 64, 1, 2, None, 0, None) == 1
    rf = L.tbik_gemm_reference_f16
    assert rf(GOOD, 512, GOOD, 256, GOOD, GOOD, 256, 1, 4, 256, 512, 64, 1, 1, None) == 4
    assert rf(GOOD, 512, GOOD, 256, GOOD, GOOD, 256, 2, 4, 256, 512, 64, 1, 2, None) == 3      # Y only with P == 1
    assert L.tbik_tree_combine(GOOD, 2, GOOD, 256, 2, 0, 256, None) == 0                       # fp16 output is offered
    assert L.tbik_row_reduce(GOOD, 2, GOOD, 0, 0, 1024, GOOD, 1 << 20, None) == 0              # and so are fp16 rows
    assert L.tbik_row_reduce(GOOD, 2, GOOD, 0, 4, 1028, GOOD, 1 << 20, None) == 2              # in leaves of 8
    for rn in (L.tbik_rmsnorm_f16,):
        assert rn(GOOD, GOOD, GOOD, 0, 4096, 1e-6, None) == 0
        assert rn(None, GOOD, GOOD, 4, 4096, 1e-6, None) == 1
        assert rn(GOOD, GOOD, GOOD, 4, 4100, 1e-6, None) == 2
        assert rn(GOOD + 8, GOOD, GOOD, 4, 4096, 1e-6, None) == 5
    for tail in (L.tbik_combine_residual_rmsnorm, L.tbik_combine_residual_rmsnorm_f16):
        assert tail(GOOD, 2, GOOD, GOOD, 1e-6, GOOD, GOOD + 65536, 0, 4096, None) == 0
        assert tail(GOOD, 3, GOOD, GOOD, 1e-6, GOOD, GOOD + 65536, 4, 4096, None) == 3
        assert tail(GOOD, 32, GOOD, GOOD, 1e-6, GOOD, GOOD + 65536, 4, 4096, None) == 7
        assert tail(GOOD, 2, GOOD, GOOD, 1e-6, GOOD, GOOD, 4, 4096, None) == 2                 # normed may not alias hidden
        assert tail(GOOD, 2, None, GOOD, 1e-6, GOOD, GOOD + 65536, 4, 4096, None) == 1


@pytest.mark.parametrize("entry", ["tbik_attention", "tbik_attention_f16"])
def test_attention_argument_validation(L, entry):
    def att(**kw):
        a = dict(Q=GOOD, K=GOOD, V=GOOD, O=GOOD, cq=GOOD, ck=GOOD, batch=2, mq=8, mk=8, tq=16, tk=16, hq=4, hkv=2, d=128,
                 sq=512, sk=256, sv=256, so=512, scale=0.1, causal=1, ws=None, wsb=0)
        a.update(kw)
        return getattr(L, entry)(a["Q"], a["K"], a["V"], a["O"], a["cq"], a["ck"], a["batch"], a["mq"], a["mk"], a["tq"],
                                 a["tk"], a["hq"], a["hkv"], a["d"], a["sq"], a["sk"], a["sv"], a["so"], a["scale"],
                                 a["causal"], a["ws"], a["wsb"], None)
    assert att(batch=0) == 0 and att(mq=0) == 0 and att(tq=0) == 0            # nothing to do: OK before any pointer is looked at
    assert att(batch=-1) == 2 and att(hq=5) == 2 and att(hkv=0) == 2          # heads_q must be a multiple of heads_kv
    assert att(sq=500) == 2 and att(sk=128) == 2 and att(so=1 << 24) == 2     # token stride below heads * 128, or too large
    assert att(d=64) == 7                                                     # only head dimension 128 is built
    assert att(Q=None) == 1 and att(cq=None) == 1 and att(K=None) == 1
    assert att(Q=GOOD + 2) == 5 and att(sk=260) == 5 and att(ck=GOOD + 2) == 5
    assert att(mk=-1) == 2
    # more than one split of keys (4096): the fold needs a workspace of the advertised size, 256-byte aligned
    need = L.tbik_attention_workspace_bytes(2, 8, 5000, 4, 2)
    assert need > 0 and L.tbik_attention_workspace_bytes(2, 8, 4096, 4, 2) == 0
    assert att(mk=5000, tk=6000) == 6 and att(mk=5000, tk=6000, ws=GOOD, wsb=need - 1) == 6
    assert att(mk=5000, tk=6000, ws=GOOD + 16, wsb=need) == 5


def test_shard_and_combine_validation(L):
    sp = L.tbik_gemm_shard_partials
    args = lambda P, part=GOOD: (GOOD, 512, GOOD, 256, part, 4, 256, 512, 64, 1, P, None, 0, None)
    assert sp(*args(3)) == 3 and sp(*args(0)) == 3 and sp(*args(16)) == 3      # not a power of two / > n_s = 8
    assert sp(*args(2, None)) == 1
    tc = L.tbik_tree_combine
    assert tc(GOOD, 3, GOOD, 256, 1, 4, 256, None) == 3
    assert tc(GOOD, 128, GOOD, 256, 1, 4, 256, None) == 3
    assert tc(None, 2, GOOD, 256, 1, 4, 256, None) == 1
    assert tc(GOOD, 2, GOOD, 100, 1, 4, 256, None) == 2
    assert tc(GOOD, 2, GOOD, 256, 9, 4, 256, None) == 4
    assert tc(GOOD, 2, GOOD, 256, 1, 0, 256, None) == 0


def test_reduction_validation(L):
    rn = L.tbik_rmsnorm
    assert rn(GOOD, GOOD, GOOD, 0, 4096, 1e-6, None) == 0
    assert rn(None, GOOD, GOOD, 4, 4096, 1e-6, None) == 1
    assert rn(GOOD, GOOD, GOOD, 4, 4100, 1e-6, None) == 2
    assert rn(GOOD + 8, GOOD, GOOD, 4, 4096, 1e-6, None) == 5
    rr = L.tbik_row_reduce
    assert rr(GOOD, 0, GOOD, 2, 0, 1024, GOOD, 1 << 20, None) == 0
    assert rr(GOOD, 0, GOOD, 2, 4, 1022, GOOD, 1 << 20, None) == 2
    assert rr(GOOD, 0, GOOD, 2, 4, 0, GOOD, 1 << 20, None) == 2
    assert rr(GOOD, 3, GOOD, 2, 4, 1024, GOOD, 1 << 20, None) == 4
    assert rr(GOOD, 0, GOOD, 5, 4, 1024, GOOD, 1 << 20, None) == 4
    assert rr(GOOD, 0, GOOD, 2, 4, 1024, None, 0, None) == 6
    assert rr(GOOD, 0, GOOD, 2, 4, 1024, GOOD, 8, None) == 6
    assert rr(None, 0, GOOD, 0, 4, 1024, GOOD, 1 << 20, None) == 1


def test_attention_variant_switch(L):
    assert L.tbik_set_attention_variant(2) == 0 and L.tbik_set_attention_variant(1) == 0
    assert L.tbik_set_attention_variant(3) == 4 and L.tbik_set_attention_variant(-1) == 4
    assert L.tbik_set_attention_variant(0) == 0


def test_variant_switch(L):
    assert L.tbik_set_gemm_variant(99) == 7
    assert L.tbik_set_gemm_variant(1) == 0
    assert L.tbik_set_gemm_variant(0) == 0


def test_product_path_does_not_import_the_oracle():
    """The binding and the sources of the library never reference oracle/ (the oracle is test infrastructure)."""
    pkg = os.path.join(ROOT, "paper_2511_17826_amd")
    for dirpath, _, files in os.walk(pkg):
        if "_build" in dirpath:
            continue
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "tbik_oracle" not in text and "from oracle" not in text and "import oracle" not in text, f


def test_fused_tail_argument_validation(L):
    f = L.tbik_combine_residual_rmsnorm
    ok = (GOOD, 2, GOOD, GOOD, 1e-6, GOOD + 0x10000, GOOD + 0x20000, 4, 4096, None)
    def call(**kw):
        names = ("partials", "P", "residual", "weight", "eps", "hidden", "normed", "M", "H", "stream")
        a = dict(zip(names, ok)); a.update(kw)
        return f(*[a[n] for n in names])
    assert call(M=0) == 0
    assert call(partials=None) == 1 and call(normed=None) == 1
    assert call(H=4100) == 2 and call(M=-1) == 2
    assert call(P=3) == 3 and call(P=0) == 3
    assert call(P=32) == 7                                   # legal shard count, not built into the fused kernel
    assert call(residual=GOOD + 2) == 5
    assert call(normed=GOOD, residual=GOOD) == 2             # normed may not share the residual's buffer


def test_fp32_gemm_entry_points_validate_like_the_others(L):
    g = L.tbik_gemm_f32
    assert g(GOOD, 512, GOOD, 256, GOOD, 256, 0, 256, 512, 64, 1, None, 0, None) == 0
    assert g(None, 512, GOOD, 256, GOOD, 256, 4, 256, 512, 64, 1, None, 0, None) == 1
    assert g(GOOD, 512, GOOD, 256, GOOD, 256, 4, 256, 500, 64, 1, None, 0, None) == 2
    assert g(GOOD, 508, GOOD, 256, GOOD, 256, 4, 256, 448, 64, 1, None, 0, None) == 2          # 7 superleaves
    assert g(GOOD, 516, GOOD, 260, GOOD, 260, 0, 256, 512, 64, 1, None, 0, None) == 0          # rows of 4 floats suffice
    assert g(GOOD, 518, GOOD, 256, GOOD, 256, 4, 256, 512, 64, 1, None, 0, None) == 5          # ldx not a multiple of 4
    assert g(GOOD, 512, GOOD, 256, GOOD, 256, 4, 256, 512, 64, 1, None, 0, None) == 6          # this shape splits K: workspace
    sp = L.tbik_gemm_shard_partials_f32
    assert sp(GOOD, 512, GOOD, 256, GOOD, 4, 256, 512, 64, 1, 3, None, 0, None) == 3
    assert sp(GOOD, 512, GOOD, 256, None, 4, 256, 512, 64, 1, 2, None, 0, None) == 1
    rf = L.tbik_gemm_reference_f32
    assert rf(GOOD, 512, GOOD, 256, GOOD, GOOD, 256, 4, 256, 512, 64, 1, 2, None) == 3         # Y only with P == 1
    assert rf(GOOD, 512, GOOD, 256, None, None, 256, 4, 256, 512, 64, 1, 1, None) == 1
