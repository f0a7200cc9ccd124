"""Seeded synthetic inputs for the TBIK kernels and for the CPU oracle that checks them.

This module only *makes data*: random draws, casts to bf16 storage and the
elementwise recipe of a workload's inputs.  It holds none of the method's
arithmetic (no tree, no reduction, no GEMM) and is the one module that the
HIP path's tests/bench and the CPU oracle's tests both use.

bf16 tensors travel as ``numpy.uint16`` arrays holding the raw bit patterns,
so that the CPU oracle and the GPU see exactly the same bits.

Workloads follow the row-parallel layers of the paper's models (Sec. 3.3:
``o_proj`` and ``down_proj`` split K across GPUs) at 8B-class and 32B-class
shapes; the tensors are random stand-ins for the activations and weights of
those layers, not items of any dataset.
"""
from __future__ import annotations

import numpy as np


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to bf16 storage (round-to-nearest-even), as uint16 bit patterns.

    Only used to put generated inputs into their storage format.
    NaN is not expected in generated data and is not special-cased.
    """
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to the fp32 values they denote (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def f32_to_f16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to IEEE binary16 storage (numpy's cast: round-to-nearest-even), as uint16 bit patterns."""
    return np.ascontiguousarray(a, dtype=np.float32).astype(np.float16).view(np.uint16)


def f16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen binary16 bit patterns (uint16) to the fp32 values they denote (exact)."""
    return np.ascontiguousarray(b, dtype=np.uint16).view(np.float16).astype(np.float32)


def _torch_fp8(fmt: str):
    import torch
    return {"e4m3": torch.float8_e4m3fn, "e5m2": torch.float8_e5m2}[fmt]


def f32_to_fp8_bits(a: np.ndarray, fmt: str = "e4m3") -> np.ndarray:
    """fp32 -> 8-bit OCP patterns ("e4m3": 4 exponent / 3 fraction bits, no infinities, max 448; "e5m2": 5 / 2), round to
    nearest even, by torch's CPU conversion.  Callers keep |a| inside the format's range (no saturation relied on)."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(_torch_fp8(fmt))
    return t.view(torch.uint8).numpy().copy()


def fp8_bits_to_f32(b: np.ndarray, fmt: str = "e4m3") -> np.ndarray:
    import torch
    t = torch.from_numpy(np.ascontiguousarray(b, dtype=np.uint8)).view(_torch_fp8(fmt))
    return t.to(torch.float32).numpy()


def to_storage(a: np.ndarray, fmt: str = "bf16") -> np.ndarray:
    """fp32 values -> storage patterns of format ``fmt``: 16-bit ("bf16", "fp16") or 8-bit ("e4m3", "e5m2")."""
    if fmt == "bf16":
        return f32_to_bf16_bits(a)
    if fmt == "fp16":
        return f32_to_f16_bits(a)
    if fmt in ("e4m3", "e5m2"):
        return f32_to_fp8_bits(a, fmt)
    raise ValueError(fmt)


def from_storage(b: np.ndarray, fmt: str = "bf16") -> np.ndarray:
    """Storage patterns of format ``fmt`` -> the fp32 values they denote (exact)."""
    if fmt == "bf16":
        return bf16_bits_to_f32(b)
    if fmt == "fp16":
        return f16_bits_to_f32(b)
    if fmt in ("e4m3", "e5m2"):
        return fp8_bits_to_f32(b, fmt)
    raise ValueError(fmt)


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


def normal_bf16(rng: np.random.Generator, shape, std: float, mean: float = 0.0, fmt: str = "bf16") -> np.ndarray:
    """N(mean, std) drawn in fp32, stored as bf16 bits (or, with ``fmt="fp16"``, as binary16 bits)."""
    v = rng.standard_normal(size=shape, dtype=np.float32) * np.float32(std) + np.float32(mean)
    return to_storage(v, fmt)


# ----------------------------------------------------------------------------
# GEMM workloads: X [M,K] bf16, W [K,N] bf16 (row-major), plus the tree
# parameters (leaf = K-elements per leaf, k_first = leaves chained before the
# first tree level, App. D.1).
# ----------------------------------------------------------------------------

def gemm_tiny(seed: int = 0):
    """Tiny case: X [4,512] ~ N(0,1), W [512,256] ~ N(0,0.02); leaf 64, 8 leaves."""
    rng = _rng(seed)
    X = normal_bf16(rng, (4, 512), 1.0)
    W = normal_bf16(rng, (512, 256), 0.02)
    return dict(X=X, W=W, M=4, K=512, N=256, leaf=64, k_first=1)


def gemm_oproj(M: int = 4096, seed: int = 1, K: int = 4096, N: int = 4096, leaf: int = 256, k_first: int = 1,
               fmt: str = "bf16"):
    """8B-class attention output projection: X [M,4096] ~ N(0,1), W [4096,4096] ~ N(0,0.02).

    The tensor is always drawn at M_max=4096 rows and the first M rows are
    returned, so row r holds the same bits for every M.
    """
    rng = _rng(seed)
    X = normal_bf16(rng, (4096, K), 1.0, fmt=fmt)[:M]
    W = normal_bf16(rng, (K, N), 0.02, fmt=fmt)
    return dict(X=np.ascontiguousarray(X), W=W, M=M, K=K, N=N, leaf=leaf, k_first=k_first)


def silu_gated_bf16(rng: np.random.Generator, shape) -> np.ndarray:
    """bf16(silu(a) * b), a, b ~ N(0,1): the input distribution of an MLP down projection."""
    a = rng.standard_normal(size=shape, dtype=np.float32)
    b = rng.standard_normal(size=shape, dtype=np.float32)
    return f32_to_bf16_bits((a / (np.float32(1.0) + np.exp(-a))) * b)


def gemm_downproj(M: int = 4096, seed: int = 2, K: int = 12288, N: int = 4096, leaf: int = 256, k_first: int = 3):
    """8B-class MLP down projection: X = bf16(silu(a)*b) [M,12288], W [12288,4096] ~ N(0,0.02).

    48 leaves of 256 = 3 * 16, hence k_first = 3 and 16 superleaves of 768.
    """
    rng = _rng(seed)
    X = silu_gated_bf16(rng, (4096, K))[:M]
    W = normal_bf16(rng, (K, N), 0.02)
    return dict(X=np.ascontiguousarray(X), W=W, M=M, K=K, N=N, leaf=leaf, k_first=k_first)


def gemm_random(seed: int, M: int, K: int, N: int, x_std: float = 1.0, w_std: float = 0.02, fmt: str = "bf16"):
    """Generic random GEMM operands of the same distributions, any shape."""
    rng = _rng(seed)
    return normal_bf16(rng, (M, K), x_std, fmt=fmt), normal_bf16(rng, (K, N), w_std, fmt=fmt)


def gemm_random_fp8(seed: int, M: int, K: int, N: int, fmt: str = "e4m3"):
    """8-bit operands as a scaled-quantisation flow leaves them: X ~ N(0,1) and W ~ N(0,1) in the scaled domain (the
    per-tensor scales that bring weights of std 0.02 into the 8-bit range are outside the GEMM), rounded to ``fmt``."""
    rng = _rng(seed)
    X = rng.standard_normal(size=(M, K), dtype=np.float32)
    W = rng.standard_normal(size=(K, N), dtype=np.float32)
    return f32_to_fp8_bits(X, fmt), f32_to_fp8_bits(W, fmt)


E2M1_VALUES = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0], dtype=np.float32)   # the magnitudes an E2M1 element can hold


def mxfp4_quantize(a: np.ndarray, scale_shift: int = 0):
    """fp32 [R, K] (K a multiple of 32) -> (packed E2M1 pairs uint8 [R, K/2], low nibble = even k; E8M0 scales uint8
    [R, K/32]).  Per block of 32 the scale is the power of two that brings the block's largest magnitude into (3, 6]
    (an all-zero block gets 2^0), shifted by `scale_shift` binades; elements are rounded to the nearest E2M1 magnitude
    (ties to the lower index).  An input recipe: nothing of the method's arithmetic."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    R, K = a.shape
    assert K % 32 == 0
    blocks = a.reshape(R, K // 32, 32)
    amax = np.abs(blocks).max(axis=2)
    e = np.where(amax > 0, np.ceil(np.log2(np.where(amax > 0, amax, 1.0) / 6.0)), 0.0).astype(np.int32) + scale_shift
    scales = np.clip(e + 127, 1, 254).astype(np.uint8)
    scaled = blocks / np.exp2(scales.astype(np.float32) - 127)[:, :, None]
    idx = np.abs(np.abs(scaled)[..., None] - E2M1_VALUES).argmin(axis=-1).astype(np.uint8)
    nib = (idx | (np.signbit(scaled).astype(np.uint8) << 3)).reshape(R, K)
    packed = (nib[:, 0::2] | (nib[:, 1::2] << 4)).astype(np.uint8)
    return packed, scales


def gemm_random_mxfp4(seed: int, M: int, K: int, N: int, scale_spread: int = 0):
    """MXFP4 operands from X ~ N(0,1), W ~ N(0,0.02) (the weight transposed, [N, K]): returns (X packed, X scales,
    Wt packed, W scales).  With `scale_spread` every block's scale is moved by a random number of binades in
    [-scale_spread, scale_spread] (the elements stay as quantised), which spreads the magnitudes of the products."""
    rng = _rng(seed)
    X = rng.standard_normal(size=(M, K), dtype=np.float32)
    Wt = rng.standard_normal(size=(N, K), dtype=np.float32) * np.float32(0.02)
    Xp, Xs = mxfp4_quantize(X)
    Wp, Ws = mxfp4_quantize(Wt)
    if scale_spread:
        Xs = (Xs.astype(np.int32) + rng.integers(-scale_spread, scale_spread + 1, size=Xs.shape)).astype(np.uint8)
        Ws = (Ws.astype(np.int32) + rng.integers(-scale_spread, scale_spread + 1, size=Ws.shape)).astype(np.uint8)
    return Xp, Xs, Wp, Ws


def mxfp8_quantize(a: np.ndarray, fmt: str = "e4m3"):
    """fp32 [R, K] (K a multiple of 32) -> (8-bit patterns uint8 [R, K], E8M0 scales uint8 [R, K/32]).  Per block of 32
    the scale is the power of two that brings the block's largest magnitude into (2^(emax-1), 2^emax] with emax the
    largest exponent of the element format (8 for E4M3, 15 for E5M2; an all-zero block gets 2^0); elements are rounded
    to nearest even by the library's conversion.  An input recipe: nothing of the method's arithmetic."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    R, K = a.shape
    assert K % 32 == 0
    emax = 8 if fmt == "e4m3" else 15
    blocks = a.reshape(R, K // 32, 32)
    amax = np.abs(blocks).max(axis=2)
    e = np.where(amax > 0, np.ceil(np.log2(np.where(amax > 0, amax, 1.0))), float(emax)).astype(np.int32) - emax
    scales = np.clip(e + 127, 1, 254).astype(np.uint8)
    scaled = blocks / np.exp2(scales.astype(np.float32) - 127)[:, :, None]
    return f32_to_fp8_bits(scaled.reshape(R, K), fmt), scales


def gemm_random_mxfp8(seed: int, M: int, K: int, N: int, fmt: str = "e4m3", scale_spread: int = 0):
    """MXFP8 operands from X ~ N(0,1), W ~ N(0,0.02) (the weight transposed, [N, K]): returns (X patterns, X scales,
    Wt patterns, W scales).  With `scale_spread` every block's scale is moved by a random number of binades in
    [-scale_spread, scale_spread] (the elements stay as quantised), which spreads the magnitudes of the products."""
    rng = _rng(seed)
    X = rng.standard_normal(size=(M, K), dtype=np.float32)
    Wt = rng.standard_normal(size=(N, K), dtype=np.float32) * np.float32(0.02)
    Xq, Xs = mxfp8_quantize(X, fmt)
    Wq, Ws = mxfp8_quantize(Wt, fmt)
    if scale_spread:
        Xs = (Xs.astype(np.int32) + rng.integers(-scale_spread, scale_spread + 1, size=Xs.shape)).astype(np.uint8)
        Ws = (Ws.astype(np.int32) + rng.integers(-scale_spread, scale_spread + 1, size=Ws.shape)).astype(np.uint8)
    return Xq, Xs, Wq, Ws


def fp6_magnitudes(fmt: str = "e2m3") -> np.ndarray:
    """The 32 magnitudes a 6-bit element can hold, by pattern (sign bit clear), from the format's definition."""
    ebits, fbits, bias = (2, 3, 1) if fmt == "e2m3" else (3, 2, 3)
    out = []
    for p in range(32):
        e, f = p >> fbits, p & ((1 << fbits) - 1)
        out.append(f * 2.0 ** (1 - bias - fbits) if e == 0 else (f + (1 << fbits)) * 2.0 ** (e - bias - fbits))
    return np.array(out, dtype=np.float32)


def fp6_pack(patterns: np.ndarray) -> np.ndarray:
    """[R, K] 6-bit patterns -> [R, 3K/4] bytes: one little-endian bit stream per row, element k in bits 6k .. 6k+5."""
    patterns = np.asarray(patterns, dtype=np.uint8)
    bits = ((patterns[..., None] >> np.arange(6, dtype=np.uint8)) & 1).astype(np.uint8)
    return np.packbits(bits.reshape(patterns.shape[0], -1), axis=1, bitorder="little")


def mxfp6_quantize(a: np.ndarray, fmt: str = "e2m3"):
    """fp32 [R, K] (K a multiple of 32) -> (packed 6-bit elements uint8 [R, 3K/4], E8M0 scales uint8 [R, K/32]).  Per block
    of 32 the scale is the power of two that brings the block's largest magnitude into the element format's top binade
    (an all-zero block gets 2^0); elements go to the nearest representable magnitude (ties to the lower pattern).  An input
    recipe: nothing of the method's arithmetic."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    R, K = a.shape
    assert K % 32 == 0
    mags = fp6_magnitudes(fmt)
    top = 2.0 if fmt == "e2m3" else 4.0                      # log2 of the top binade's lower end: values up to 7.5 / 28
    blocks = a.reshape(R, K // 32, 32)
    amax = np.abs(blocks).max(axis=2)
    e = np.where(amax > 0, np.floor(np.log2(np.where(amax > 0, amax, 1.0))) - top, 0.0).astype(np.int32)
    scales = np.clip(e + 127, 1, 254).astype(np.uint8)
    scaled = blocks / np.exp2(scales.astype(np.float32) - 127)[:, :, None]
    idx = np.abs(np.abs(scaled)[..., None] - mags).argmin(axis=-1).astype(np.uint8)
    pat = (idx | (np.signbit(scaled).astype(np.uint8) << 5)).reshape(R, K)
    return fp6_pack(pat), scales


def gemm_random_mxfp6(seed: int, M: int, K: int, N: int, fmt: str = "e2m3", scale_spread: int = 0):
    """MXFP6 operands from X ~ N(0,1), W ~ N(0,0.02) (the weight transposed, [N, K]): returns (X packed, X scales,
    Wt packed, W scales).  With `scale_spread` every block's scale is moved by a random number of binades in
    [-scale_spread, scale_spread] (the elements stay as quantised)."""
    rng = _rng(seed)
    X = rng.standard_normal(size=(M, K), dtype=np.float32)
    Wt = rng.standard_normal(size=(N, K), dtype=np.float32) * np.float32(0.02)
    Xp, Xs = mxfp6_quantize(X, fmt)
    Wp, Ws = mxfp6_quantize(Wt, fmt)
    if scale_spread:
        Xs = (Xs.astype(np.int32) + rng.integers(-scale_spread, scale_spread + 1, size=Xs.shape)).astype(np.uint8)
        Ws = (Ws.astype(np.int32) + rng.integers(-scale_spread, scale_spread + 1, size=Ws.shape)).astype(np.uint8)
    return Xp, Xs, Wp, Ws


def gemm_random_f32(seed: int, M: int, K: int, N: int, x_std: float = 1.0, w_std: float = 0.02, exp_spread: int = 0):
    """fp32 operands X [M,K] ~ N(0, x_std), W [K,N] ~ N(0, w_std) with full 24-bit significands; with ``exp_spread`` every
    element is scaled by a random power of two in [-exp_spread, exp_spread] (cancellation and absorption cases)."""
    rng = _rng(seed)
    X = rng.standard_normal(size=(M, K), dtype=np.float32) * np.float32(x_std)
    W = rng.standard_normal(size=(K, N), dtype=np.float32) * np.float32(w_std)
    if exp_spread:
        X = X * np.exp2(rng.integers(-exp_spread, exp_spread + 1, size=(M, K))).astype(np.float32)
        W = W * np.exp2(rng.integers(-exp_spread, exp_spread + 1, size=(K, N))).astype(np.float32)
    return np.ascontiguousarray(X, dtype=np.float32), np.ascontiguousarray(W, dtype=np.float32)


def gemm_small_integers(seed: int, M: int, K: int, N: int, mag: int = 8, fmt: str = "bf16"):
    """Integer-valued operands with |x|,|w| <= mag.

    Every partial sum stays far below 2**24, so any summation order gives the
    exact integer: such inputs test indexing and layout, not rounding.
    """
    rng = _rng(seed)
    X = rng.integers(-mag, mag + 1, size=(M, K)).astype(np.float32)
    W = rng.integers(-mag, mag + 1, size=(K, N)).astype(np.float32)
    return to_storage(X, fmt), to_storage(W, fmt)


def gemm_leaf_sparse(seed: int, M: int, K: int, N: int, superleaf: int, exp_spread: int = 12, fmt: str = "bf16"):
    """Operands with exactly one non-zero product per (row, column, superleaf).

    In every superleaf (``superleaf`` consecutive k) X has one non-zero column
    position per row -- the same position is used for W's only non-zero row in
    that superleaf -- so each superleaf sum is a single exact product whatever
    the order inside the leaf, and only the tree between superleaves rounds.
    Magnitudes are random bf16 values scaled by 2**e, e uniform in
    [-exp_spread, exp_spread], which makes the tree's roundings visible.
    (binary16 storage has a 5-bit exponent: use exp_spread <= 6 with ``fmt="fp16"``
    to keep every value a normal number.)
    """
    assert K % superleaf == 0
    rng = _rng(seed)
    ns = K // superleaf
    X = np.zeros((M, K), dtype=np.float32)
    W = np.zeros((K, N), dtype=np.float32)
    pos = rng.integers(0, superleaf, size=ns)
    for j in range(ns):
        k = j * superleaf + int(pos[j])
        X[:, k] = rng.standard_normal(M).astype(np.float32) * np.exp2(
            rng.integers(-exp_spread, exp_spread + 1, size=M)).astype(np.float32)
        W[k, :] = rng.standard_normal(N).astype(np.float32) * np.exp2(
            rng.integers(-exp_spread, exp_spread + 1, size=N)).astype(np.float32)
    return to_storage(X, fmt), to_storage(W, fmt)


# ----------------------------------------------------------------------------
# Attention workloads: packed variable-length sequences, grouped-query heads
# (8B-class: 32 query heads, 8 key/value heads, head dimension 128).
# ----------------------------------------------------------------------------

def attention_inputs(seed: int, q_lens, k_lens, Hq: int = 32, Hkv: int = 8, D: int = 128, std: float = 1.0,
                     fmt: str = "bf16"):
    """Q [sum(q_lens), Hq, D], K and V [sum(k_lens), Hkv, D] ~ N(0, std) as 16-bit patterns of `fmt`, plus the int32 prefix sums
    cu_q, cu_k [batch + 1].  Sequence b has q_lens[b] query tokens (its last positions) and k_lens[b] keys."""
    rng = _rng(seed)
    q_lens, k_lens = np.asarray(q_lens, dtype=np.int64), np.asarray(k_lens, dtype=np.int64)
    assert q_lens.shape == k_lens.shape
    cu_q = np.concatenate([[0], np.cumsum(q_lens)]).astype(np.int32)
    cu_k = np.concatenate([[0], np.cumsum(k_lens)]).astype(np.int32)
    Q = normal_bf16(rng, (int(cu_q[-1]), Hq, D), std, fmt=fmt)
    K = normal_bf16(rng, (int(cu_k[-1]), Hkv, D), std, fmt=fmt)
    V = normal_bf16(rng, (int(cu_k[-1]), Hkv, D), std, fmt=fmt)
    return dict(Q=Q, K=K, V=V, cu_q=cu_q, cu_k=cu_k, Hq=Hq, Hkv=Hkv, D=D, scale=float(D) ** -0.5)


# ----------------------------------------------------------------------------
# Reduction workloads
# ----------------------------------------------------------------------------

def rmsnorm_inputs(M: int, H: int, seed: int = 3, fmt: str = "bf16"):
    """x [M,H] ~ N(0,1), weight [H] ~ N(1,0.1), both stored in `fmt`; drawn at 8192 rows, first M returned."""
    rng = _rng(seed + 1000 * H)
    w = normal_bf16(rng, (H,), 0.1, mean=1.0, fmt=fmt)
    x = normal_bf16(rng, (8192, H), 1.0, fmt=fmt)[:M]
    return np.ascontiguousarray(x), w


def logits_f32(M: int, V: int = 151936, seed: int = 3, std: float = 3.0) -> np.ndarray:
    """fp32 logits [M,V] ~ N(0,3); row r is the same for every M (rows drawn one stream each)."""
    out = np.empty((M, V), dtype=np.float32)
    for r in range(M):
        out[r] = _rng(seed * 1_000_003 + r).standard_normal(size=V, dtype=np.float32) * np.float32(std)
    return out


def sample_elements(seed: int, M: int, N: int, n_rows: int = 64, n_cols: int = 256):
    """A seeded grid of (row, col) output positions for spot checks at large shapes.

    Always includes the first and last row and column, so the ragged edges of
    a tiling are covered.
    """
    rng = _rng(seed)
    rows = np.unique(np.concatenate([[0, M - 1], rng.integers(0, M, size=max(0, min(n_rows, M) - 2))]))
    cols = np.unique(np.concatenate([[0, N - 1], rng.integers(0, N, size=max(0, min(n_cols, N) - 2))]))
    rr, cc = np.meshgrid(rows, cols, indexing="ij")
    return rr.ravel().astype(np.int64), cc.ravel().astype(np.int64)


# ----------------------------------------------------------------------------
# 32B-class decoder-layer chain (hidden 5120, intermediate 25600, 40 query / 8 KV heads of 128, vocabulary 151936)
# ----------------------------------------------------------------------------

CHAIN_DIMS = dict(hidden=5120, inter=25600, q_heads=40, kv_heads=8, head_dim=128, vocab=151936, tokens=512, leaf=128)


def chain_tensors(device, seed: int = 4):
    """Random-init weights ~N(0,0.02) (bf16), norm weights 1, input x [512,5120] ~N(0,1) (bf16), drawn on `device`
    with a seeded torch generator (the lm_head alone is 1.5 GB, too slow to draw on the host)."""
    import torch
    d = CHAIN_DIMS
    g = torch.Generator(device=device)
    g.manual_seed(seed)

    def w(k, n):
        return (torch.randn((k, n), generator=g, device=device, dtype=torch.float32) * 0.02).to(torch.bfloat16)

    qkv_out = (d["q_heads"] + 2 * d["kv_heads"]) * d["head_dim"]
    return dict(
        x=torch.randn((d["tokens"], d["hidden"]), generator=g, device=device, dtype=torch.float32).to(torch.bfloat16),
        norm1=torch.ones(d["hidden"], device=device, dtype=torch.bfloat16),
        norm2=torch.ones(d["hidden"], device=device, dtype=torch.bfloat16),
        w_qkv=w(d["hidden"], qkv_out), w_o=w(d["q_heads"] * d["head_dim"], d["hidden"]),
        w_gate=w(d["hidden"], d["inter"]), w_up=w(d["hidden"], d["inter"]), w_down=w(d["inter"], d["hidden"]),
        w_lm=w(d["hidden"], d["vocab"]),
    )
