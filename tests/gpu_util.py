"""Helpers for the GPU parity tests: moving bit patterns to and from the device, tolerance checks."""
import hashlib

import numpy as np
import torch

from paper_2511_17826_amd import synthetic as syn


def dev_bf16(bits: np.ndarray) -> torch.Tensor:
    """uint16 bf16 bit patterns -> bfloat16 tensor on cuda:0 (same bits)."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).to("cuda:0")


def dev_f16(bits: np.ndarray) -> torch.Tensor:
    """uint16 binary16 bit patterns -> float16 tensor on cuda:0 (same bits)."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.float16).to("cuda:0")


def dev_f32(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to("cuda:0")


def host_bf16_bits(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


host_f16_bits = host_bf16_bits      # both are 16-bit patterns


def host_f32(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().cpu().numpy()


def u32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


def digest(t: torch.Tensor) -> str:
    """Hash of a tensor's bytes (for 'number of distinct outputs must be 1' checks)."""
    return hashlib.sha1(t.contiguous().view(torch.uint8).cpu().numpy().tobytes()).hexdigest()


def fp64_ref(Xb, Wb, rows=None, cols=None, fmt="bf16"):
    """fp64 brute-force values and A = sum_k |x_k w_k| (whole matrix or sampled positions)."""
    X = syn.from_storage(Xb, fmt).astype(np.float64)
    W = syn.from_storage(Wb, fmt).astype(np.float64)
    if rows is None:
        return X @ W, np.abs(X) @ np.abs(W)
    y = np.einsum("ik,ki->i", X[rows], W[:, cols])
    a = np.einsum("ik,ki->i", np.abs(X[rows]), np.abs(W[:, cols]))
    return y, a


def check_fp32_against_fp64(y_gpu, y64, A, tol=1e-5):
    """Stated tolerance for fp32 outputs: |y_gpu - y64| <= 1e-5 * sum|x_k w_k| per element, and relative
    error <= 1e-3 wherever |y64| >= 0.01 * A (away from cancellation)."""
    err = np.abs(y_gpu.astype(np.float64) - y64)
    assert np.all(err <= tol * A + 1e-300), "max err/A = %g" % float(np.max(err / np.maximum(A, 1e-300)))
    big = np.abs(y64) >= 0.01 * A
    if np.any(big):
        assert np.max(err[big] / np.abs(y64[big])) <= 1e-3


def _bf16_spacing(v, fmt="bf16"):
    """Distance between neighbouring bf16 (or binary16) values at magnitude |v| (fp64 array)."""
    if fmt == "fp16":
        return 2.0 ** (np.floor(np.log2(np.maximum(np.abs(v), 2.0 ** -14))) - 10)
    e = np.floor(np.log2(np.maximum(np.abs(v), 2.0 ** -126)))
    return 2.0 ** (e - 7)


def check_bf16_against_oracle(ybf_gpu, y32_gpu, y32_orc, fmt="bf16"):
    """bf16 outputs (fmt="fp16": binary16 outputs, same statement with that format's spacing).  (1) The GPU's bf16 value is exactly the round-to-nearest-even of the GPU's own fp32
    value (one rounding, at the root).  (2) It equals bf16(oracle fp32) except where a bf16 rounding boundary
    lies between the two fp32 values (widened by one fp32 ulp): there the two roundings may fall on different
    sides, and then they are at most |gpu - oracle| + one bf16 spacing apart -- exactly one bf16 ulp unless the
    value is so close to zero that the fp32 difference itself spans several bf16 steps (cancellation).
    Returns the number of such exceptions."""
    assert np.array_equal(ybf_gpu, syn.to_storage(y32_gpu, fmt))
    want = syn.to_storage(y32_orc, fmt)
    bad = ybf_gpu != want
    n = int(np.count_nonzero(bad))
    if n:
        o = y32_orc[bad].astype(np.float64)
        g = y32_gpu[bad].astype(np.float64)
        ulp32 = 2.0 ** (np.floor(np.log2(np.maximum(np.maximum(np.abs(o), np.abs(g)), 2.0 ** -126))) - 23)
        lo = np.minimum(o, g) - ulp32
        hi = np.maximum(o, g) + ulp32
        # a rounding boundary inside [lo, hi]  <=>  the two ends round to different bf16 values
        assert np.all(syn.to_storage(lo.astype(np.float32), fmt) != syn.to_storage(hi.astype(np.float32), fmt))
        vg = syn.from_storage(ybf_gpu[bad], fmt).astype(np.float64)
        vo = syn.from_storage(want[bad], fmt).astype(np.float64)
        spacing = _bf16_spacing(np.maximum(np.abs(vg), np.abs(vo)), fmt)
        assert np.all(np.abs(vg - vo) <= np.abs(g - o) + spacing)
        near = np.abs(g - o) < 0.25 * _bf16_spacing(np.minimum(np.abs(o), np.abs(g)), fmt)
        same_sign = np.sign(vg) == np.sign(vo)
        step = np.abs(ybf_gpu[bad].astype(np.int64) - want[bad].astype(np.int64))
        assert np.all(step[near & same_sign] == 1)
    return n
