"""MI355X-native Tree-Based Invariant Kernels (TBIK): HIP kernels behind a C ABI, plus a thin binding.

``binding``   the Python face of ``libtbik.so`` (same names as ``include/tbik.h``)
``synthetic`` seeded input generators shared by the tests, the benchmark and the CPU oracle's tests
``build``     compiles the library in-tree with hipcc for gfx950
"""
from .binding import (  # noqa: F401
    TBIK_BF16, TBIK_F16, TBIK_F32, TBIK_LOGSOFTMAX, TBIK_MAX, TBIK_SUM, TbikError, attention_workspace_bytes, gemm_workspace_bytes, lib,
    tbik_attention, tbik_attention_f16, tbik_combine_residual_rmsnorm, tbik_combine_residual_rmsnorm_f16, tbik_gemm, tbik_gemm_f16, tbik_gemm_f32, tbik_gemm_reference, tbik_gemm_reference_f32, tbik_gemm_reference_f16,
    tbik_gemm_shard_partials, tbik_gemm_shard_partials_f16, tbik_gemm_shard_partials_f32, tbik_rmsnorm, tbik_rmsnorm_f16, tbik_row_reduce,
    tbik_set_gemm_variant, tbik_tree_combine, variant_names,
)
