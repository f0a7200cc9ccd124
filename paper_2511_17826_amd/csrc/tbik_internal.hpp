// Host-side declarations shared between the translation units of libtbik.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/tbik.h"

namespace tbik {

// Resolved description of one GEMM request; validated by the C ABI layer before any launch.
struct GemmArgs {
    const uint16_t *X;   // x_dtype [M, ldx] (fp32 and 8-bit operands: the pointer is cast)
    int64_t ldx;
    const uint16_t *W;   // x_dtype [K, ldw]
    int64_t ldw;
    float *partials;     // fp32 [P, M, N] or nullptr
    void *Y;             // [M, ldy] of y_dtype or nullptr
    int64_t ldy;
    int y_dtype;         // tbik_dtype
    int M, N, K;
    int superleaf;       // leaf * k_first
    int ns;              // number of superleaves (power of two)
    int P;               // shards (power of two, <= ns)
    int x_dtype;         // TBIK_BF16, TBIK_F16 or TBIK_F32: storage format of X, W (and of a 16-bit Y)
    int swiglu;          // 1: W is [gate | up], N = 2 I columns; Y is act [M, I] = SiLU(gate) * up in x_dtype.  Only the
                         // 128 x 128 tile of the 16-bit kernels, P == 1, I % 64 == 0 (gemm_tiled_supports() says).
};

// Reference kernel: one wavefront per 32x32 tile and shard.  Writes partials (if set) and, when P == 1
// and Y is set, the rounded output.
hipError_t launch_gemm_reference(const GemmArgs &a, hipStream_t s);

// Tiled kernels.  `variant` selects the tile shape (see kVariantNames); returns hipErrorInvalidValue
// if the variant cannot run this shape.  Same outputs as the reference kernel.
hipError_t launch_gemm_tiled(const GemmArgs &a, int variant, hipStream_t s);
bool gemm_tiled_supports(const GemmArgs &a, int variant);

// act = round16(SiLU(gate) * up), elementwise on [M, I] 16-bit tensors of format dtype.
hipError_t launch_silu_mul(const uint16_t *gate, int64_t ldg, const uint16_t *up, int64_t ldu, uint16_t *act, int64_t lda,
                           int dtype, int M, int I, hipStream_t s);
// The same on the tree-combined partials of a [gate | up] GEMM: partials fp32 [P, M, 2 I]; gate = round16(T(..)[m, i]),
// up = round16(T(..)[m, I + i]).  I % 4 == 0.
hipError_t launch_tree_combine_swiglu(const float *partials, int P, uint16_t *act, int64_t lda, int dtype, int M, int I,
                                      hipStream_t s);

// The same two for fp32 operands (x_dtype TBIK_F32: X and W point to float, Y is fp32); tiles of 128 or 32 rows.
hipError_t launch_gemm_f32_reference(const GemmArgs &a, hipStream_t s);
hipError_t launch_gemm_f32_tiled(const GemmArgs &a, int variant, hipStream_t s);   // variant: tile shape, see kVariantNames
bool gemm_f32_tiled_supports(const GemmArgs &a);

// The same for 8-bit floating-point operands (x_dtype TBIK_FP8_E4M3 or TBIK_FP8_E5M2): X points to [M, ldx] bytes, W
// to the TRANSPOSED weight [N, ldw] bytes; Y is fp32 or bf16.  rows: 128, 64 or 32 rows per workgroup tile.
hipError_t launch_gemm_fp8_reference(const GemmArgs &a, hipStream_t s);
hipError_t launch_gemm_fp8_tiled(const GemmArgs &a, int rows, hipStream_t s);
bool gemm_fp8_tiled_supports(const GemmArgs &a);

// The same for MXFP4 operands (x_dtype TBIK_MXFP4): X points to [M, ldx] BYTES of packed element pairs (ldx >= K / 2),
// W to the transposed weight [N, ldw] bytes; the block scales travel beside.  Y is fp32 or bf16.
struct Mxfp4Scales {
    const uint8_t *Xs;   // [M, ldxs], ldxs >= K / 32
    int64_t ldxs;
    const uint8_t *Ws;   // [N, ldws]
    int64_t ldws;
    int packed = 0;      // set by the tiled launchers only: Xs, Ws point at their re-tiled copies
};
hipError_t launch_gemm_mxfp4_reference(const GemmArgs &a, const Mxfp4Scales &sc, hipStream_t s);
// rows: 128, 64 or 32.  packed_ws: nullptr or mxfp4_retiled_scales_bytes(M, N, K) bytes of device memory for re-tiled scales.
hipError_t launch_gemm_mxfp4_tiled(const GemmArgs &a, const Mxfp4Scales &sc, int rows, void *packed_ws, hipStream_t s);
size_t mxfp4_retiled_scales_bytes(int M, int N, int K);
bool gemm_mxfp4_tiled_supports(const GemmArgs &a, const Mxfp4Scales &sc);

// The same for MXFP8 operands: the 8-bit kernels with one E8M0 scale per block of 32 k beside each operand (a.x_dtype
// names the element format, TBIK_FP8_E4M3 or TBIK_FP8_E5M2; X [M, ldx] bytes, W the transposed weight [N, ldw] bytes).
hipError_t launch_gemm_mxfp8_reference(const GemmArgs &a, const Mxfp4Scales &sc, hipStream_t s);
// rows: 128, 64 or 32.  packed_ws: nullptr or mxfp8_retiled_scales_bytes(M, N, K) bytes of device memory for re-tiled scales.
hipError_t launch_gemm_mxfp8_tiled(const GemmArgs &a, const Mxfp4Scales &sc, int rows, void *packed_ws, hipStream_t s);
size_t mxfp8_retiled_scales_bytes(int M, int N, int K);
bool gemm_mxfp8_tiled_supports(const GemmArgs &a, const Mxfp4Scales &sc);

// The same for MXFP6 operands (a.x_dtype TBIK_FP6_E2M3 or TBIK_FP6_E3M2): X [M, ldx] bytes of packed 6-bit elements
// (ldx >= 3 K / 4), W the transposed weight [N, ldw] bytes; one tile shape, 128 x 128.
hipError_t launch_gemm_mxfp6_reference(const GemmArgs &a, const Mxfp4Scales &sc, hipStream_t s);
hipError_t launch_gemm_mxfp6_tiled(const GemmArgs &a, const Mxfp4Scales &sc, void *packed_ws, hipStream_t s);
bool gemm_mxfp6_tiled_supports(const GemmArgs &a, const Mxfp4Scales &sc);
size_t mxfp6_retiled_scales_bytes(int M, int N, int K);

// Y = T(partials[0..P)) elementwise + one rounding.
hipError_t launch_tree_combine(const float *partials, int P, void *Y, int64_t ldy, int y_dtype, int M, int N,
                               hipStream_t s);

// Alg. 2 round by round on P rank buffers [P, n], in place: afterwards every buffer holds T(buffers).
hipError_t launch_tree_allreduce(float *bufs, int P, int64_t n, hipStream_t s);

// dtype: TBIK_BF16 or TBIK_F16, the format of every 16-bit tensor of the call.
hipError_t launch_rmsnorm(const uint16_t *x, const uint16_t *w, uint16_t *y, int M, int H, float eps, int dtype, hipStream_t s);
hipError_t launch_combine_residual_rmsnorm(const float *partials, int P, const uint16_t *res, const uint16_t *w,
                                           uint16_t *hidden, uint16_t *normed, int M, int H, float eps, int dtype, hipStream_t s);

// Resolved description of one attention call; validated by the C ABI layer.
struct AttnArgs {
    const uint16_t *Q, *K, *V;    // token-major: [tokens, heads, 128]
    uint16_t *O;
    int dtype;                    // TBIK_BF16 or TBIK_F16: the format of Q, K, V and O
    const int32_t *cu_q, *cu_k;   // device, [batch + 1]
    int batch, max_seqlen_q, max_seqlen_k, total_q, total_k;
    int heads_q, heads_kv;
    int64_t q_stride, k_stride, v_stride, o_stride;
    float scale;
    int causal;
    void *workspace;              // attention_workspace(...) bytes or more, or nullptr if that is 0
    size_t workspace_bytes;
};
size_t attention_workspace(int batch, int max_seqlen_q, int max_seqlen_k, int heads_q, int heads_kv);
hipError_t launch_attention(const AttnArgs &a, hipStream_t s);
int set_attention_variant(int v);   // 0 = default, 1 = two workgroups per CU, 2 = two groups of wavefronts taking turns; returns the previous value, -1 if illegal

size_t row_reduce_workspace(int M, int64_t V, int x_dtype, int op);
hipError_t launch_row_reduce(const void *x, int x_dtype, void *out, int op, int M, int64_t V, void *ws, hipStream_t s);
int set_row_wait_limit(int polls);   // returns the previous limit
// The same launches with the library's fixed per-device scratch array (TBIK_STATIC_SCRATCH_BYTES) as workspace; no
// allocation.  The first call on a device looks the array's address up.  The caller has checked that the shape fits.
hipError_t launch_row_reduce_static(const void *x, int x_dtype, void *out, int op, int M, int64_t V, hipStream_t s);

enum { VARIANT_AUTO = 0, VARIANT_REFERENCE = 1, VARIANT_T128 = 2, VARIANT_T32 = 3, VARIANT_T64 = 4, VARIANT_COUNT = 5 };

}  // namespace tbik
