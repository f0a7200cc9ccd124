/*
 * tbik.h -- C ABI of the Tree-Based Invariant Kernels (TBIK) for AMD MI355X (gfx950).
 *
 * The library computes matrix products and row reductions whose floating-point
 * summation order is one fixed binary tree, so that the output bits do not depend
 * on the batch size M, on the position of a row in the batch, or on the number P
 * of tensor-parallel shards the reduction dimension K is split into; and attention
 * with a fixed key tile, whose bits do not depend on how queries are batched.
 * Operands are bf16, fp16 or (matrix products) fp32; all accumulation is fp32.
 *
 * Vocabulary (Sec. 4.2, App. D.1):
 *   leaf        number of consecutive K-elements in one tile of the K dimension (Block_K)
 *   k_first     number of leaves accumulated in one chain before the first tree level (K_first)
 *               0 selects the odd part of K / leaf, the smallest value that leaves a power of two of superleaves
 *   superleaf   leaf * k_first consecutive k; its products are accumulated in ascending k from +0
 *   n_s         K / (leaf * k_first), the number of superleaves; must be a power of two
 *   P           number of K-shards (the tensor-parallel size C); a power of two, P <= n_s
 *   T(...)      the full-binary-tree reduction of App. C over the n_s superleaf sums
 *
 * Conventions for every call
 *   - All data pointers are DEVICE pointers owned by the caller.  The library never
 *     allocates, frees or keeps device memory; scratch space is passed in as `workspace`.
 *   - Matrices are row-major; leading dimensions (ld*) are in ELEMENTS.
 *   - bf16 is the 16-bit brain-float storage format (upper half of an IEEE binary32); fp16 is IEEE binary16.
 *   - `hip_stream` is a hipStream_t cast to void* (NULL = the default stream).  All work is
 *     enqueued on it; no call synchronises.  Outputs are valid once the stream reaches that point.
 *   - Every call returns a tbik_status.  Arguments are validated before the first launch,
 *     so a failing call has launched nothing.  M == 0 or N == 0 (V == 0 rows excepted, see
 *     tbik_row_reduce) is TBIK_OK and does nothing.
 *   - Determinism contract: for fixed (leaf, k_first) the bits of row m of an output depend only
 *     on row m of the input and on the weights -- not on M, the row's position, P, the stream,
 *     the internal kernel variant or the number of repetitions; and
 *     tbik_gemm(...) == tbik_tree_combine(tbik_gemm_shard_partials(..., P)) bit for bit for
 *     every legal P (Theorem 1, App. C).
 */
#ifndef TBIK_H
#define TBIK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    TBIK_OK = 0,
    TBIK_ERR_NULL = 1,        /* a required pointer is NULL                                             */
    TBIK_ERR_SHAPE = 2,       /* negative size; K % (leaf*k_first) != 0; n_s not a power of two;
                                 leaf*k_first not a multiple of 16; a leading dimension too small      */
    TBIK_ERR_SHARDS = 3,      /* P < 1, P not a power of two, P > n_s, or P > TBIK_MAX_SHARDS           */
    TBIK_ERR_DTYPE = 4,       /* unknown tbik_dtype / tbik_rowop, or a combination that is not offered */
    TBIK_ERR_ALIGN = 5,       /* a pointer or leading dimension violates the stated alignment          */
    TBIK_ERR_WORKSPACE = 6,   /* workspace missing or smaller than the matching *_workspace_bytes()    */
    TBIK_ERR_UNSUPPORTED = 7, /* legal request that this build does not implement                      */
    TBIK_ERR_HIP = 8          /* a HIP runtime call failed; see tbik_last_hip_error()                  */
} tbik_status;

typedef enum {
    TBIK_F32 = 0, TBIK_BF16 = 1, TBIK_F16 = 2,
    TBIK_FP8_E4M3 = 3,        /* OCP 8-bit float, 4 exponent / 3 fraction bits, bias 7, no infinities, max 448 */
    TBIK_FP8_E5M2 = 4,        /* OCP 8-bit float, 5 exponent / 2 fraction bits, bias 15, IEEE-style inf / NaN  */
    TBIK_MXFP4 = 5,           /* OCP MXFP4: 4-bit E2M1 elements, one E8M0 scale per block of 32 consecutive k     */
    TBIK_FP6_E2M3 = 6,        /* OCP 6-bit float, 2 exponent / 3 fraction bits, bias 1, no infinities or NaN, max 7.5 */
    TBIK_FP6_E3M2 = 7         /* OCP 6-bit float, 3 exponent / 2 fraction bits, bias 3, no infinities or NaN, max 28  */
} tbik_dtype;
typedef enum { TBIK_SUM = 0, TBIK_MAX = 1, TBIK_LOGSOFTMAX = 2 } tbik_rowop;

#define TBIK_MAX_SHARDS 64

/*
 * Y[M,N] = X[M,K] * W[K,N] with the whole K on this device (tensor-parallel size 1, the
 * training-side call).  Sec. 3.3 states the product; Sec. 4.2 and App. D.1 (Alg. 1) state the
 * order: per output element, each superleaf's bf16 x bf16 products are accumulated in fp32 in
 * ascending k starting from +0, and the n_s superleaf sums are combined by T (App. C).  The
 * result is rounded once to y_dtype (round-to-nearest-even for TBIK_BF16).
 *
 *   X   device, bf16, [M, ldx], ldx >= K     W   device, bf16, [K, ldw], ldw >= N
 *   Y   device, y_dtype, [M, ldy], ldy >= N
 *   Alignment: X, W 16 bytes, ldx and ldw multiples of 8; Y 4 bytes (TBIK_F32) / 2 bytes (TBIK_BF16).
 *   workspace  device scratch of at least tbik_gemm_workspace_bytes(M,N,K,leaf,k_first) bytes,
 *              256-byte aligned; may be NULL when that size is 0.  Contents are undefined afterwards.
 * Errors: NULL, SHAPE, DTYPE, ALIGN, WORKSPACE, HIP.
 */
int tbik_gemm(const void *X, int64_t ldx, const void *W, int64_t ldw, void *Y, int64_t ldy,
              tbik_dtype y_dtype, int M, int N, int K, int leaf, int k_first,
              void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Tensor-parallel emulation, local stage (Sec. 3.3 row-parallel split; Sec. 4.2 "Intra-GPU
 * reduction"): shard p owns k in [p*K/P, (p+1)*K/P), i.e. n_s/P whole superleaves, and
 *   partials[p][m][n] = T(superleaf sums of shard p)            (fp32, never rounded to bf16)
 * which is exactly what rank p of a P-way tensor-parallel group would hold before the
 * all-reduce.  A real rank calls this with P = 1 on its own X_p [M, K/P], W_p [K/P, N].
 *
 *   partials   device, fp32, dense [P, M, N]
 *   workspace  at least tbik_gemm_workspace_bytes(...) bytes (same rule as tbik_gemm)
 * Errors: NULL, SHAPE, SHARDS, ALIGN, WORKSPACE, HIP.
 */
int tbik_gemm_shard_partials(const void *X, int64_t ldx, const void *W, int64_t ldw, float *partials,
                             int M, int N, int K, int leaf, int k_first, int P,
                             void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Tensor-parallel emulation, top of the tree (Sec. 4.2 "Inter-GPU reduction"; App. D.2, Alg. 2):
 *   Y = T(partials[0], ..., partials[P-1]) elementwise, in the order of Alg. 2's reduce phase
 * (level l adds buffer r + 2^l into buffer r for r mod 2^(l+1) == 0), followed by the one
 * rounding to y_dtype.  The partial buffers stand in for what the ranks would exchange.
 *
 *   partials   device, fp32, dense [P, M, N], 16-byte aligned     Y   device, [M, ldy], ldy >= N
 *   y_dtype    TBIK_F32, TBIK_BF16 or TBIK_F16 (both 16-bit roundings are to nearest, ties to even)
 * Errors: NULL, SHAPE, SHARDS, DTYPE, ALIGN, HIP.
 */
int tbik_tree_combine(const float *partials, int P, void *Y, int64_t ldy, tbik_dtype y_dtype,
                      int M, int N, void *hip_stream);

/*
 * The tree all-reduce of App. D.2 (Alg. 2) taken literally on one GPU: the P buffers stand for the ranks' tensors, a
 * send/receive pair is a read of the partner's buffer.  Reduce phase: in round l = 0 .. log2(P) - 1 every rank r with
 * r mod 2^(l+1) == 0 adds the buffer of rank r + 2^l to its own (own + received) and that partner drops out; broadcast
 * phase: the same pairs in reverse order, the receiver copying.  Afterwards every buffer holds T(buffers), the value
 * tbik_tree_combine gives before its rounding -- in 2 log2(P) rounds (one launch each) instead of one pass, which is
 * what the wire protocol would do and what it costs to do it that way in memory.
 *
 *   bufs   device, fp32, dense [P, n], 16-byte aligned, updated in place; rows of n elements must keep that alignment
 *          for the vector path (n % 4 == 0), any n works
 * Errors: NULL, SHAPE, SHARDS, ALIGN, HIP.
 */
int tbik_tree_allreduce(float *bufs, int P, int64_t n, void *hip_stream);

/*
 * The gated activation between the two GEMMs of the MLP block (implementation appendix, "other kernels":
 * SiLU is one of the position-wise kernels that every configuration shares):
 *   act[m][i] = round16( SiLU(gate[m][i]) * up[m][i] ),   SiLU(g) = g / (1 + e^-g)
 * in fp32: e^-g and the reciprocal are the hardware's approximate instructions (about one fp32 ulp each), the two
 * products are rounded multiplications, and the result is rounded once to the tensors' format.  An output is one of
 * the two 16-bit neighbours of the exact value (nearly always the nearest); for gate below about -87 it may be zero
 * where the exact value is below 1e-36 in magnitude.  Position-wise: an element's bits depend on its own gate and up
 * only, and every entry point of this library that applies the activation gives the same bits.
 *
 *   gate, up, act   device, 16-bit of format `dtype` (TBIK_BF16 or TBIK_F16), [M, I] with leading dimensions
 *                   ldg, ldu, lda >= I; gate and up may be the two halves of one [M, 2 I] buffer; act may not
 *                   overlap them unless it is exactly gate or exactly up with the same leading dimension
 *   16-byte aligned pointers, I and leading dimensions multiples of 8 take the vector path; anything else works.
 * Errors: NULL, SHAPE, DTYPE, HIP.
 */
int tbik_silu_mul(const void *gate, int64_t ldg, const void *up, int64_t ldu, void *act, int64_t lda,
                  tbik_dtype dtype, int M, int I, void *hip_stream);

/*
 * The first GEMM of the MLP block with the activation applied before anything is stored (Sec. 3.3: gate_proj and
 * up_proj are column-parallel, each output element is a whole-K sum; Sec. 4.2 / App. D.1 for the order of that sum):
 *   gate = round16( X W_gu[:, 0:I] ),  up = round16( X W_gu[:, I:2I] )     each exactly tbik_gemm's output for that half
 *   act  = tbik_silu_mul(gate, up)                                         bit for bit
 * gate and up are never stored as 16-bit tensors: for batches that fill the chip with 128-row tiles the activation is
 * the GEMM kernel's epilogue (the fp32 accumulators of a channel's gate and up columns sit in one lane); for a K split
 * it is applied by the kernel that combines the fp32 partial sums; other shapes pass through the workspace.  The bits
 * of row m of act depend only on row m of X and on W_gu, as for tbik_gemm.
 *
 *   X      device, 16-bit, [M, ldx], ldx >= K          W_gu   device, 16-bit, [K, ldw], ldw >= 2 I: gate columns, then up
 *   act    device, 16-bit, [M, lda], lda >= I          dtype  TBIK_BF16 or TBIK_F16: the format of all three
 *   I      a multiple of 8; ldx, ldw below 2^22
 *   workspace  device, 256-byte aligned, at least tbik_gemm_swiglu_workspace_bytes(...) bytes (may be NULL if that is 0)
 *   Alignment as for tbik_gemm; act 2 bytes (16 bytes and lda % 8 == 0 for vector stores).
 * Errors: NULL, SHAPE, DTYPE, ALIGN, WORKSPACE, HIP.
 */
size_t tbik_gemm_swiglu_workspace_bytes(int M, int I, int K, int leaf, int k_first);
int tbik_gemm_swiglu(const void *X, int64_t ldx, const void *W_gu, int64_t ldw, void *act, int64_t lda,
                     tbik_dtype dtype, int M, int I, int K, int leaf, int k_first,
                     void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Batch-invariant RMSNorm (App. B: every row is reduced on its own in a fixed order), with the
 * tree order of App. C along the row:
 *   ss = TreeSum_i(x_i^2),  r = 1 / sqrt(ss / H + eps),  y_i = bf16((x_i * r) * w_i)
 * TreeSum: leaves are in-order fp32 sums of 8 consecutive elements (16 bytes of bf16), the leaf
 * count is padded with +0 leaves to a power of two, then T.  All arithmetic in fp32, one
 * rounding to bf16 at the end.
 *
 *   x, y   device, bf16, dense [M, H]     weight   device, bf16, [H]
 *   Alignment: x, y, weight 16 bytes; H a multiple of 8.  H <= 65536.
 * Errors: NULL, SHAPE, ALIGN, HIP.
 */
int tbik_rmsnorm(const void *x, const void *weight, void *y, int M, int H, float eps, void *hip_stream);

/*
 * Fused tail of a row-parallel layer (a fusion that keeps the determinism contract): what a decoder layer does
 * with the tree all-reduce's result (Sec. 3.3, Alg. 2) before the next block,
 *   Y = bf16(T(partials[0..P)))      exactly tbik_tree_combine with a bf16 output,
 *   Hd = bf16(Y + R)                 the residual add in fp32, rounded once,
 *   O = RMSNorm(Hd; weight, eps)     exactly tbik_rmsnorm,
 * in one pass over the partials.  The bits of Hd and O are those of the three steps done one after the other.
 *
 *   partials   device, fp32, dense [P, M, H]         residual   device, bf16, dense [M, H]
 *   weight     device, bf16, [H]                     hidden, normed   device, bf16, dense [M, H] (written)
 *   hidden may be the same buffer as residual (updated in place); normed may not share a buffer with either.
 *   P a power of two, P <= 16 (larger legal P: TBIK_ERR_UNSUPPORTED).  H a multiple of 8, H <= 65536; 16-byte alignment.
 * Errors: NULL, SHAPE, SHARDS, UNSUPPORTED, ALIGN, HIP.
 */
int tbik_combine_residual_rmsnorm(const float *partials, int P, const void *residual, const void *weight, float eps,
                                  void *hidden, void *normed, int M, int H, void *hip_stream);

/*
 * Batch-invariant row reductions over dense rows x[M, V] (App. B; softmax in fp32 per Sec. 2.1):
 *   TBIK_SUM         out[m]   = TreeSum_i x[m,i]                                   out fp32 [M]
 *   TBIK_MAX         out[m]   = max_i x[m,i]                                       out fp32 [M]
 *   TBIK_LOGSOFTMAX  out[m,i] = (x[m,i] - mx) - log(TreeSum_j exp(x[m,j] - mx)),   out fp32 [M, V]
 *                    mx = max_j x[m,j]
 * TreeSum leaves are in-order fp32 sums of one 16-byte chunk of the row (4 fp32 or 8 bf16 or fp16
 * elements; the last leaf may be short), padded with +0 leaves to a power of two, then T.
 * x_dtype TBIK_BF16 and TBIK_F16 inputs are widened to fp32 first (exact).  V == 0 is TBIK_ERR_SHAPE.
 *
 *   x          device, x_dtype, dense [M, V], 16-byte aligned, V a multiple of 4 (fp32) / 8 (bf16, fp16)
 *   workspace  at least tbik_row_reduce_workspace_bytes(M, V, op) bytes, 256-byte aligned
 * Errors: NULL, SHAPE, DTYPE, ALIGN, WORKSPACE, HIP.
 */
int tbik_row_reduce(const void *x, tbik_dtype x_dtype, void *out, tbik_rowop op, int M, int64_t V,
                    void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * tbik_row_reduce for callers that cannot allocate device memory and have no workspace to pass: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, kernels, results (bit for
 * bit) and errors as tbik_row_reduce, except that the scratch is a fixed array of TBIK_STATIC_SCRATCH_BYTES inside
 * the library's device code, one copy per GPU, held until the process ends.  The call allocates and frees nothing.
 *   - A shape whose tbik_row_reduce_workspace_bytes(M, V, op) exceeds TBIK_STATIC_SCRATCH_BYTES is refused with
 *     TBIK_ERR_WORKSPACE and nothing is launched (log-softmax over V = 151936 fp32 logits fits up to 10000 rows).
 *   - The first call on a device looks the array's address up (with that device current); a call with M == 0 does
 *     only that, so a caller can make one before it starts capturing a graph.
 *   - All calls on one GPU share the one array, which keeps the previous call's contents; every call clears what
 *     it needs at zero itself.  Calls that overlap in time on one GPU (different streams) race: order them.
 */
#define TBIK_STATIC_SCRATCH_BYTES (4u << 20)
int tbik_row_reduce_static(const void *x, tbik_dtype x_dtype, void *out, tbik_rowop op, int M, int64_t V,
                           void *hip_stream);

/*
 * Batch-invariant attention on packed variable-length sequences (implementation appendix, "Framework Modifications
 * for vLLM and FSDP": the attention kernel uses a FIXED tile size, prefill and decode run the same kernel, and the
 * serving stack's decode-side optimisations are off; Sec. 2.1: fp32 accumulators).  For sequence b, query head h, query i (of Lq = cu_q[b+1] - cu_q[b] queries, which
 * are the LAST Lq positions of a sequence with Lk = cu_k[b+1] - cu_k[b] keys):
 *     O = softmax_j( scale * q . k_j ) applied to v_j  over the visible keys j,
 *     visible: j < Lk and (causal == 0 or j <= i + Lk - Lq);   a query that sees no key gives 0.
 * Order of the arithmetic (fixed, part of the contract): keys in tiles of 64 at absolute positions [64 t, 64 t + 64),
 * ascending; per tile the streaming-softmax step in fp32 with base-2 exponentials (scores scaled by
 * scale * log2 e), the tile's weights rounded to bf16 for the product with V, fp32 accumulation; one division by
 * the sum of weights and one rounding to bf16 at the end.  Beyond 4096 keys the key axis is also cut into SPLITS of 64
 * tiles at absolute positions: each split runs the recurrence from the empty state, and the splits' states (running
 * maximum m, sum l, accumulator o) are folded in ascending order by
 *     M = max(mA, mB);  a = exp2(mA - M), b = exp2(mB - M);  l = fl(lA a) + fl(lB b);  o = fl(oA a) + fl(oB b).
 * (Where the paper turns the split of the key axis off to keep decode and prefill identical, a fixed split in every
 * phase keeps them identical too and lets the splits of a long sequence be computed at once: a decode step on few
 * long sequences then runs one workgroup per split and a second kernel for the fold; bigger calls let each workgroup
 * walk its splits itself.  Same bits either way.)  The bits of a query's output depend only on its own
 * row of Q and on the keys and values it sees -- not on the batch, on the number of queries per sequence in the
 * call (prefill, decode step, chunk), or on the query's position in the packed tensor.
 *
 *   Q, O   device, bf16, token t / head h / channel d at [t * stride + h * head_dim + d]; Q has heads_q heads
 *   K, V   device, bf16, same layout with heads_kv heads; query head h reads key/value head h / (heads_q / heads_kv)
 *   cu_seqlens_q, cu_seqlens_k   DEVICE, int32 [batch + 1], non-decreasing prefix sums of the sequences' query and key
 *          counts; values are clamped to [0, total_q] / [0, total_k] inside the kernel
 *   max_seqlen_q   at least the largest Lq: batch x max_seqlen_q bounds the tokens the launch and the workspace are sized
 *          for (with a smaller value the last queries of the call may be left unwritten); never the bits;
 *   max_seqlen_k   at least the largest Lk (keys of a sequence past it are left out); decides the workspace and how the
 *          call is cut into workgroups, never the bits; values above total_k are taken as total_k
 *          total_q, total_k: tokens in Q/O and in K/V
 *   workspace   at least tbik_attention_workspace_bytes(batch, max_seqlen_q, max_seqlen_k, heads_q, heads_kv) bytes,
 *          256-byte aligned; that is 0 (and the pointer may be NULL) when max_seqlen_k <= 4096, else 68 KiB per
 *          128 rows of (query, head) of batch x max_seqlen_q tokens and -- below 512 such blocks -- per split of
 *          max_seqlen_k, but never more than 4608 x 68 KiB = 306 MiB (for the usual head counts): a call with more
 *          blocks than that is launched in pieces that take turns at the area.  Contents on entry do not matter; calls
 *          that share a workspace must not overlap in time
 *   head_dim 128 (other values: TBIK_ERR_UNSUPPORTED); heads_q a multiple of heads_kv; strides in elements, multiples
 *   of 8, at least heads * head_dim, below 2^24; pointers 16-byte aligned.  O must not overlap Q, K or V.
 * Errors: NULL, SHAPE, UNSUPPORTED, ALIGN, WORKSPACE, HIP.
 */
int tbik_attention(const void *Q, const void *K, const void *V, void *O,
                   const int32_t *cu_seqlens_q, const int32_t *cu_seqlens_k, int batch, int max_seqlen_q, int max_seqlen_k,
                   int total_q, int total_k, int heads_q, int heads_kv, int head_dim,
                   int64_t q_stride, int64_t k_stride, int64_t v_stride, int64_t o_stride,
                   float scale, int causal, void *workspace, size_t workspace_bytes, void *hip_stream);
size_t tbik_attention_workspace_bytes(int batch, int max_seqlen_q, int max_seqlen_k, int heads_q, int heads_kv);

/*
 * tbik_attention for IEEE binary16 tensors: Q, K, V and O are fp16; the scores, the softmax state and the output
 * accumulators are fp32 as above, the tile's weights are rounded to fp16 for the product with V (to nearest-even, on
 * the subnormal grid of 2^-24 below 2^-14, so a weight below 2^-25 of the running maximum's contributes nothing),
 * and O takes one rounding to fp16.  Same tile, splits, order, arguments, workspace, limits and errors.
 */
int tbik_attention_f16(const void *Q, const void *K, const void *V, void *O,
                       const int32_t *cu_seqlens_q, const int32_t *cu_seqlens_k, int batch, int max_seqlen_q, int max_seqlen_k,
                       int total_q, int total_k, int heads_q, int heads_kv, int head_dim,
                       int64_t q_stride, int64_t k_stride, int64_t v_stride, int64_t o_stride,
                       float scale, int causal, void *workspace, size_t workspace_bytes, void *hip_stream);

/* Scratch sizes (pure host functions; 0 if the arguments are illegal or no scratch is needed).
 * tbik_gemm_workspace_bytes covers tbik_gemm and tbik_gemm_shard_partials for any legal P. */
size_t tbik_gemm_workspace_bytes(int M, int N, int K, int leaf, int k_first);
size_t tbik_row_reduce_workspace_bytes(int M, int64_t V, tbik_rowop op);

/* Reference kernel of tbik_gemm_shard_partials / tbik_gemm: one wavefront per 32x32 output tile,
 * operands read straight from global memory, no workspace.  Slow, but its schedule is trivially
 * independent of M and P; the tuned kernels must reproduce its bits.  Same arguments and errors
 * as tbik_gemm_shard_partials; with y != NULL and P == 1 it also writes the rounded output. */
int tbik_gemm_reference(const void *X, int64_t ldx, const void *W, int64_t ldw, float *partials,
                        void *Y, int64_t ldy, tbik_dtype y_dtype,
                        int M, int N, int K, int leaf, int k_first, int P, void *hip_stream);

/*
 * The same three calls for fp16 operands (the kernel table of the paper, "Block size setting for TBIK", lists FP16
 * beside BF16 with the same blocks; Sec. 4.2, App. C and App. D.1 do not depend on the storage format):
 * X and W hold IEEE binary16 values (subnormals included), every product is exact in fp32, the order of the
 * fp32 additions is the one stated for tbik_gemm, and y_dtype is TBIK_F32 or TBIK_F16 (one rounding to
 * nearest-even; overflow gives infinity).  Arguments, alignment, workspace rule (tbik_gemm_workspace_bytes),
 * determinism contract and errors are those of tbik_gemm, tbik_gemm_shard_partials and tbik_gemm_reference;
 * partials of fp16 operands are combined by tbik_tree_combine like any others.
 */
int tbik_gemm_f16(const void *X, int64_t ldx, const void *W, int64_t ldw, void *Y, int64_t ldy,
                  tbik_dtype y_dtype, int M, int N, int K, int leaf, int k_first,
                  void *workspace, size_t workspace_bytes, void *hip_stream);
int tbik_gemm_shard_partials_f16(const void *X, int64_t ldx, const void *W, int64_t ldw, float *partials,
                                 int M, int N, int K, int leaf, int k_first, int P,
                                 void *workspace, size_t workspace_bytes, void *hip_stream);
int tbik_gemm_reference_f16(const void *X, int64_t ldx, const void *W, int64_t ldw, float *partials,
                            void *Y, int64_t ldy, tbik_dtype y_dtype,
                            int M, int N, int K, int leaf, int k_first, int P, void *hip_stream);

/*
 * The same three calls for fp32 operands (third row of that kernel table).  X and W hold IEEE binary32 values and Y
 * is fp32.  The product of two fp32 numbers is not exact in fp32 and the paper does not say how a leaf accumulates
 * then; this library's definition: one fused multiply-add per k (a single rounding of x*w + acc), in ascending k
 * from +0 inside a superleaf -- the fp32 matrix instruction computes exactly that chain, and so does fmaf on a CPU --
 * and above the superleaves the tree stated for tbik_gemm.  (For operands that happen to be bf16 or fp16 numbers every
 * product is exact and the chain is the plain left-to-right fp32 sum; the 16-bit calls add the 16 products of a matrix
 * instruction in that instruction's own fixed order, so their fp32 output agrees with it closely, not bit for bit.)
 * ldx and ldw are multiples of 4 here (16 bytes); the other
 * arguments, the workspace rule (tbik_gemm_workspace_bytes), the determinism contract and the errors are those of
 * tbik_gemm, tbik_gemm_shard_partials and tbik_gemm_reference.  Superleaves that are not a multiple of 32 run on the
 * reference kernel.
 */
int tbik_gemm_f32(const void *X, int64_t ldx, const void *W, int64_t ldw, void *Y, int64_t ldy,
                  int M, int N, int K, int leaf, int k_first,
                  void *workspace, size_t workspace_bytes, void *hip_stream);
int tbik_gemm_shard_partials_f32(const void *X, int64_t ldx, const void *W, int64_t ldw, float *partials,
                                 int M, int N, int K, int leaf, int k_first, int P,
                                 void *workspace, size_t workspace_bytes, void *hip_stream);
int tbik_gemm_reference_f32(const void *X, int64_t ldx, const void *W, int64_t ldw, float *partials,
                            void *Y, int64_t ldy, int M, int N, int K, int leaf, int k_first, int P, void *hip_stream);

/*
 * The same three calls for 8-bit floating-point operands (the paper's outlook, "Limitations and future work": bringing
 * the guarantee to quantised types).  X and the weight hold OCP E4M3 or E5M2 patterns (`x_dtype`, the same for both),
 * widened exactly.  A product of two of them has at most 8 significant bits and is exact in fp32, so the order contract
 * of tbik_gemm carries over word for word: per output element each superleaf's products are accumulated in fp32 in
 * ascending k from +0, the superleaf sums are combined by T, the result is rounded once.  (As with the 16-bit calls, the
 * 64 products of one matrix instruction are added in that instruction's own fixed order: for 8-bit operands a chain of
 * four fp32-rounded steps of 16 consecutive k in ascending order, for the 6- and 4-bit formats below two steps of 32,
 * each step a fixed-point sum that keeps 13 bits below the largest product of every eight and 31 bits below its top.)
 * Scales of a quantisation scheme are outside this call: they multiply the output.
 *
 * The weight is taken TRANSPOSED: Wt [N, ldwt], ldwt >= K, one row per output channel, k contiguous -- the layout 8-bit
 * weights are stored in, and the one the matrix instruction wants for both operands.
 *
 *   X    device, 8-bit, [M, ldx], ldx >= K         Wt   device, 8-bit, [N, ldwt], ldwt >= K
 *   Y    device, y_dtype (TBIK_F32 or TBIK_BF16), [M, ldy], ldy >= N        partials  device, fp32, dense [P, M, N]
 *   leaf * k_first a multiple of 64 (128 for the tiled kernel; else the reference kernel runs); ldx, ldwt multiples
 *   of 16; X, Wt 16-byte aligned; the other alignment rules, the workspace rule (tbik_gemm_fp8_workspace_bytes), the
 *   determinism contract and the errors are those of tbik_gemm, tbik_gemm_shard_partials and tbik_gemm_reference.
 */
size_t tbik_gemm_fp8_workspace_bytes(int M, int N, int K, int leaf, int k_first);
int tbik_gemm_fp8(const void *X, int64_t ldx, const void *Wt, int64_t ldwt, void *Y, int64_t ldy,
                  tbik_dtype y_dtype, tbik_dtype x_dtype, int M, int N, int K, int leaf, int k_first,
                  void *workspace, size_t workspace_bytes, void *hip_stream);
int tbik_gemm_shard_partials_fp8(const void *X, int64_t ldx, const void *Wt, int64_t ldwt, float *partials,
                                 tbik_dtype x_dtype, int M, int N, int K, int leaf, int k_first, int P,
                                 void *workspace, size_t workspace_bytes, void *hip_stream);
int tbik_gemm_reference_fp8(const void *X, int64_t ldx, const void *Wt, int64_t ldwt, float *partials,
                            void *Y, int64_t ldy, tbik_dtype y_dtype, tbik_dtype x_dtype,
                            int M, int N, int K, int leaf, int k_first, int P, void *hip_stream);

/*
 * The same three calls for OCP MXFP4 operands (microscaling: the low-bit format this GPU generation multiplies at four
 * times the bf16 rate).  An element is a 4-bit E2M1 number (0, 0.5, 1, 1.5, 2, 3, 4, 6 and their negatives) times
 * 2^(s - 127), s the E8M0 scale byte of its block of 32 consecutive k (s = 255, NaN, is out of contract).  Two elements
 * share a byte, the one with the even k in the low four bits.  A product of two elements has at most four significant
 * bits and a power-of-two scale, so it is exact in fp32 (as long as it stays in range) and the order contract of
 * tbik_gemm holds word for word: per output element each superleaf's products are accumulated in fp32 in ascending k
 * from +0, the superleaf sums are combined by T, the result is rounded once.  (The 64 products of one matrix instruction
 * are added in that instruction's own fixed order, as for the other formats.)
 *
 * The packing runs along k, so the weight is taken TRANSPOSED: one row per output channel.
 *
 *   X    device, [M, ldx] bytes, ldx >= K / 2        Xs   device, [M, ldxs] scale bytes, ldxs >= K / 32
 *   Wt   device, [N, ldwt] bytes, ldwt >= K / 2      Ws   device, [N, ldws] scale bytes, ldws >= K / 32
 *   Y    device, y_dtype (TBIK_F32 or TBIK_BF16), [M, ldy], ldy >= N        partials  device, fp32, dense [P, M, N]
 *   leaf * k_first a multiple of 64 (256 for the tiled kernel; else the reference kernel runs); K a multiple of 64;
 *   X, Wt 16-byte aligned with ldx, ldwt multiples of 16; Xs, Ws 8-byte aligned with ldxs, ldws multiples of 8 (the
 *   tiled kernel; the reference kernel takes any); the workspace rule (tbik_gemm_mxfp4_workspace_bytes: from 128 rows on
 *   it includes room for a copy of the scales in the order the kernel reads them, which tbik_gemm_mxfp4 makes first), the
 *   determinism contract and the errors are those of tbik_gemm, tbik_gemm_shard_partials and tbik_gemm_reference.
 */
size_t tbik_gemm_mxfp4_workspace_bytes(int M, int N, int K, int leaf, int k_first);
int tbik_gemm_mxfp4(const void *X, int64_t ldx, const void *Xs, int64_t ldxs, const void *Wt, int64_t ldwt,
                    const void *Ws, int64_t ldws, void *Y, int64_t ldy, tbik_dtype y_dtype,
                    int M, int N, int K, int leaf, int k_first,
                    void *workspace, size_t workspace_bytes, void *hip_stream);
int tbik_gemm_shard_partials_mxfp4(const void *X, int64_t ldx, const void *Xs, int64_t ldxs, const void *Wt, int64_t ldwt,
                                   const void *Ws, int64_t ldws, float *partials,
                                   int M, int N, int K, int leaf, int k_first, int P,
                                   void *workspace, size_t workspace_bytes, void *hip_stream);
int tbik_gemm_reference_mxfp4(const void *X, int64_t ldx, const void *Xs, int64_t ldxs, const void *Wt, int64_t ldwt,
                              const void *Ws, int64_t ldws, float *partials, void *Y, int64_t ldy, tbik_dtype y_dtype,
                              int M, int N, int K, int leaf, int k_first, int P, void *hip_stream);

/*
 * The same three calls for OCP MXFP8 operands (quantised types of the paper's "Limitations and future work"; the order
 * contract is that of Sec. 4.2, App. C and App. D.1 as stated for tbik_gemm).  An element is an 8-bit float of format
 * x_dtype (TBIK_FP8_E4M3 or TBIK_FP8_E5M2, as for tbik_gemm_fp8) times 2^(s - 127), s the E8M0 scale byte of its block
 * of 32 consecutive k (s = 255, NaN, is out of contract).  A product has at most eight significant bits and a
 * power-of-two scale, so it is exact in fp32 (as long as it stays in range): per output element each superleaf's
 * products are accumulated in fp32 in ascending k from +0, the superleaf sums are combined by T, the result is rounded
 * once.  (The 64 products of one matrix instruction are added in that instruction's own fixed order, as for the other
 * formats.)  The scales run along k, so the weight is taken TRANSPOSED: one row per output channel.
 *
 *   X    device, [M, ldx] bytes, ldx >= K            Xs   device, [M, ldxs] scale bytes, ldxs >= K / 32
 *   Wt   device, [N, ldwt] bytes, ldwt >= K          Ws   device, [N, ldws] scale bytes, ldws >= K / 32
 *   Y    device, y_dtype (TBIK_F32 or TBIK_BF16), [M, ldy], ldy >= N        partials  device, fp32, dense [P, M, N]
 *   leaf * k_first a multiple of 64 (128 for the tiled kernel; else the reference kernel runs); X, Wt 16-byte aligned
 *   with ldx, ldwt multiples of 16; Xs, Ws 4-byte aligned with ldxs, ldws multiples of 4 (the tiled kernel; the
 *   reference kernel takes any); the workspace rule (tbik_gemm_mxfp8_workspace_bytes: from 128 rows on it includes room
 *   for a copy of the scales in the order the kernel reads them, which tbik_gemm_mxfp8 makes first), the determinism
 *   contract and the errors are those of tbik_gemm, tbik_gemm_shard_partials and tbik_gemm_reference.
 */
size_t tbik_gemm_mxfp8_workspace_bytes(int M, int N, int K, int leaf, int k_first);
int tbik_gemm_mxfp8(const void *X, int64_t ldx, const void *Xs, int64_t ldxs, const void *Wt, int64_t ldwt,
                    const void *Ws, int64_t ldws, void *Y, int64_t ldy, tbik_dtype y_dtype, tbik_dtype x_dtype,
                    int M, int N, int K, int leaf, int k_first,
                    void *workspace, size_t workspace_bytes, void *hip_stream);
int tbik_gemm_shard_partials_mxfp8(const void *X, int64_t ldx, const void *Xs, int64_t ldxs, const void *Wt, int64_t ldwt,
                                   const void *Ws, int64_t ldws, float *partials, tbik_dtype x_dtype,
                                   int M, int N, int K, int leaf, int k_first, int P,
                                   void *workspace, size_t workspace_bytes, void *hip_stream);
int tbik_gemm_reference_mxfp8(const void *X, int64_t ldx, const void *Xs, int64_t ldxs, const void *Wt, int64_t ldwt,
                              const void *Ws, int64_t ldws, float *partials, void *Y, int64_t ldy, tbik_dtype y_dtype,
                              tbik_dtype x_dtype, int M, int N, int K, int leaf, int k_first, int P, void *hip_stream);

/*
 * The same three calls for OCP MXFP6 operands (quantised types of the paper's "Limitations and future work"; the order
 * contract is that of Sec. 4.2, App. C and App. D.1 as stated for tbik_gemm).  An element is a 6-bit float of format
 * x_dtype (TBIK_FP6_E2M3 or TBIK_FP6_E3M2) times 2^(s - 127), s the E8M0 scale byte of its block of 32 consecutive k
 * (s = 255, NaN, is out of contract).  The elements of a row form one little-endian bit stream, element k in bits
 * 6 k .. 6 k + 5: a block is 24 bytes.  A product has at most eight significant bits and a power-of-two scale, so it is
 * exact in fp32 (as long as it stays in range): per output element each superleaf's products are accumulated in fp32 in
 * ascending k from +0, the superleaf sums are combined by T, the result is rounded once.  (The 64 products of one
 * matrix instruction are added in that instruction's own fixed order, as for the other formats.)  The weight is taken
 * TRANSPOSED: one row per output channel.
 *
 *   X    device, [M, ldx] bytes, ldx >= 3 K / 4      Xs   device, [M, ldxs] scale bytes, ldxs >= K / 32
 *   Wt   device, [N, ldwt] bytes, ldwt >= 3 K / 4    Ws   device, [N, ldws] scale bytes, ldws >= K / 32
 *   Y    device, y_dtype (TBIK_F32 or TBIK_BF16), [M, ldy], ldy >= N        partials  device, fp32, dense [P, M, N]
 *   leaf * k_first a multiple of 64 (128 for the tiled kernel; else the reference kernel runs); X, Wt 16-byte aligned
 *   with ldx, ldwt multiples of 16; Xs, Ws 4-byte aligned with ldxs, ldws multiples of 4 (the tiled kernel; the
 *   reference kernel takes scales at any address); the workspace rule (tbik_gemm_mxfp6_workspace_bytes: from 128 rows on
 *   it includes room for a copy of the scales in the order the kernel reads them, which tbik_gemm_mxfp6 makes first),
 *   the determinism contract and the errors are those of tbik_gemm, tbik_gemm_shard_partials and tbik_gemm_reference.
 */
size_t tbik_gemm_mxfp6_workspace_bytes(int M, int N, int K, int leaf, int k_first);
int tbik_gemm_mxfp6(const void *X, int64_t ldx, const void *Xs, int64_t ldxs, const void *Wt, int64_t ldwt,
                    const void *Ws, int64_t ldws, void *Y, int64_t ldy, tbik_dtype y_dtype, tbik_dtype x_dtype,
                    int M, int N, int K, int leaf, int k_first,
                    void *workspace, size_t workspace_bytes, void *hip_stream);
int tbik_gemm_shard_partials_mxfp6(const void *X, int64_t ldx, const void *Xs, int64_t ldxs, const void *Wt, int64_t ldwt,
                                   const void *Ws, int64_t ldws, float *partials, tbik_dtype x_dtype,
                                   int M, int N, int K, int leaf, int k_first, int P,
                                   void *workspace, size_t workspace_bytes, void *hip_stream);
int tbik_gemm_reference_mxfp6(const void *X, int64_t ldx, const void *Xs, int64_t ldxs, const void *Wt, int64_t ldwt,
                              const void *Ws, int64_t ldws, float *partials, void *Y, int64_t ldy, tbik_dtype y_dtype,
                              tbik_dtype x_dtype, int M, int N, int K, int leaf, int k_first, int P, void *hip_stream);

/*
 * tbik_rmsnorm and tbik_combine_residual_rmsnorm for tensors of IEEE binary16 (App. B and Alg. 2 do not depend on
 * the storage format): every 16-bit tensor of the call (x, weight, y; residual, hidden, normed) is fp16, widened
 * exactly, all arithmetic is the fp32 arithmetic stated above in the same order, and each output takes one rounding
 * to fp16 (nearest-even; overflow gives infinity) where the bf16 calls round to bf16.  Same arguments, limits,
 * aliasing rule and errors.
 */
int tbik_rmsnorm_f16(const void *x, const void *weight, void *y, int M, int H, float eps, void *hip_stream);
int tbik_combine_residual_rmsnorm_f16(const float *partials, int P, const void *residual, const void *weight, float eps,
                                      void *hidden, void *normed, int M, int H, void *hip_stream);

/* Forces an internal GEMM variant (testing and tuning only; the bits never depend on it).
 * 0 = choose from the shape (default); other values are listed in tbik_variant_name(). */
int tbik_set_gemm_variant(int variant);
const char *tbik_variant_name(int variant);      /* NULL past the last variant */

/* Forces one of the two attention kernels (testing and tuning only; the bits never depend on it):
 * 0 = default, 1 = two independent workgroups per compute unit, 2 = one workgroup whose two groups of wavefronts take
 * turns at the matrix and vector pipes.  Other values: TBIK_ERR_DTYPE. */
int tbik_set_attention_variant(int variant);

/* Log-softmax of rows longer than one block lets the workgroups of a row wait for each other a bounded number of
 * polls; a workgroup whose wait runs out finishes its block by itself (it walks the whole row), with the same bits.
 * This sets the bound (testing only: 0 makes the waits run out, so that this path is exercised).  Returns the
 * previous bound; negative values are taken as 0. */
int tbik_set_row_wait_limit(int polls);

const char *tbik_status_string(int status);
int tbik_last_hip_error(void);                    /* hipError_t of the last TBIK_ERR_HIP, as int */
const char *tbik_version(void);

#ifdef __cplusplus
}
#endif
#endif /* TBIK_H */
