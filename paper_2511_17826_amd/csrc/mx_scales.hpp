// Re-tiling of the E8M0 block scales of microscaling operands, shared by the MXFP8 and MXFP4 GEMM kernels.
#pragma once

#include "tbik_device.hpp"

namespace tbik {

// The scales of both operands, [rows, ld] bytes with 4 * DWORDS per stage of the tiled kernel, copied into the order in
// which that kernel takes them: dword d of (row block, stage, row r of the block) goes to
//   out[((block * stages + stage) * block_rows + r) * DWORDS + d]
// (rows past the end repeat the last one), so that a stage's scales of a row block are consecutive bytes and a
// wavefront's load of them touches two cache lines instead of one per row.  One thread per dword, X's first, then Wt's
// (blocks of 128 rows, behind the x_total dwords of X); consecutive threads write consecutive dwords (the reads, one
// cache line per row, are served by the caches: a line holds the scales of 32 / DWORDS stages).
template <int DWORDS>
__global__ __launch_bounds__(256) void mx_scales_retile_kernel(const uint8_t *__restrict__ Xs, int64_t ldxs, int x_rows, int x_block_rows,
                                                               const uint8_t *__restrict__ Ws, int64_t ldws, int w_rows,
                                                               int stages, uint32_t *__restrict__ out, int64_t x_total, int64_t total) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const bool x = i < x_total;
        const int64_t j = x ? i : i - x_total;                    // = ((block * stages + stage) * block_rows + r) * DWORDS + d
        const int rows = x ? x_rows : w_rows, block_rows = x ? x_block_rows : 128;
        const int64_t q = j / DWORDS;
        const int d = (int)(j - q * DWORDS);
        const int64_t bs = q / block_rows;
        const int r = (int)(q - bs * block_rows);
        const int64_t block = bs / stages;
        const int stage = (int)(bs - block * stages);
        const int64_t row = block * block_rows + r, src_row = row < rows ? row : rows - 1;
        const uint8_t *src = x ? Xs + src_row * ldxs : Ws + src_row * ldws;
        out[i] = *reinterpret_cast<const uint32_t *>(src + 4 * (stage * DWORDS + d));
    }
}

// Bytes of the re-tiled copies for operands of M and N rows and `stages` stages along K.
template <int DWORDS>
inline size_t mx_retiled_scales_bytes(int M, int N, int stages) {
    return ((((size_t)M + 127) / 128) * 128 + (((size_t)N + 127) / 128) * 128) * (size_t)stages * DWORDS * 4;
}

// One launch; x_block_rows: the tile height of the GEMM launch that follows (32, 64 or 128).  Returns where the re-tiled
// X scales and Wt scales start inside `out`.  The sources are 4-byte aligned with row strides that are multiples of 4.
template <int DWORDS>
inline hipError_t launch_mx_scales_retile(const uint8_t *Xs, int64_t ldxs, int M, int x_block_rows, const uint8_t *Ws, int64_t ldws, int N,
                                          int stages, void *out, const uint8_t **x_out, const uint8_t **w_out, hipStream_t s) {
    const int64_t xrows = ((int64_t)M + x_block_rows - 1) / x_block_rows * x_block_rows, wrows = ((int64_t)N + 127) / 128 * 128;
    const int64_t x_total = xrows * stages * DWORDS, total = x_total + wrows * stages * DWORDS, blocks = (total + 255) / 256;
    uint32_t *o = reinterpret_cast<uint32_t *>(out);
    hipLaunchKernelGGL(mx_scales_retile_kernel<DWORDS>, dim3((unsigned)(blocks < 4096 ? blocks : 4096)), dim3(256), 0, s, Xs, ldxs, M,
                       x_block_rows, Ws, ldws, N, stages, o, x_total, total);
    *x_out = reinterpret_cast<const uint8_t *>(o);
    *w_out = reinterpret_cast<const uint8_t *>(o + x_total);
    return hipGetLastError();
}

}  // namespace tbik
