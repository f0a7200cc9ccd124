// Reference Tree-Based MatMul kernel (App. D.1, Alg. 1) for gfx950.
//
// One wavefront computes one 32x32 output tile of one K-shard.  Operands come straight from
// global memory, so there is no tiling schedule to reason about: the kernel loops over the
// shard's superleaves in ascending k; inside a superleaf it chains
// v_mfma_f32_32x32x16_bf16 (v_mfma_f32_32x32x16_f16 for binary16 operands) over ascending groups
// of 16 k into an accumulator that starts at +0; after each superleaf the carry-over step of Alg. 1 folds the accumulator into the stash of
// waiting subtrees.  The tuned kernels issue the same MFMA opcode over the same k -> (step, slot)
// map and the same fp32 additions, so they must reproduce this kernel's bits.
#include "tbik_device.hpp"
#include "tbik_internal.hpp"

namespace tbik {

constexpr int REF_MAX_LEVELS = 28;

template <bool F16>
__global__ __launch_bounds__(64) void gemm_reference_kernel(
        const uint16_t *__restrict__ X, int64_t ldx, const uint16_t *__restrict__ W, int64_t ldw,
        float *__restrict__ partials, void *__restrict__ Y, int64_t ldy, int y_dtype,
        int M, int N, int K, int superleaf, int ns_per_shard) {
    const int lane = threadIdx.x;
    const int i = lane & 31;      // row of A / column of B held by this lane
    const int g = lane >> 5;      // which group of 8 k inside a step of 16
    const int m0 = blockIdx.y * 32, n0 = blockIdx.x * 32;
    const int p = blockIdx.z;
    const int64_t kbase = (int64_t)p * ns_per_shard * superleaf;

    const bool row_ok = (m0 + i) < M;
    const bool col_ok = (n0 + i) < N;
    const uint16_t *xrow = X + (int64_t)(m0 + i) * ldx;
    const uint16_t *wcol = W + (n0 + i);

    float stash[REF_MAX_LEVELS][16];
    f32x16 acc;

    for (int j = 0; j < ns_per_shard; ++j) {
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
        const int64_t k0 = kbase + (int64_t)j * superleaf;
        for (int kk = 0; kk < superleaf; kk += 16) {
            const int64_t k = k0 + kk + 8 * g;
            union { uint4 u; bf16x8 v; } a, b;
            a.u = make_uint4(0, 0, 0, 0);
            if (row_ok) a.u = *reinterpret_cast<const uint4 *>(xrow + k);
            uint32_t w[8];
#pragma unroll
            for (int t = 0; t < 8; ++t) w[t] = col_ok ? (uint32_t)wcol[(k + t) * ldw] : 0u;
            b.u = make_uint4(w[0] | (w[1] << 16), w[2] | (w[3] << 16), w[4] | (w[5] << 16), w[6] | (w[7] << 16));
            acc = mfma_32x32x16<F16>(a.v, b.v, acc);
        }
        // carry-over: superleaf j completes as many subtrees as j has trailing one bits
        const int t = __builtin_ctz(~(unsigned)j);
        for (int l = 0; l < t; ++l) {
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = stash[l][r] + acc[r];
        }
        if (j + 1 < ns_per_shard) {
#pragma unroll
            for (int r = 0; r < 16; ++r) stash[t][r] = acc[r];
        }
    }

    // D layout of the 32x32 MFMA: register r of lane l is D[8*(r/4) + 4*(l/32) + r%4][l%32].
    const int col = n0 + i;
    if (!col_ok) return;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int row = m0 + 8 * (r >> 2) + 4 * g + (r & 3);
        if (row >= M) continue;
        if (partials) partials[((int64_t)p * M + row) * N + col] = acc[r];
        if (Y) {
            if (y_dtype == TBIK_F32) reinterpret_cast<float *>(Y)[(int64_t)row * ldy + col] = acc[r];
            else reinterpret_cast<uint16_t *>(Y)[(int64_t)row * ldy + col] = (uint16_t)f32_to_16_bits<F16>(acc[r]);
        }
    }
}

hipError_t launch_gemm_reference(const GemmArgs &a, hipStream_t s) {
    if (a.M <= 0 || a.N <= 0) return hipSuccess;
    dim3 grid((a.N + 31) / 32, (a.M + 31) / 32, a.P);
    if (grid.y > 65535u || grid.z > 65535u) return hipErrorInvalidValue;
    void *Y = (a.P == 1) ? a.Y : nullptr;
    auto kernel = (a.x_dtype == TBIK_F16) ? gemm_reference_kernel<true> : gemm_reference_kernel<false>;
    hipLaunchKernelGGL(kernel, grid, dim3(64), 0, s, a.X, a.ldx, a.W, a.ldw, a.partials, Y, a.ldy,
                       a.y_dtype, a.M, a.N, a.K, a.superleaf, a.ns / a.P);
    return hipGetLastError();
}

}  // namespace tbik
