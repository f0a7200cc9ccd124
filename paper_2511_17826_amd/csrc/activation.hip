// The gated activation between the two GEMMs of the MLP block (implementation appendix, "other kernels"):
// act = round16( SiLU(gate) * up ), position-wise.  Two forms: on 16-bit gate and up tensors, and directly on the fp32
// partial sums of a K-split [gate | up] GEMM, where the tree combine (Alg. 2, reduce phase) and the rounding of gate and
// up come first.  HBM-bound: 4 bytes read and 2 written per element (16-bit form).
#include "tbik_device.hpp"
#include "tbik_internal.hpp"

namespace tbik {

// Vector path: I % 8 == 0, 16-byte aligned rows; a thread owns 8 consecutive channels of a row.
template <bool F16>
__global__ __launch_bounds__(256) void silu_mul_vec8_kernel(const uint16_t *__restrict__ gate, int64_t ldg,
                                                            const uint16_t *__restrict__ up, int64_t ldu,
                                                            uint16_t *__restrict__ act, int64_t lda, int64_t M, int64_t I) {
    const int64_t chunks_per_row = I >> 3;
    const int64_t total = M * chunks_per_row;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; q < total; q += stride) {
        const int64_t row = q / chunks_per_row;
        const int64_t col = (q - row * chunks_per_row) << 3;
        const uint4 gv = *reinterpret_cast<const uint4 *>(gate + row * ldg + col);
        const uint4 uv = *reinterpret_cast<const uint4 *>(up + row * ldu + col);
        float g[8], u[8];
        unpack8<F16>(gv, g);
        unpack8<F16>(uv, u);
        float a[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) a[e] = silu_mul(g[e], u[e]);
        uint4 o;
        o.x = pack_16x2<F16>(a[0], a[1]);
        o.y = pack_16x2<F16>(a[2], a[3]);
        o.z = pack_16x2<F16>(a[4], a[5]);
        o.w = pack_16x2<F16>(a[6], a[7]);
        *reinterpret_cast<uint4 *>(act + row * lda + col) = o;
    }
}

template <bool F16>
__global__ __launch_bounds__(256) void silu_mul_scalar_kernel(const uint16_t *__restrict__ gate, int64_t ldg,
                                                              const uint16_t *__restrict__ up, int64_t ldu,
                                                              uint16_t *__restrict__ act, int64_t lda, int64_t M, int64_t I) {
    const int64_t total = M * I;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += stride) {
        const int64_t row = e / I, col = e - row * I;
        float g, u;
        if constexpr (F16) {
            g = (float)__builtin_bit_cast(_Float16, gate[row * ldg + col]);
            u = (float)__builtin_bit_cast(_Float16, up[row * ldu + col]);
        } else {
            g = bf16_bits_to_f32(gate[row * ldg + col]);
            u = bf16_bits_to_f32(up[row * ldu + col]);
        }
        act[row * lda + col] = (uint16_t)f32_to_16_bits<F16>(silu_mul(g, u));
    }
}

static dim3 grid_for(int64_t work) {
    int64_t blocks = (work + 255) / 256;
    if (blocks > 256 * 64) blocks = 256 * 64;
    if (blocks < 1) blocks = 1;
    return dim3((unsigned)blocks);
}

hipError_t launch_silu_mul(const uint16_t *gate, int64_t ldg, const uint16_t *up, int64_t ldu, uint16_t *act, int64_t lda,
                           int dtype, int M, int I, hipStream_t s) {
    if (M <= 0 || I <= 0) return hipSuccess;
    const bool f16 = (dtype == TBIK_F16);
    const auto a16 = [](const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; };
    const bool vec = I % 8 == 0 && ldg % 8 == 0 && ldu % 8 == 0 && lda % 8 == 0 && a16(gate) && a16(up) && a16(act);
    dim3 block(256);
    if (vec) {
        dim3 grid = grid_for((int64_t)M * (I / 8));
        if (f16) hipLaunchKernelGGL(silu_mul_vec8_kernel<true>, grid, block, 0, s, gate, ldg, up, ldu, act, lda, (int64_t)M, (int64_t)I);
        else hipLaunchKernelGGL(silu_mul_vec8_kernel<false>, grid, block, 0, s, gate, ldg, up, ldu, act, lda, (int64_t)M, (int64_t)I);
    } else {
        dim3 grid = grid_for((int64_t)M * I);
        if (f16) hipLaunchKernelGGL(silu_mul_scalar_kernel<true>, grid, block, 0, s, gate, ldg, up, ldu, act, lda, (int64_t)M, (int64_t)I);
        else hipLaunchKernelGGL(silu_mul_scalar_kernel<false>, grid, block, 0, s, gate, ldg, up, ldu, act, lda, (int64_t)M, (int64_t)I);
    }
    return hipGetLastError();
}

// On the partial sums of a K-split [gate | up] GEMM: a thread owns 4 consecutive channels of a row; it forms
// T(partials) for its gate and its up columns in the order of Alg. 2's reduce phase, rounds both to 16 bits (the
// outputs the two GEMMs would have stored), and applies the activation.
template <int P, bool F16>
__global__ __launch_bounds__(256) void tree_combine_swiglu_kernel(const float *__restrict__ partials, uint16_t *__restrict__ act,
                                                                  int64_t lda, int64_t M, int64_t I) {
    const int64_t quads_per_row = I >> 2;
    const int64_t total = M * quads_per_row;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t plane = M * 2 * I;
    for (int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; q < total; q += stride) {
        const int64_t row = q / quads_per_row;
        const int64_t col = (q - row * quads_per_row) << 2;
        const float *src = partials + row * 2 * I + col;
        f32x4 gin[P], uin[P];
#pragma unroll
        for (int p = 0; p < P; ++p) {
            gin[p] = *reinterpret_cast<const f32x4 *>(src + (int64_t)p * plane);
            uin[p] = *reinterpret_cast<const f32x4 *>(src + (int64_t)p * plane + I);
        }
        float a[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            float gv[P], uv[P];
#pragma unroll
            for (int p = 0; p < P; ++p) { gv[p] = gin[p][e]; uv[p] = uin[p][e]; }
            a[e] = silu_mul(through_16_bits<F16>(tree_of<P>(gv)), through_16_bits<F16>(tree_of<P>(uv)));
        }
        uint16_t *dst = act + row * lda + col;
        const uint32_t lo = pack_16x2<F16>(a[0], a[1]), hi = pack_16x2<F16>(a[2], a[3]);
        if ((reinterpret_cast<uintptr_t>(dst) & 7) == 0) {
            *reinterpret_cast<uint2 *>(dst) = make_uint2(lo, hi);
        } else {
            dst[0] = (uint16_t)lo; dst[1] = (uint16_t)(lo >> 16); dst[2] = (uint16_t)hi; dst[3] = (uint16_t)(hi >> 16);
        }
    }
}

template <int P>
static hipError_t launch_combine_swiglu_p(const float *partials, uint16_t *act, int64_t lda, int dtype, int M, int I, hipStream_t s) {
    dim3 grid = grid_for((int64_t)M * (I / 4)), block(256);
    if (dtype == TBIK_F16) hipLaunchKernelGGL((tree_combine_swiglu_kernel<P, true>), grid, block, 0, s, partials, act, lda, (int64_t)M, (int64_t)I);
    else hipLaunchKernelGGL((tree_combine_swiglu_kernel<P, false>), grid, block, 0, s, partials, act, lda, (int64_t)M, (int64_t)I);
    return hipGetLastError();
}

hipError_t launch_tree_combine_swiglu(const float *partials, int P, uint16_t *act, int64_t lda, int dtype, int M, int I,
                                      hipStream_t s) {
    if (M <= 0 || I <= 0) return hipSuccess;
    if (I % 4 != 0 || (reinterpret_cast<uintptr_t>(partials) & 15) != 0) return hipErrorInvalidValue;
    switch (P) {
        case 2: return launch_combine_swiglu_p<2>(partials, act, lda, dtype, M, I, s);
        case 4: return launch_combine_swiglu_p<4>(partials, act, lda, dtype, M, I, s);
        case 8: return launch_combine_swiglu_p<8>(partials, act, lda, dtype, M, I, s);
        case 16: return launch_combine_swiglu_p<16>(partials, act, lda, dtype, M, I, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace tbik
