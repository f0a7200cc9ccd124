// Top-of-tree combine (Sec. 4.2 "Inter-GPU reduction"; App. D.2, Alg. 2 reduce phase) on one GPU.
//
// The P partial tensors stand in for the ranks' buffers.  Per element the kernel performs exactly
// the additions of Alg. 2: at level l, buffer r (r mod 2^(l+1) == 0) receives buffer r + 2^l.
// Then the single rounding to the output type.  HBM-bound: 4*P bytes read + 2 or 4 written per element.
#include "tbik_device.hpp"
#include "tbik_internal.hpp"

namespace tbik {

// Vector path: N % 4 == 0; each thread owns 4 consecutive columns of one row.
template <int P, int OUT, bool STREAM>   // OUT: tbik_dtype of Y; STREAM: the planes are read around the caches
__global__ __launch_bounds__(256) void tree_combine_vec4_kernel(const float *__restrict__ partials, void *__restrict__ Y,
                                                                int64_t ldy, int64_t M, int64_t N) {
    const int64_t quads_per_row = N >> 2;
    const int64_t total = M * quads_per_row;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t plane = M * N;
    for (int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; q < total; q += stride) {
        const int64_t row = q / quads_per_row;
        const int64_t col = (q - row * quads_per_row) << 2;
        const float *src = partials + row * N + col;
        f32x4 in[P];
#pragma unroll
        for (int p = 0; p < P; ++p) {
            const f32x4 *ptr = reinterpret_cast<const f32x4 *>(src + (int64_t)p * plane);
            in[p] = STREAM ? __builtin_nontemporal_load(ptr) : *ptr;
        }
        float vx[P], vy[P], vz[P], vw[P];
#pragma unroll
        for (int p = 0; p < P; ++p) { vx[p] = in[p][0]; vy[p] = in[p][1]; vz[p] = in[p][2]; vw[p] = in[p][3]; }
        const float x = tree_of<P>(vx), y = tree_of<P>(vy), z = tree_of<P>(vz), w = tree_of<P>(vw);
        if (OUT != TBIK_F32) {
            uint16_t *dst = reinterpret_cast<uint16_t *>(Y) + row * ldy + col;
            const uint32_t lo = pack_16x2<OUT == TBIK_F16>(x, y);
            const uint32_t hi = pack_16x2<OUT == TBIK_F16>(z, w);
            if ((reinterpret_cast<uintptr_t>(dst) & 7) == 0) {
                *reinterpret_cast<uint2 *>(dst) = make_uint2(lo, hi);
            } else {
                dst[0] = (uint16_t)lo; dst[1] = (uint16_t)(lo >> 16); dst[2] = (uint16_t)hi; dst[3] = (uint16_t)(hi >> 16);
            }
        } else {
            float *dst = reinterpret_cast<float *>(Y) + row * ldy + col;
            if ((reinterpret_cast<uintptr_t>(dst) & 15) == 0) {
                *reinterpret_cast<float4 *>(dst) = make_float4(x, y, z, w);
            } else {
                dst[0] = x; dst[1] = y; dst[2] = z; dst[3] = w;
            }
        }
    }
}

// Scalar path for any N.
template <int P, int OUT>   // OUT: tbik_dtype of Y
__global__ __launch_bounds__(256) void tree_combine_scalar_kernel(const float *__restrict__ partials, void *__restrict__ Y,
                                                                  int64_t ldy, int64_t M, int64_t N) {
    const int64_t total = M * N;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += stride) {
        const int64_t row = e / N, col = e - row * N;
        float v[P];
#pragma unroll
        for (int p = 0; p < P; ++p) v[p] = partials[(int64_t)p * total + e];
        const float y = tree_of<P>(v);
        if (OUT != TBIK_F32) reinterpret_cast<uint16_t *>(Y)[row * ldy + col] = (uint16_t)f32_to_16_bits<OUT == TBIK_F16>(y);
        else reinterpret_cast<float *>(Y)[row * ldy + col] = y;
    }
}

template <int P, int OUT>
static hipError_t launch_p_out(const float *partials, void *Y, int64_t ldy, int M, int N, hipStream_t s) {
    const bool vec = (N % 4 == 0) && ((reinterpret_cast<uintptr_t>(partials) & 15) == 0);
    const int64_t work = vec ? (int64_t)M * (N / 4) : (int64_t)M * N;
    int64_t blocks = (work + 255) / 256;
    if (blocks > 256 * 64) blocks = 256 * 64;   // grid-stride beyond 64 blocks per CU
    if (blocks < 1) blocks = 1;
    dim3 grid((unsigned)blocks), block(256);
    // Hundreds of MiB of planes come from HBM and are read once: streaming loads (544 MiB at P = 8: 106 -> 101 us).
    // Smaller sets are usually still in the memory-side cache of the kernel that wrote them, where plain loads are faster.
    const bool stream = (int64_t)P * M * N * 4 > ((int64_t)192 << 20);
    if (vec && stream) hipLaunchKernelGGL((tree_combine_vec4_kernel<P, OUT, true>), grid, block, 0, s, partials, Y, ldy, (int64_t)M, (int64_t)N);
    else if (vec) hipLaunchKernelGGL((tree_combine_vec4_kernel<P, OUT, false>), grid, block, 0, s, partials, Y, ldy, (int64_t)M, (int64_t)N);
    else hipLaunchKernelGGL((tree_combine_scalar_kernel<P, OUT>), grid, block, 0, s, partials, Y, ldy, (int64_t)M, (int64_t)N);
    return hipGetLastError();
}

template <int P>
static hipError_t launch_p(const float *partials, void *Y, int64_t ldy, int y_dtype, int M, int N, hipStream_t s) {
    switch (y_dtype) {
        case TBIK_F32: return launch_p_out<P, TBIK_F32>(partials, Y, ldy, M, N, s);
        case TBIK_BF16: return launch_p_out<P, TBIK_BF16>(partials, Y, ldy, M, N, s);
        case TBIK_F16: return launch_p_out<P, TBIK_F16>(partials, Y, ldy, M, N, s);
        default: return hipErrorInvalidValue;
    }
}

// Alg. 2 taken literally, round by round, on P buffers that stand for the ranks (App. D.2): in round l of the reduce
// phase every rank r with r mod 2^(l+1) == 0 "receives" the buffer of rank r + 2^l and adds it to its own (own + received,
// as the listing has it); the broadcast phase runs the same pairs backwards, the receiver copying.  One launch per
// round handles all pairs of that round.
template <bool ADD>
__global__ __launch_bounds__(256) void allreduce_round_kernel(float *__restrict__ bufs, int64_t n, int stride_ranks, int pairs) {
    // 16-byte accesses only when every rank's buffer starts on a 16-byte boundary (n a multiple of 4)
    const int64_t quads = (n & 3) ? 0 : (n >> 2), total = quads * pairs, step = (int64_t)gridDim.x * blockDim.x;
    for (int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; q < total; q += step) {
        const int64_t pair = q / quads, i = (q - pair * quads) << 2;
        float *low = bufs + (pair * 2 * stride_ranks) * n + i;              // rank r
        float *high = low + (int64_t)stride_ranks * n;                      // rank r + 2^l
        if (ADD) {
            const f32x4 a = *reinterpret_cast<const f32x4 *>(low), b = *reinterpret_cast<const f32x4 *>(high);
            *reinterpret_cast<f32x4 *>(low) = f32x4{a[0] + b[0], a[1] + b[1], a[2] + b[2], a[3] + b[3]};
        } else {
            *reinterpret_cast<f32x4 *>(high) = *reinterpret_cast<const f32x4 *>(low);
        }
    }
    // element by element otherwise
    const int64_t tail = n - 4 * quads;
    for (int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; q < tail * pairs; q += step) {
        const int64_t pair = q / tail, i = (n - tail) + (q - pair * tail);
        float *low = bufs + (pair * 2 * stride_ranks) * n + i;
        float *high = low + (int64_t)stride_ranks * n;
        if (ADD) *low = *low + *high;
        else *high = *low;
    }
}

hipError_t launch_tree_allreduce(float *bufs, int P, int64_t n, hipStream_t s) {
    if (n <= 0 || P <= 1) return hipSuccess;
    auto grid_of = [&](int pairs) {
        int64_t blocks = (((n & 3) ? n : n / 4) * pairs + 255) / 256;
        if (blocks > 256 * 64) blocks = 256 * 64;
        return dim3((unsigned)(blocks < 1 ? 1 : blocks));
    };
    for (int st = 1; st < P; st *= 2)                                       // reduce phase, level by level
        hipLaunchKernelGGL(allreduce_round_kernel<true>, grid_of(P / (2 * st)), dim3(256), 0, s, bufs, n, st, P / (2 * st));
    for (int st = P / 2; st >= 1; st /= 2)                                  // broadcast phase
        hipLaunchKernelGGL(allreduce_round_kernel<false>, grid_of(P / (2 * st)), dim3(256), 0, s, bufs, n, st, P / (2 * st));
    return hipGetLastError();
}

hipError_t launch_tree_combine(const float *partials, int P, void *Y, int64_t ldy, int y_dtype, int M, int N,
                               hipStream_t s) {
    if (M <= 0 || N <= 0) return hipSuccess;
    switch (P) {
        case 1: return launch_p<1>(partials, Y, ldy, y_dtype, M, N, s);
        case 2: return launch_p<2>(partials, Y, ldy, y_dtype, M, N, s);
        case 4: return launch_p<4>(partials, Y, ldy, y_dtype, M, N, s);
        case 8: return launch_p<8>(partials, Y, ldy, y_dtype, M, N, s);
        case 16: return launch_p<16>(partials, Y, ldy, y_dtype, M, N, s);
        case 32: return launch_p<32>(partials, Y, ldy, y_dtype, M, N, s);
        case 64: return launch_p<64>(partials, Y, ldy, y_dtype, M, N, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace tbik
