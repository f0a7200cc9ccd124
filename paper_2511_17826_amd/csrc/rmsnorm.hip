// Batch-invariant RMSNorm (App. B) with the tree order of App. C along the row.
//
// One wavefront owns one row, whatever M is, so a row's arithmetic cannot depend on the batch.
// Leaf c of the row's tree is the in-order fp32 sum of the squares of elements 8c..8c+7 (one
// 16-byte load).  Leaves 64s..64s+63 sit in the 64 lanes of the wavefront: tree levels 0..5 are
// lane-pair additions, the higher levels combine the per-segment sums in registers by the
// carry-over scheme.  Leaves past the end of the row are +0, as in the definition.
// HBM-bound: 2H bytes read + 2H written per row (the second read of x hits in cache).
#include "tbik_device.hpp"
#include "tbik_internal.hpp"

namespace tbik {

constexpr int RMS_ROWS_PER_BLOCK = 4;
constexpr int RMS_MAX_SEG_LEVELS = 8;   // up to 2^7 = 128 segments of 64 leaves of 8 elements = 65536 columns

// F16 in the kernels below: the rows, the weight and the outputs are IEEE binary16 instead of bf16 (squares of
// either are exact in fp32; one rounding to nearest-even at the end).
//
// Register-resident variant for rows of at most 64*CPL chunks (H <= 512*CPL): the row is read once, kept as packed
// 16-bit values in registers across the reduction and normalised from there.  Same leaves, same tree, same bits as the
// two-pass kernel below.
template <int CPL, bool F16>
__global__ __launch_bounds__(64 * RMS_ROWS_PER_BLOCK) void rmsnorm_regs_kernel(
        const uint16_t *__restrict__ x, const uint16_t *__restrict__ w, uint16_t *__restrict__ y,
        int M, int H, float eps, int nseg2) {
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * RMS_ROWS_PER_BLOCK + (threadIdx.x >> 6);
    if (row >= M) return;                              // whole wavefront leaves together
    const int nchunks = H >> 3;
    const uint4 *xr = reinterpret_cast<const uint4 *>(x + (int64_t)row * H);
    const uint4 *wr = reinterpret_cast<const uint4 *>(w);
    uint4 *yr = reinterpret_cast<uint4 *>(y + (int64_t)row * H);

    uint4 xv[CPL];
#pragma unroll
    for (int s = 0; s < CPL; ++s) {
        const int c = s * 64 + lane;
        xv[s] = (c < nchunks) ? xr[c] : make_uint4(0, 0, 0, 0);
    }
    TreeStash<RMS_MAX_SEG_LEVELS> st;
    float ss = 0.0f;
#pragma unroll
    for (int s = 0; s < CPL; ++s) {
        float f[8], leaf = 0.0f;
        unpack8<F16>(xv[s], f);                             // a chunk past the row is all +0: its leaf is +0
#pragma unroll
        for (int e = 0; e < 8; ++e) leaf = leaf + f[e] * f[e];
        if (s < nseg2) ss = st.push(wave_tree_sum(leaf), (unsigned)s);
    }
    for (int s = CPL; s < nseg2; ++s) ss = st.push(wave_tree_sum(0.0f), (unsigned)s);   // padding segments
    const float ms = ss / (float)H;
    const float r = 1.0f / sqrtf(ms + eps);
#pragma unroll
    for (int s = 0; s < CPL; ++s) {
        const int c = s * 64 + lane;
        if (c < nchunks) {
            float f[8], g[8];
            unpack8<F16>(xv[s], f);
            unpack8<F16>(wr[c], g);
            float o[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float t = f[e] * r;
                o[e] = t * g[e];
            }
            yr[c] = make_uint4(pack_16x2<F16>(o[0], o[1]), pack_16x2<F16>(o[2], o[3]), pack_16x2<F16>(o[4], o[5]), pack_16x2<F16>(o[6], o[7]));
        }
    }
}

template <bool F16>
__global__ __launch_bounds__(64 * RMS_ROWS_PER_BLOCK) void rmsnorm_kernel(
        const uint16_t *__restrict__ x, const uint16_t *__restrict__ w, uint16_t *__restrict__ y,
        int M, int H, float eps, int nseg2) {
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * RMS_ROWS_PER_BLOCK + (threadIdx.x >> 6);
    if (row >= M) return;                              // whole wavefront leaves together
    const int nchunks = H >> 3;
    const uint4 *xr = reinterpret_cast<const uint4 *>(x + (int64_t)row * H);
    const uint4 *wr = reinterpret_cast<const uint4 *>(w);
    uint4 *yr = reinterpret_cast<uint4 *>(y + (int64_t)row * H);

    TreeStash<RMS_MAX_SEG_LEVELS> st;
    float ss = 0.0f;
    for (int seg = 0; seg < nseg2; ++seg) {
        const int c = seg * 64 + lane;
        float leaf = 0.0f;
        if (c < nchunks) {
            float f[8];
            unpack8<F16>(xr[c], f);
#pragma unroll
            for (int e = 0; e < 8; ++e) leaf = leaf + f[e] * f[e];
        }
        ss = st.push(wave_tree_sum(leaf), (unsigned)seg);
    }
    const float ms = ss / (float)H;
    const float r = 1.0f / sqrtf(ms + eps);

    for (int c = lane; c < nchunks; c += 64) {
        float f[8], g[8];
        unpack8<F16>(xr[c], f);
        unpack8<F16>(wr[c], g);
        float o[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float t = f[e] * r;
            o[e] = t * g[e];
        }
        yr[c] = make_uint4(pack_16x2<F16>(o[0], o[1]), pack_16x2<F16>(o[2], o[3]), pack_16x2<F16>(o[4], o[5]), pack_16x2<F16>(o[6], o[7]));
    }
}

// Fused tail of a row-parallel layer: per element Y = bf16(T(partials[0..P))) as the top-of-tree combine does
// (Alg. 2's additions, one rounding), H = bf16(Y + R) with the residual R, then the RMSNorm above over the row of H.
// One wavefront per row; first pass: combine, add, store H, leaf sums of squares; second pass: re-read H (the
// wavefront's own stores, served by the cache) and scale.  Bit for bit the three separate calls.
template <int P, bool F16>
__global__ __launch_bounds__(64 * RMS_ROWS_PER_BLOCK) void combine_residual_rmsnorm_kernel(
        const float *__restrict__ partials, const uint16_t *res, const uint16_t *__restrict__ w,
        uint16_t *hidden, uint16_t *__restrict__ normed, int M, int H, float eps, int nseg2) {
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * RMS_ROWS_PER_BLOCK + (threadIdx.x >> 6);
    if (row >= M) return;                              // whole wavefront leaves together
    const int nchunks = H >> 3;
    const int64_t plane = (int64_t)M * H;
    const bool stream = plane * P * 4 > ((int64_t)192 << 20);   // uniform: planes that no cache holds are read around the caches
    const float *pr = partials + (int64_t)row * H;
    const uint4 *rr = reinterpret_cast<const uint4 *>(res + (int64_t)row * H);
    const uint4 *wr = reinterpret_cast<const uint4 *>(w);
    uint4 *hr = reinterpret_cast<uint4 *>(hidden + (int64_t)row * H);
    uint4 *yr = reinterpret_cast<uint4 *>(normed + (int64_t)row * H);

    TreeStash<RMS_MAX_SEG_LEVELS> st;
    float ss = 0.0f;
    for (int seg = 0; seg < nseg2; ++seg) {
        const int c = seg * 64 + lane;
        float leaf = 0.0f;
        if (c < nchunks) {
            float4 lo[P], hi[P];
#pragma unroll
            for (int p = 0; p < P; ++p) {
                if (stream) {
                    typedef float nt_f32x4 __attribute__((ext_vector_type(4)));
                    const nt_f32x4 a = __builtin_nontemporal_load(reinterpret_cast<const nt_f32x4 *>(pr + (int64_t)p * plane + c * 8));
                    const nt_f32x4 b = __builtin_nontemporal_load(reinterpret_cast<const nt_f32x4 *>(pr + (int64_t)p * plane + c * 8 + 4));
                    lo[p] = make_float4(a[0], a[1], a[2], a[3]);
                    hi[p] = make_float4(b[0], b[1], b[2], b[3]);
                } else {
                    lo[p] = *reinterpret_cast<const float4 *>(pr + (int64_t)p * plane + c * 8);
                    hi[p] = *reinterpret_cast<const float4 *>(pr + (int64_t)p * plane + c * 8 + 4);
                }
            }
            float y[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float v[P];
#pragma unroll
                for (int p = 0; p < P; ++p) {
                    const float4 &q = (e < 4) ? lo[p] : hi[p];
                    v[p] = (e & 3) == 0 ? q.x : (e & 3) == 1 ? q.y : (e & 3) == 2 ? q.z : q.w;
                }
                y[e] = tree_of<P>(v);
            }
            float r[8], yb[8], h[8];
            unpack8<F16>(rr[c], r);
            unpack8<F16>(make_uint4(pack_16x2<F16>(y[0], y[1]), pack_16x2<F16>(y[2], y[3]), pack_16x2<F16>(y[4], y[5]), pack_16x2<F16>(y[6], y[7])), yb);
#pragma unroll
            for (int e = 0; e < 8; ++e) h[e] = yb[e] + r[e];
            const uint4 hv = make_uint4(pack_16x2<F16>(h[0], h[1]), pack_16x2<F16>(h[2], h[3]), pack_16x2<F16>(h[4], h[5]), pack_16x2<F16>(h[6], h[7]));
            hr[c] = hv;
            float f[8];
            unpack8<F16>(hv, f);
#pragma unroll
            for (int e = 0; e < 8; ++e) leaf = leaf + f[e] * f[e];
        }
        ss = st.push(wave_tree_sum(leaf), (unsigned)seg);
    }
    const float ms = ss / (float)H;
    const float rinv = 1.0f / sqrtf(ms + eps);

    for (int c = lane; c < nchunks; c += 64) {
        float f[8], g[8];
        unpack8<F16>(hr[c], f);
        unpack8<F16>(wr[c], g);
        float o[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float t = f[e] * rinv;
            o[e] = t * g[e];
        }
        yr[c] = make_uint4(pack_16x2<F16>(o[0], o[1]), pack_16x2<F16>(o[2], o[3]), pack_16x2<F16>(o[4], o[5]), pack_16x2<F16>(o[6], o[7]));
    }
}

template <bool F16>
static hipError_t rmsnorm_of(const uint16_t *x, const uint16_t *w, uint16_t *y, int M, int H, float eps, hipStream_t s) {
    if (M <= 0) return hipSuccess;
    const int nchunks = H / 8;
    int n2 = 1;
    while (n2 < nchunks) n2 *= 2;
    const int nseg2 = n2 < 64 ? 1 : n2 / 64;
    dim3 grid((M + RMS_ROWS_PER_BLOCK - 1) / RMS_ROWS_PER_BLOCK), block(64 * RMS_ROWS_PER_BLOCK);
    const int cpl = (nchunks + 63) / 64;
    if (cpl <= 2) hipLaunchKernelGGL((rmsnorm_regs_kernel<2, F16>), grid, block, 0, s, x, w, y, M, H, eps, nseg2);
    else if (cpl <= 4) hipLaunchKernelGGL((rmsnorm_regs_kernel<4, F16>), grid, block, 0, s, x, w, y, M, H, eps, nseg2);
    else if (cpl <= 8) hipLaunchKernelGGL((rmsnorm_regs_kernel<8, F16>), grid, block, 0, s, x, w, y, M, H, eps, nseg2);
    else if (cpl <= 10) hipLaunchKernelGGL((rmsnorm_regs_kernel<10, F16>), grid, block, 0, s, x, w, y, M, H, eps, nseg2);
    else if (cpl <= 16) hipLaunchKernelGGL((rmsnorm_regs_kernel<16, F16>), grid, block, 0, s, x, w, y, M, H, eps, nseg2);
    else hipLaunchKernelGGL(rmsnorm_kernel<F16>, grid, block, 0, s, x, w, y, M, H, eps, nseg2);
    return hipGetLastError();
}

hipError_t launch_rmsnorm(const uint16_t *x, const uint16_t *w, uint16_t *y, int M, int H, float eps, int dtype, hipStream_t s) {
    return dtype == TBIK_F16 ? rmsnorm_of<true>(x, w, y, M, H, eps, s) : rmsnorm_of<false>(x, w, y, M, H, eps, s);
}

template <bool F16>
static hipError_t tail_of(const float *partials, int P, const uint16_t *res, const uint16_t *w, uint16_t *hidden,
                          uint16_t *normed, int M, int H, float eps, hipStream_t s) {
    if (M <= 0) return hipSuccess;
    const int nchunks = H / 8;
    int n2 = 1;
    while (n2 < nchunks) n2 *= 2;
    const int nseg2 = n2 < 64 ? 1 : n2 / 64;
    dim3 grid((M + RMS_ROWS_PER_BLOCK - 1) / RMS_ROWS_PER_BLOCK), block(64 * RMS_ROWS_PER_BLOCK);
    switch (P) {
        case 1: hipLaunchKernelGGL((combine_residual_rmsnorm_kernel<1, F16>), grid, block, 0, s, partials, res, w, hidden, normed, M, H, eps, nseg2); break;
        case 2: hipLaunchKernelGGL((combine_residual_rmsnorm_kernel<2, F16>), grid, block, 0, s, partials, res, w, hidden, normed, M, H, eps, nseg2); break;
        case 4: hipLaunchKernelGGL((combine_residual_rmsnorm_kernel<4, F16>), grid, block, 0, s, partials, res, w, hidden, normed, M, H, eps, nseg2); break;
        case 8: hipLaunchKernelGGL((combine_residual_rmsnorm_kernel<8, F16>), grid, block, 0, s, partials, res, w, hidden, normed, M, H, eps, nseg2); break;
        case 16: hipLaunchKernelGGL((combine_residual_rmsnorm_kernel<16, F16>), grid, block, 0, s, partials, res, w, hidden, normed, M, H, eps, nseg2); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_combine_residual_rmsnorm(const float *partials, int P, const uint16_t *res, const uint16_t *w,
                                           uint16_t *hidden, uint16_t *normed, int M, int H, float eps, int dtype, hipStream_t s) {
    return dtype == TBIK_F16 ? tail_of<true>(partials, P, res, w, hidden, normed, M, H, eps, s)
                             : tail_of<false>(partials, P, res, w, hidden, normed, M, H, eps, s);
}

}  // namespace tbik
