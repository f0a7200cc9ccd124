// Tiled Tree-Based MatMul kernels (App. D.1, Alg. 1) for gfx950.
//
// A workgroup of 4 wavefronts owns one BM x BN output tile of one K-shard and walks the shard's
// superleaves in ascending k.  Per superleaf each wavefront chains v_mfma_f32_32x32x16_bf16 over
// ascending groups of 16 k into accumulators that start at +0 (the same opcode and k -> (step,
// slot) map as the reference kernel, which is what makes all variants bit-identical); when a
// superleaf ends, the carry-over step folds the accumulators into the stash of waiting subtrees,
// which lives in registers (one wavefront per SIMD, up to 512 VGPR+AGPR per lane).
//
// Operands are staged through LDS in K-steps of 64 with double buffering: X rows keep their
// K-contiguous order; W ([K,N], N contiguous) is transposed in registers on the way in, so both
// MFMA operands are read from LDS as 16-byte, K-contiguous fragments.  Rows are padded to
// 144 bytes, which spreads a fragment read of 16 rows over all 64 LDS banks.
#include "tbik_device.hpp"
#include "tbik_internal.hpp"

namespace tbik {

constexpr int BK = 64;                 // K-elements per LDS stage
constexpr int PITCH = BK * 2 + 16;     // bytes per LDS row (64 bf16 + 16 pad)

template <int MT, int NT>              // 32x32 MFMA tiles per wavefront
struct Acc {
    f32x16 t[MT][NT];
};

// Stash of finished subtrees (App. D.1: accumulator buffer S[level]); every slot is addressed statically.
template <int LEVELS, int MT, int NT>
struct TileStash {
    Acc<MT, NT> s[LEVELS > 0 ? LEVELS : 1];
};

template <int MT, int NT>
__device__ __forceinline__ void add_left_sibling(Acc<MT, NT> &acc, const Acc<MT, NT> &left) {
#pragma unroll
    for (int a = 0; a < MT; ++a)
#pragma unroll
        for (int b = 0; b < NT; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc.t[a][b][r] = left.t[a][b][r] + acc.t[a][b][r];
}

// Evaluates T over 2^L consecutive superleaves into acc (App. C), leaves in ascending k.
template <int L>
struct SubtreeWalker {
    template <class Leaf, class A, class S>
    __device__ __forceinline__ static void run(Leaf &leaf, A &acc, S &stash) {
#pragma nounroll
        for (int half = 0; half < 2; ++half) {
            SubtreeWalker<L - 1>::run(leaf, acc, stash);
            if (half == 0) stash.s[L - 1] = acc;
            else add_left_sibling(acc, stash.s[L - 1]);
        }
    }
};
template <>
struct SubtreeWalker<0> {
    template <class Leaf, class A, class S>
    __device__ __forceinline__ static void run(Leaf &leaf, A &acc, S &) { leaf(); }
};

struct TiledParams {
    const uint16_t *X;
    const uint16_t *W;
    float *partials;
    void *Y;
    int64_t ldx, ldw, ldy;
    int M, N;
    int y_bf16;
    int stages_per_superleaf;   // superleaf / BK
    int ns_per_shard;
    int64_t k_per_shard;
    int tiles_n;
};

// ---------------------------------------------------------------------------------------------
// BM = 32*MT*WM rows, BN = 32*NT*WN columns, WM*WN = 4 wavefronts.
template <int LEVELS, int WM, int WN, int MT, int NT>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
void gemm_tiled_kernel(const TiledParams p) {
    constexpr int BM = 32 * MT * WM, BN = 32 * NT * WN;
    constexpr int A_BYTES = BM * PITCH, B_BYTES = BN * PITCH;
    constexpr int A_CHUNKS = BM * (BK / 8);                 // 16-byte chunks of the X tile
    constexpr int A_PER_THREAD = (A_CHUNKS + 255) / 256;
    constexpr int B_BLOCKS = (BK / 4) * (BN / 8);           // 4(k) x 8(n) blocks of the W tile
    constexpr int B_PER_THREAD = (B_BLOCKS + 255) / 256;
    static_assert(WM * WN == 4, "four wavefronts");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr int STAGE_BYTES = A_BYTES + B_BYTES;          // stage layout: [X tile | W tile]

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int li = lane & 31, lg = lane >> 5;

    const int tile = blockIdx.x;
    const int tm = tile / p.tiles_n, tn = tile % p.tiles_n;
    const int m0 = tm * BM, n0 = tn * BN;
    const int shard = blockIdx.y;
    const int64_t kbase = (int64_t)shard * p.k_per_shard;

    // ---- global -> register staging ----
    uint4 areg[A_PER_THREAD];
    uint4 breg[B_PER_THREAD][4];

    // Rows past M and columns past N are never stored, and an output element depends only on its own
    // row of X and column of W, so out-of-range lanes simply re-read the last valid row / column block.
    auto gload = [&](int64_t k0) {
#pragma unroll
        for (int i = 0; i < A_PER_THREAD; ++i) {
            const int c = tid + 256 * i;
            const int row = min(m0 + (c >> 3), p.M - 1), kc = c & 7;
            if (A_CHUNKS % 256 == 0 || c < A_CHUNKS)
                areg[i] = *reinterpret_cast<const uint4 *>(p.X + (int64_t)row * p.ldx + k0 + kc * 8);
        }
#pragma unroll
        for (int i = 0; i < B_PER_THREAD; ++i) {
            const int b = tid + 256 * i;
            const int nblk = b % (BN / 8), kblk = b / (BN / 8);
            const int col = min(n0 + nblk * 8, p.N - 8);
            if (B_BLOCKS % 256 == 0 || b < B_BLOCKS) {
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    breg[i][t] = *reinterpret_cast<const uint4 *>(p.W + (k0 + kblk * 4 + t) * p.ldw + col);
            }
        }
    };

    auto lstore = [&](int buf) {
#pragma unroll
        for (int i = 0; i < A_PER_THREAD; ++i) {
            const int c = tid + 256 * i;
            const int row = c >> 3, kc = c & 7;
            if (c < A_CHUNKS) *reinterpret_cast<uint4 *>((smem + buf * STAGE_BYTES) + row * PITCH + kc * 16) = areg[i];
        }
#pragma unroll
        for (int i = 0; i < B_PER_THREAD; ++i) {
            const int b = tid + 256 * i;
            const int nblk = b % (BN / 8), kblk = b / (BN / 8);
            if (b < B_BLOCKS) {
                const uint32_t r0[4] = {breg[i][0].x, breg[i][0].y, breg[i][0].z, breg[i][0].w};
                const uint32_t r1[4] = {breg[i][1].x, breg[i][1].y, breg[i][1].z, breg[i][1].w};
                const uint32_t r2[4] = {breg[i][2].x, breg[i][2].y, breg[i][2].z, breg[i][2].w};
                const uint32_t r3[4] = {breg[i][3].x, breg[i][3].y, breg[i][3].z, breg[i][3].w};
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    // column 2q: low halves of word q of the four k rows; column 2q+1: high halves
                    const uint2 even = make_uint2((r0[q] & 0xffffu) | (r1[q] << 16), (r2[q] & 0xffffu) | (r3[q] << 16));
                    const uint2 odd = make_uint2((r0[q] >> 16) | (r1[q] & 0xffff0000u), (r2[q] >> 16) | (r3[q] & 0xffff0000u));
                    unsigned char *dst = (smem + buf * STAGE_BYTES + A_BYTES) + (nblk * 8 + 2 * q) * PITCH + kblk * 8;
                    *reinterpret_cast<uint2 *>(dst) = even;
                    *reinterpret_cast<uint2 *>(dst + PITCH) = odd;
                }
            }
        }
    };

    Acc<MT, NT> acc;
    TileStash<LEVELS, MT, NT> stash;

    const int total_stages = p.ns_per_shard * p.stages_per_superleaf;
    gload(kbase);
    lstore(0);
    __syncthreads();

    int s = 0;             // global stage counter of the software pipeline (runs across superleaves)

    // One superleaf: accumulators start at +0, then stages_per_superleaf LDS stages of MFMA chains.
    auto superleaf = [&]() {
#pragma unroll
        for (int a = 0; a < MT; ++a)
#pragma unroll
            for (int b = 0; b < NT; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc.t[a][b][r] = 0.0f;
#pragma nounroll
        for (int q = 0; q < p.stages_per_superleaf; ++q, ++s) {
            const int buf = s & 1;
            if (s + 1 < total_stages) gload(kbase + (int64_t)(s + 1) * BK);
            const unsigned char *Ab = (smem + buf * STAGE_BYTES) + (wm * MT * 32 + li) * PITCH + lg * 16;
            const unsigned char *Bb = (smem + buf * STAGE_BYTES + A_BYTES) + (wn * NT * 32 + li) * PITCH + lg * 16;
#pragma unroll
            for (int ks = 0; ks < BK / 16; ++ks) {
                bf16x8 af[MT], bfr[NT];
#pragma unroll
                for (int a = 0; a < MT; ++a) af[a] = *reinterpret_cast<const bf16x8 *>(Ab + a * 32 * PITCH + ks * 32);
#pragma unroll
                for (int b = 0; b < NT; ++b) bfr[b] = *reinterpret_cast<const bf16x8 *>(Bb + b * 32 * PITCH + ks * 32);
#pragma unroll
                for (int a = 0; a < MT; ++a)
#pragma unroll
                    for (int b = 0; b < NT; ++b)
                        acc.t[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[a], bfr[b], acc.t[a][b], 0, 0, 0);
            }
            if (s + 1 < total_stages) lstore(buf ^ 1);
            __syncthreads();
        }
    };

    // The shard's subtree of depth LEVELS, walked as nested two-trip loops: the first trip of the
    // loop at level l leaves its subtree sum in the stash slot of that level, the second trip adds
    // the slot to its own sum (left sibling + right sibling).  Every slot is named statically.
    SubtreeWalker<LEVELS>::run(superleaf, acc, stash);

    // ---- epilogue: acc holds T(superleaves of this shard) ----
    float *part = p.partials ? p.partials + (int64_t)shard * p.M * p.N : nullptr;
#pragma unroll
    for (int a = 0; a < MT; ++a) {
#pragma unroll
        for (int b = 0; b < NT; ++b) {
            const int col = n0 + (wn * NT + b) * 32 + li;
            if (col >= p.N) continue;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + (wm * MT + a) * 32 + 8 * (r >> 2) + 4 * lg + (r & 3);
                if (row >= p.M) continue;
                const float v = acc.t[a][b][r];
                if (part) part[(int64_t)row * p.N + col] = v;
                if (p.Y) {
                    if (p.y_bf16) reinterpret_cast<uint16_t *>(p.Y)[(int64_t)row * p.ldy + col] = (uint16_t)f32_to_bf16_bits(v);
                    else reinterpret_cast<float *>(p.Y)[(int64_t)row * p.ldy + col] = v;
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------

static int levels_for(int ns_per_shard) {
    int l = 0;
    while ((1 << l) < ns_per_shard) ++l;
    return l;
}

bool gemm_tiled_supports(const GemmArgs &a, int variant) {
    if (variant != VARIANT_T128 && variant != VARIANT_T32) return false;
    if (a.N % 8 != 0 || a.superleaf % BK != 0) return false;
    if (levels_for(a.ns / a.P) > 4) return false;
    if ((int64_t)a.P > 65535) return false;
    return true;
}

template <int WM, int WN, int MT, int NT>
static hipError_t launch_shape(const GemmArgs &a, hipStream_t s) {
    constexpr int BM = 32 * MT * WM, BN = 32 * NT * WN;
    TiledParams p;
    p.X = a.X; p.W = a.W; p.partials = a.partials; p.Y = (a.P == 1) ? a.Y : nullptr;
    p.ldx = a.ldx; p.ldw = a.ldw; p.ldy = a.ldy;
    p.M = a.M; p.N = a.N;
    p.y_bf16 = (a.y_dtype == TBIK_BF16);
    p.stages_per_superleaf = a.superleaf / BK;
    p.ns_per_shard = a.ns / a.P;
    p.k_per_shard = (int64_t)a.K / a.P;
    p.tiles_n = (a.N + BN - 1) / BN;
    const int64_t tiles = (int64_t)p.tiles_n * ((a.M + BM - 1) / BM);
    if (tiles > 0x7fffffff) return hipErrorInvalidValue;
    dim3 grid((unsigned)tiles, a.P), block(256);
    const size_t lds = 2 * (size_t)(BM + BN) * PITCH;
    const int levels = levels_for(p.ns_per_shard);
#define TBIK_LAUNCH(L)                                                                                   \
    case L: {                                                                                            \
        auto k = gemm_tiled_kernel<L, WM, WN, MT, NT>;                                                   \
        hipError_t e = hipFuncSetAttribute((const void *)k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); \
        if (e != hipSuccess) return e;                                                                   \
        hipLaunchKernelGGL(k, grid, block, lds, s, p);                                                   \
        break;                                                                                           \
    }
    switch (levels) {
        TBIK_LAUNCH(0)
        TBIK_LAUNCH(1)
        TBIK_LAUNCH(2)
        TBIK_LAUNCH(3)
        TBIK_LAUNCH(4)
        default: return hipErrorInvalidValue;
    }
#undef TBIK_LAUNCH
    return hipGetLastError();
}

hipError_t launch_gemm_tiled(const GemmArgs &a, int variant, hipStream_t s) {
    if (a.M <= 0 || a.N <= 0) return hipSuccess;
    if (!gemm_tiled_supports(a, variant)) return hipErrorInvalidValue;
    if (variant == VARIANT_T128) return launch_shape<2, 2, 2, 2>(a, s);   // 128 x 128, wave tile 64 x 64
    return launch_shape<1, 4, 1, 1>(a, s);                                // 32 x 128, wave tile 32 x 32
}

}  // namespace tbik
