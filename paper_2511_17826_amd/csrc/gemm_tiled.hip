// Tiled Tree-Based MatMul kernels (App. D.1, Alg. 1) for gfx950.
//
// A workgroup of 4 wavefronts owns one BM x 128 output tile of one K-shard and walks the shard's
// superleaves in ascending k.  Per superleaf each wavefront chains v_mfma_f32_32x32x16_bf16 over
// ascending groups of 16 k into accumulators that start at +0 (the same opcode and k -> (step,
// slot) map as the reference kernel, which is what makes all variants bit-identical); when a
// superleaf ends, the carry-over step folds the accumulators into the stash of waiting subtrees,
// which lives in registers (one wavefront per SIMD, up to 512 VGPR+AGPR per lane).
//
// Operands are staged through LDS in K-steps of 64 (three stage buffers), both in their global
// orientation, written with 16-byte stores:
//   X tile [BM][64]  rows of 128 B; the 16-byte chunk c of row r sits at position c ^ ((r>>1)&7),
//                    so the 16 rows of a fragment read (ds_read_b128) hit all 64 banks once;
//   W tile [64][128] rows of 256 B; chunk c of row k sits at position c ^ (4*(k&3)); the MFMA's
//                    B operand (8 consecutive k of one column per lane) is fetched with the
//                    transposing LDS read ds_read_b64_tr_b16, whose 16-lane groups read 4 rows x
//                    16 columns: with the swizzle the 4 rows fall into different banks.
#include "tbik_device.hpp"
#include "tbik_internal.hpp"

namespace tbik {

constexpr int BK = 64;                 // K-elements per LDS stage
constexpr int BN_TILE = 128;           // columns per workgroup tile
constexpr int A_ROW = BK * 2;          // bytes per LDS row of the X tile
constexpr int B_ROW = BN_TILE * 2;     // bytes per LDS row of the W tile

// Stash levels kept in registers by the 128x128 tile (the rest go to LDS).
#ifndef TBIK_ABLATE
#define TBIK_ABLATE 0   // development only: bit mask that removes pipeline pieces for timing experiments
#endif
#ifndef TBIK_MAX_REG_LEVELS
#define TBIK_MAX_REG_LEVELS 4
#endif

typedef short v4i16 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// Waits until at most N of this wavefront's vector-memory loads are outstanding, then joins the workgroup
// barrier.  Deliberately not __syncthreads(): its fence would wait for all loads.
template <int N>
__device__ __forceinline__ void wait_loads_and_barrier() {
    static_assert(N >= 0 && N < 64, "vmcnt range");
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(N) : "memory");
}

// global_load_lds_dwordx4: every lane fetches 16 bytes from its own global address; lane i's bytes land at
// LDS address m0 + 16*i.  Written in assembly so that the compiler does not see an LDS write it would
// guard with a full wait before later LDS reads; completion is tracked by hand with vmcnt (above).
__device__ __forceinline__ void load_16B_per_lane_to_lds(const void *gptr, unsigned lds_wave_base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_wave_base), "v"(gptr) : "memory", "m0");
}

template <int MT, int NT>              // 32x32 MFMA tiles per wavefront
struct Acc {
    f32x16 t[MT][NT];
};

// Stash of finished subtrees (App. D.1: accumulator buffer S[level]); every slot is addressed statically.
// Levels below REG_LEVELS live in registers; the levels above (written and read once per 2^level
// superleaves) live in LDS, 16 floats per lane and slot-row, each lane owning its own 16-byte columns.
template <int REG_LEVELS, int MT, int NT>
struct TileStash {
    Acc<MT, NT> s[REG_LEVELS > 0 ? REG_LEVELS : 1];
    unsigned char *lds;          // base of the LDS stash area (per workgroup)
    static constexpr int LDS_LEVEL_BYTES = MT * NT * 16 * 4 * 256;

    __device__ __forceinline__ void lds_store(int level, const Acc<MT, NT> &acc) const {
        f32x4 *dst = reinterpret_cast<f32x4 *>(lds + (level - REG_LEVELS) * LDS_LEVEL_BYTES) + threadIdx.x;
#pragma unroll
        for (int a = 0; a < MT; ++a)
#pragma unroll
            for (int b = 0; b < NT; ++b)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    f32x4 v = {acc.t[a][b][4 * q], acc.t[a][b][4 * q + 1], acc.t[a][b][4 * q + 2], acc.t[a][b][4 * q + 3]};
                    dst[((a * NT + b) * 4 + q) * 256] = v;
                }
    }
    __device__ __forceinline__ void lds_add_left(int level, Acc<MT, NT> &acc) const {
        const f32x4 *src = reinterpret_cast<const f32x4 *>(lds + (level - REG_LEVELS) * LDS_LEVEL_BYTES) + threadIdx.x;
#pragma unroll
        for (int a = 0; a < MT; ++a)
#pragma unroll
            for (int b = 0; b < NT; ++b)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const f32x4 v = src[((a * NT + b) * 4 + q) * 256];
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc.t[a][b][4 * q + e] = v[e] + acc.t[a][b][4 * q + e];
                }
    }
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
template <int L, int REG_LEVELS>
struct SubtreeWalker {
    template <class Leaf, class A, class S>
    __device__ __forceinline__ static void run(Leaf &leaf, A &acc, S &stash) {
#pragma nounroll
        for (int half = 0; half < 2; ++half) {
            SubtreeWalker<L - 1, REG_LEVELS>::run(leaf, acc, stash);
            if constexpr (L - 1 < REG_LEVELS) {
                if (half == 0) stash.s[L - 1] = acc;
                else add_left_sibling(acc, stash.s[L - 1]);
            } else {
                if (half == 0) stash.lds_store(L - 1, acc);
                else stash.lds_add_left(L - 1, acc);
            }
        }
    }
};
template <int REG_LEVELS>
struct SubtreeWalker<0, REG_LEVELS> {
    template <class Leaf, class A, class S>
    __device__ __forceinline__ static void run(Leaf &leaf, A &, S &) { leaf(); }
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
    static_assert(BN == BN_TILE && WM * WN == 4, "tile shape");
    constexpr int A_BYTES = BM * A_ROW, B_BYTES = BK * B_ROW;
    constexpr int STAGE_BYTES = A_BYTES + B_BYTES;          // stage layout: [X tile | W tile]

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int li = lane & 31, lg = lane >> 5;

    const int tile = blockIdx.x;
    const int tm = tile / p.tiles_n, tn = tile % p.tiles_n;
    const int m0 = tm * BM, n0 = tn * BN;
    const int shard = blockIdx.y;
    const int64_t kbase = (int64_t)shard * p.k_per_shard;

    // ---- global -> LDS, without passing through registers (global_load_lds_dwordx4) ----
    // One such instruction moves 64 x 16 bytes: lane i's chunk lands at LDS base + 16*i, so a
    // wavefront fills 1 KiB of consecutive LDS = 8 rows of the X tile or 4 rows of the W tile, and
    // the swizzle is applied on the global side (which chunk a lane fetches).  Rows past M and
    // columns past N are never stored, and an output element depends only on its own row of X and
    // column of W, so out-of-range lanes simply re-read the last valid row / column block.
    constexpr int A_LOADS = BM / 32;          // per wavefront and stage (BM rows / 8 rows / 4 wavefronts)
    constexpr int B_LOADS = BK / 16;          // 64 rows / 4 rows / 4 wavefronts
    const uint16_t *agp[A_LOADS];
#pragma unroll
    for (int j = 0; j < A_LOADS; ++j) {
        const int r = (wave * A_LOADS + j) * 8 + (lane >> 3);
        const int c = (lane & 7) ^ ((r >> 1) & 7);
        agp[j] = p.X + (int64_t)min(m0 + r, p.M - 1) * p.ldx + kbase + c * 8;
    }
    const uint16_t *bgp[B_LOADS];
#pragma unroll
    for (int j = 0; j < B_LOADS; ++j) {
        const int kk = (wave * B_LOADS + j) * 4 + (lane >> 4);
        const int c = (lane & 15) ^ ((lane >> 4) << 2);
        bgp[j] = p.W + (kbase + kk) * p.ldw + min(n0 + c * 8, p.N - 8);
    }
    const int64_t bstep = (int64_t)BK * p.ldw;

    const unsigned smem_lds = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    auto issue_stage = [&](int stage, int buf) {
        const unsigned base = smem_lds + buf * STAGE_BYTES;
#pragma unroll
        for (int j = 0; j < A_LOADS; ++j)
            load_16B_per_lane_to_lds(agp[j] + (int64_t)stage * BK, base + (wave_u * A_LOADS + j) * 1024);
#pragma unroll
        for (int j = 0; j < B_LOADS; ++j)
            load_16B_per_lane_to_lds(bgp[j] + (int64_t)stage * bstep, base + A_BYTES + (wave_u * B_LOADS + j) * 1024);
    };
    constexpr int LOADS_PER_STAGE = A_LOADS + B_LOADS;

    // ---- LDS fragment addresses (bytes inside a stage) ----
    // X fragment a: row wm*MT*32 + a*32 + li, chunk 2*ks + lg  ->  position (2*ks) ^ (lg ^ ((li>>1)&7)).
    const int a_row_off = (wm * MT * 32 + li) * A_ROW;
    const int a_sw = (lg ^ ((li >> 1) & 7)) << 4;
    // W fragment b, half h: a 16-lane group reads rows k0..k0+3 (k0 = 16*ks + 8*lg + 4*h), 16 columns.
    const int l16 = lane & 15, e = l16 >> 2;
    int b_off[NT];
#pragma unroll
    for (int b = 0; b < NT; ++b) {
        const int col = (wn * NT + b) * 32 + ((lane >> 4) & 1) * 16 + (l16 & 3) * 4;
        b_off[b] = A_BYTES + (lg * 8 + e) * B_ROW + ((((col >> 3) ^ (e << 2))) << 4) + ((col >> 2) & 1) * 8;
    }

    // big tiles keep at most three stash levels in registers, the rest in LDS behind the stage buffers
    constexpr int REG_LEVELS = (MT * NT >= 4 && LEVELS > TBIK_MAX_REG_LEVELS) ? TBIK_MAX_REG_LEVELS : LEVELS;
    Acc<MT, NT> acc;
    TileStash<REG_LEVELS, MT, NT> stash;
    stash.lds = smem + 4 * STAGE_BYTES;

    const int total_stages = p.ns_per_shard * p.stages_per_superleaf;

    // Fragment registers, double buffered over the K-steps of 16: while the MFMAs of one step run,
    // the LDS reads of the next step (or of the first step of the next stage) are in flight.
    bf16x8 af[2][MT], bfr[2][NT];
    auto read_frags = [&](int set, int buf, int ks) {
        const unsigned char *sb = smem + buf * STAGE_BYTES;
#pragma unroll
        for (int a = 0; a < MT; ++a)
            af[set][a] = *reinterpret_cast<const bf16x8 *>(sb + a_row_off + a * 32 * A_ROW + (a_sw ^ (ks << 5)));
#pragma unroll
        for (int b = 0; b < NT; ++b) {
            union { v4i16 h[2]; bf16x8 v; } u;
#pragma unroll
            for (int h = 0; h < 2; ++h)
                u.h[h] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) v4i16 *)(sb + b_off[b] + ks * 16 * B_ROW + h * 4 * B_ROW));
            bfr[set][b] = u.v;
        }
    };

    // Software pipeline over a ring of four LDS stage buffers.  At the top of stage s: wait until this
    // wavefront's loads of stage s+1 have landed (those of stage s+2 may still be in flight), meet the
    // other wavefronts at a barrier -- now stage s+1 is complete in LDS and nobody reads the buffer of
    // stage s-1 any more -- and start the loads of stage s+3 into that buffer.  The barrier is written
    // in assembly on purpose: a fence would make the compiler drain every outstanding load.
    issue_stage(0, 0);
    issue_stage(min(1, total_stages - 1), 1);
    issue_stage(min(2, total_stages - 1), 2);
    wait_loads_and_barrier<LOADS_PER_STAGE * 2>();      // stage 0 landed everywhere
    read_frags(0, 0, 0);

    int s = 0;             // global stage counter of the software pipeline (runs across superleaves)
    int cur = 0;           // ring slot of stage s

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
            const int nxt = (cur + 1) & 3;
            wait_loads_and_barrier<LOADS_PER_STAGE>();    // stage s+1 landed; stage s-1's buffer is free
            issue_stage(min(s + 3, total_stages - 1), (cur + 3) & 3);
#pragma unroll
            for (int ks = 0; ks < BK / 16; ++ks) {
                if (ks + 1 < BK / 16) read_frags((ks + 1) & 1, cur, ks + 1);
                else read_frags(0, nxt, 0);
#pragma unroll
                for (int a = 0; a < MT; ++a)
#pragma unroll
                    for (int b = 0; b < NT; ++b)
                        acc.t[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[ks & 1][a], bfr[ks & 1][b], acc.t[a][b], 0, 0, 0);
            }
            cur = nxt;
        }
    };

    // The shard's subtree of depth LEVELS, walked as nested two-trip loops: the first trip of the
    // loop at level l leaves its subtree sum in the stash slot of that level, the second trip adds
    // the slot to its own sum (left sibling + right sibling).  Every slot is named statically.
    SubtreeWalker<LEVELS, REG_LEVELS>::run(superleaf, acc, stash);
    wait_loads_and_barrier<0>();                          // no load may still be writing LDS when the workgroup ends

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
    const int levels = levels_for(p.ns_per_shard);
    const int lds_levels = (MT * NT >= 4 && levels > TBIK_MAX_REG_LEVELS) ? levels - TBIK_MAX_REG_LEVELS : 0;
    const size_t lds = 4 * ((size_t)BM * A_ROW + (size_t)BK * B_ROW) + (size_t)lds_levels * MT * NT * 16 * 4 * 256;
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
