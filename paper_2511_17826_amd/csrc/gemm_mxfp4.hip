// Tree-Based MatMul on OCP MXFP4 operands for gfx950: 4-bit E2M1 elements, one E8M0 (power-of-two) scale per block of
// 32 consecutive k, for the activations and for the weight alike.
//
// The method is that of the other formats (Sec. 4.2, App. C, App. D.1, Alg. 1): a superleaf's products are accumulated
// in ascending k from +0, the superleaf sums are combined by the tree T.  A scaled 4-bit product has at most four
// significant bits: exact in fp32.  The matrix instruction is v_mfma_scale_f32_32x32x64_f8f6f4 with both operands in
// the 4-bit format: 64 k per instruction; lane l carries row (or column) l % 32 and the 32 consecutive k of half l / 32
// of the step -- 16 bytes, exactly one scale block, whose scale the lane hands over in a byte of a register.  The
// packing runs along k, so the weight is taken TRANSPOSED like the 8-bit one: Wt [N, K/2] bytes, Ws [N, K/32] scales.
//
// Two kernels that must agree bit for bit: a reference (one wavefront per 32 x 32 tile and shard, operands straight
// from global memory) and the tiled kernel (128 x 128 tile, 4 wavefronts of 64 x 64, stages of 256 k = 128 bytes per
// row plus 8 scale bytes per row, a ring of 4 LDS slots of 34 KiB filled by direct global->LDS loads).
#include <atomic>
#include <type_traits>

#include "mx_scales.hpp"
#include "tbik_device.hpp"
#include "tbik_internal.hpp"
#include "tree_walk.hpp"

namespace tbik {

namespace {

template <int V>
using Int = std::integral_constant<int, V>;

typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// One MFMA: D = A(32 x 64) * B(64 x 32) + C, both operands E2M1 (format code 4) in the low four registers of the
// operand, each lane's 32 elements times 2^(scale - 127) with the lane's scale in the low byte of sa / sb.
__device__ __forceinline__ f32x16 mfma_32x32x64_mxfp4(i32x4 a, i32x4 b, f32x16 c, int sa, int sb) {
    const i32x8 a8 = {a[0], a[1], a[2], a[3], 0, 0, 0, 0}, b8 = {b[0], b[1], b[2], b[3], 0, 0, 0, 0};
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a8, b8, c, 4, 4, 0, sa, 0, sb);
}

constexpr int REF_MAX_LEVELS = 28;

__global__ __launch_bounds__(64) void gemm_mxfp4_reference_kernel(
        const uint8_t *__restrict__ X, int64_t ldx, const uint8_t *__restrict__ Xs, int64_t ldxs,
        const uint8_t *__restrict__ Wt, int64_t ldw, const uint8_t *__restrict__ Ws, int64_t ldws,
        float *__restrict__ partials, void *__restrict__ Y, int64_t ldy, int y_dtype,
        int M, int N, int superleaf, int ns_per_shard) {
    const int lane = threadIdx.x;
    const int i = lane & 31;      // row of X / row of Wt (= output column) held by this lane
    const int g = lane >> 5;      // which half of a step of 64 k
    const int m0 = blockIdx.y * 32, n0 = blockIdx.x * 32;
    const int p = blockIdx.z;
    const int64_t kbase = (int64_t)p * ns_per_shard * superleaf;
    const bool row_ok = (m0 + i) < M;
    const bool col_ok = (n0 + i) < N;
    const int64_t xr = row_ok ? m0 + i : 0, wr = col_ok ? n0 + i : 0;   // rows past the edge compute on a valid row, never stored

    float stash[REF_MAX_LEVELS][16];
    f32x16 acc;
    for (int j = 0; j < ns_per_shard; ++j) {
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
        const int64_t k0 = kbase + (int64_t)j * superleaf;
        for (int kk = 0; kk < superleaf; kk += 64) {
            const int64_t k = k0 + kk + 32 * g;
            const i32x4 a = *reinterpret_cast<const i32x4 *>(X + xr * ldx + k / 2);
            const i32x4 b = *reinterpret_cast<const i32x4 *>(Wt + wr * ldw + k / 2);
            const int sa = Xs[xr * ldxs + k / 32], sb = Ws[wr * ldws + k / 32];
            acc = mfma_32x32x64_mxfp4(a, b, acc, sa, sb);
        }
        const int t = __builtin_ctz(~(unsigned)j);     // carry-over: as many finished subtrees as j has trailing ones
        for (int l = 0; l < t; ++l) {
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = stash[l][r] + acc[r];
        }
        if (j + 1 < ns_per_shard) {
#pragma unroll
            for (int r = 0; r < 16; ++r) stash[t][r] = acc[r];
        }
    }
    const int col = n0 + i;
    if (!col_ok) return;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int row = m0 + 8 * (r >> 2) + 4 * g + (r & 3);
        if (row >= M) continue;
        if (partials) partials[((int64_t)p * M + row) * N + col] = acc[r];
        if (Y) {
            if (y_dtype == TBIK_F32) reinterpret_cast<float *>(Y)[(int64_t)row * ldy + col] = acc[r];
            else reinterpret_cast<uint16_t *>(Y)[(int64_t)row * ldy + col] = (uint16_t)f32_to_bf16_bits(acc[r]);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Tiled kernel.  A stage is 256 k: a [128 rows x 128 bytes] tile of X, one of Wt, and 8 scale bytes per row of each.
// A stage slot: four regions of 8 KiB, one per loading wavefront, [32 rows of the X tile | 32 rows of the Wt tile]
// (rows of 128 bytes, the 16-byte chunk c of row r at position c ^ ((r >> 1) & 7): the layout of the 8-bit kernel), then
// the X scales (row r at 8 r) and the Wt scales.  A lane's operand for one MFMA is chunk 2 ks + lg of its row and its
// scale is byte 2 ks + lg of the row's eight.
constexpr int BKB = 128;               // bytes of k per LDS stage row (256 k)
// Three tile shapes as for the other formats: 128 x 128, and 64 x 128 / 32 x 128 (four wavefronts side by side) for small
// batches, where the 4-bit weight is the traffic.  The X scale area always has four 256-byte parts, one per loading
// wavefront: wavefront w brings the scales of rows (32 w) mod BM onward, so with fewer than 128 rows some parts repeat
// others, and a reader takes row R from part R / 32.
constexpr int KSTEPS4 = 4;             // MFMA K-steps (64 k) per stage
constexpr int B_LOADS4 = 4;            // 1 KiB loads of Wt rows per wavefront and stage

template <int N>
__device__ __forceinline__ void wait_loads_and_barrier() {
    static_assert(N >= 0 && N < 64, "vmcnt range");
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(N) : "memory");
}

struct Mx4Params {
    const uint8_t *X, *Xs, *Wt, *Ws;
    float *partials;
    void *Y;
    int64_t ldx, ldxs, ldw, ldws, ldy;
    int M, N;
    int y_bf16;
    int stages_per_superleaf;   // superleaf / 256
    int ns_per_shard;
    int64_t k_per_shard;
    int tiles_n, tiles, work;
    int vector_stores;
    int stream_stores;
    int scales_packed;          // Xs, Ws are the re-tiled copies (mx_scales_retile_kernel<2>, blocks of this launch's tile height)
    int stages_total;           // K / 256
};

typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

template <int LEVELS, int WM, int WN, int MT, int NT, int RING4>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
void gemm_mxfp4_tiled_kernel(const Mx4Params p) {
    constexpr int BM = 32 * MT * WM, BN = 32 * NT * WN;
    static_assert(BN == 128 && WM * WN == 4, "tile shape");
    constexpr int A_LOADS4 = BM / 32;                           // 1 KiB loads of X rows per wavefront and stage
    constexpr int REGION4 = (A_LOADS4 + B_LOADS4) * 1024;
    constexpr int SCALES_AT = 4 * REGION4;                      // offset of the X scales in a slot; the Wt scales follow 1 KiB later
    constexpr int STAGE4 = SCALES_AT + 2048;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int li = lane & 31, lg = lane >> 5;
    const int stages_per_item = p.ns_per_shard * p.stages_per_superleaf;

    // ---- global -> LDS ----
    // Per wavefront and stage: four 1 KiB loads of X rows, four of Wt rows (as in the 8-bit kernel: one m0, instruction
    // offsets -4 .. 3 KiB), then two 256-byte loads of scales (4 bytes per lane: lanes 2 r', 2 r' + 1 bring the eight
    // scale bytes of row 32 w + r'), with an m0 of their own.
    constexpr int LOADS_PER_STAGE = A_LOADS4 + B_LOADS4 + 2;
    constexpr int WCOLS = 32 * NT;
    constexpr int STORES_F32 = MT * (32 * WCOLS / 4 / 64);
    constexpr int STORES_BF16 = MT * (32 * WCOLS / 8 / 64);
    static_assert(LOADS_PER_STAGE * (RING4 - 1) + STORES_F32 < 64 && STORES_F32 != STORES_BF16, "vmcnt range");
    constexpr int LANE_BIAS = 4096;
    unsigned aoff[A_LOADS4], boff[B_LOADS4], xsoff, wsoff;
    const char *a_ptr = nullptr, *b_ptr = nullptr, *xs_ptr = nullptr, *ws_ptr = nullptr;
    int issue_item = blockIdx.x;
    int issue_stage = 0;

    auto point_loads_at = [&](int item) __attribute__((always_inline)) {
        const int tile = item % p.tiles, shard = item / p.tiles;
        const int m0 = (tile / p.tiles_n) * BM, n0 = (tile % p.tiles_n) * BN;
        const int64_t kbase = (int64_t)shard * p.k_per_shard;
        a_ptr = uniform_pointer(reinterpret_cast<const char *>(p.X + (int64_t)m0 * p.ldx + kbase / 2));
        b_ptr = uniform_pointer(reinterpret_cast<const char *>(p.Wt + (int64_t)n0 * p.ldw + kbase / 2) - LANE_BIAS);
        if (p.scales_packed) {                         // a stage's scale bytes of a row block are consecutive: two cache lines per load
            const int64_t stage0 = kbase / 256;
            xs_ptr = uniform_pointer(reinterpret_cast<const char *>(p.Xs) + ((int64_t)(m0 / BM) * p.stages_total + stage0) * (BM * 8));
            ws_ptr = uniform_pointer(reinterpret_cast<const char *>(p.Ws) + ((int64_t)(n0 / BN) * p.stages_total + stage0) * (BN * 8) - 1024);
        } else {                                       // straight from the caller's [rows, K / 32] arrays: a cache line per row
            xs_ptr = uniform_pointer(reinterpret_cast<const char *>(p.Xs + (int64_t)m0 * p.ldxs + kbase / 32));
            ws_ptr = uniform_pointer(reinterpret_cast<const char *>(p.Ws + (int64_t)n0 * p.ldws + kbase / 32) - 1024);
        }
#pragma unroll
        for (int j = 0; j < A_LOADS4; ++j) {
            const int r = (wave * A_LOADS4 + j) * 8 + (lane >> 3);
            const int c = (lane & 7) ^ ((r >> 1) & 7);
            aoff[j] = (unsigned)(min(r, p.M - 1 - m0) * (int)p.ldx + c * 16) + (unsigned)((A_LOADS4 - j) * 1024);
        }
#pragma unroll
        for (int j = 0; j < B_LOADS4; ++j) {
            const int r = (wave * B_LOADS4 + j) * 8 + (lane >> 3);
            const int c = (lane & 7) ^ ((r >> 1) & 7);
            boff[j] = (unsigned)(min(r, p.N - 1 - n0) * (int)p.ldw + c * 16) + (unsigned)(LANE_BIAS - j * 1024);
        }
        const int rs = wave * 32 + (lane >> 1);
        if (p.scales_packed) {
            xsoff = (unsigned)((rs % BM) * 8 + 4 * (lane & 1));
            wsoff = (unsigned)(rs * 8 + 4 * (lane & 1));
        } else {
            xsoff = (unsigned)(min(rs % BM, p.M - 1 - m0) * (int)p.ldxs + 4 * (lane & 1));
            wsoff = (unsigned)(min(rs, p.N - 1 - n0) * (int)p.ldws + 4 * (lane & 1));    // + 1024 - 1024: the Wt scales' instruction offset
        }
    };

    const unsigned smem_lds = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const unsigned m0_in_stage = smem_lds + wave_u * REGION4 + A_LOADS4 * 1024;
    const unsigned m0_scales = smem_lds + SCALES_AT + wave_u * 256;
    const int xs_step = p.scales_packed ? BM * 8 : 8, ws_step = p.scales_packed ? BN * 8 : 8;   // scale bytes per stage
    auto issue_part = [&](int slot, auto part_c) __attribute__((always_inline)) {
        constexpr int PART = decltype(part_c)::value;
        if (PART == 0 && __builtin_expect(issue_stage == stages_per_item, 0)) {
            if (issue_item + (int)gridDim.x < p.work) {
                issue_item += gridDim.x;
                point_loads_at(issue_item);
                issue_stage = 0;
            } else {                                   // past the end: load the last stage again (nobody consumes it)
                issue_stage = stages_per_item - 1;
                a_ptr -= BKB;
                b_ptr -= BKB;
                xs_ptr -= xs_step;
                ws_ptr -= ws_step;
            }
        }
        const unsigned m0v = m0_in_stage + slot * STAGE4;
        if constexpr (PART < A_LOADS4) load_16B_per_lane_to_lds<(PART - A_LOADS4) * 1024, PART == 0>(a_ptr, aoff[PART], m0v);
        load_16B_per_lane_to_lds<PART * 1024, false>(b_ptr, boff[PART], m0v);
        if (PART == B_LOADS4 - 1) {
            const unsigned m0s = m0_scales + slot * STAGE4;
            load_4B_per_lane_to_lds<0, true>(xs_ptr, xsoff, m0s);
            load_4B_per_lane_to_lds<1024, false>(ws_ptr, wsoff, m0s);
            ++issue_stage;
            a_ptr += BKB;
            b_ptr += BKB;
            xs_ptr += xs_step;
            ws_ptr += ws_step;
        }
    };
    auto issue_next_stage = [&](int slot) {
        issue_part(slot, Int<0>{});
        issue_part(slot, Int<1>{});
        issue_part(slot, Int<2>{});
        issue_part(slot, Int<3>{});
    };

    // ---- LDS fragment addresses (bytes inside a stage) ----
    int a_off[MT], b_off[NT], as_off[MT], bs_off[NT];
#pragma unroll
    for (int a = 0; a < MT; ++a) {
        const int R = (wm * MT + a) * 32 + li;
        a_off[a] = (R / (8 * A_LOADS4)) * REGION4 + (R % (8 * A_LOADS4)) * BKB;
        as_off[a] = SCALES_AT + R * 8;
    }
#pragma unroll
    for (int b = 0; b < NT; ++b) {
        b_off[b] = (wn * NT + b) * REGION4 + A_LOADS4 * 1024 + li * BKB;
        bs_off[b] = SCALES_AT + 1024 + ((wn * NT + b) * 32 + li) * 8;
    }
    const int sw = (li >> 1) & 7;
    int c_off[KSTEPS4];
#pragma unroll
    for (int ks = 0; ks < KSTEPS4; ++ks) c_off[ks] = ((2 * ks + lg) ^ sw) << 4;
    const unsigned sh_even = 8u * lg, sh_odd = 16u + 8u * lg;   // bit position of scale byte 2 ks + lg in its dword, ks even / odd

    // Fragment registers: two sets, the reads run one K-step ahead of the MFMAs.  Scales: the eight bytes of each of
    // the lane's four rows, fetched once per stage (for the next stage after the last K-step's bytes are taken out).
    i32x4 fr[2][MT + NT];
    u32x2 scl[MT + NT];
    auto read_frag_op = [&](int f, int set, int slot, int ks) {
        const unsigned char *sb = smem + slot * STAGE4;
        fr[set][f] = *reinterpret_cast<const i32x4 *>(sb + (f < MT ? a_off[f] : b_off[f - MT]) + c_off[ks]);
    };
    auto read_scales = [&](int slot) {
        const unsigned char *sb = smem + slot * STAGE4;
#pragma unroll
        for (int f = 0; f < MT + NT; ++f) scl[f] = *reinterpret_cast<const u32x2 *>(sb + (f < MT ? as_off[f] : bs_off[f - MT]));
    };

    Acc<MT, NT> acc, acc2;
    TileStash<LEVELS - 1, MT, NT> stash;

    point_loads_at(issue_item);
#pragma unroll
    for (int i = 0; i < RING4 - 1; ++i) issue_next_stage(i);
    wait_loads_and_barrier<LOADS_PER_STAGE * (RING4 - 2)>();      // stage 0 landed everywhere
#pragma unroll
    for (int f = 0; f < MT + NT; ++f) read_frag_op(f, 0, 0, 0);
    read_scales(0);

    int cur = 0;
    int stores_in_flight = 0;          // output stores share the counter of the loads (see the 16-bit kernel)

    auto stage = [&](auto first, Acc<MT, NT> &a) {
        constexpr bool FIRST = decltype(first)::value;
        const int nxt = (cur + 1 == RING4) ? 0 : cur + 1;
        constexpr int ALLOW = LOADS_PER_STAGE * (RING4 - 3);
        if (__builtin_expect(stores_in_flight == 0, 1)) {
            wait_loads_and_barrier<ALLOW>();                  // stage s+1 landed; the slot of stage s-1 is free
        } else {
            if (stores_in_flight == STORES_F32) wait_loads_and_barrier<ALLOW + STORES_F32>();
            else if (stores_in_flight == STORES_BF16) wait_loads_and_barrier<ALLOW + STORES_BF16>();
            else wait_loads_and_barrier<0>();
            stores_in_flight = 0;
        }
        const int free_slot = cur == 0 ? RING4 - 1 : cur - 1;
        constexpr int NM = MT * NT;
#pragma unroll
        for (int ks = 0; ks < KSTEPS4; ++ks) {
            const bool ahead_in_stage = ks + 1 < KSTEPS4;
            const int t_ks = ahead_in_stage ? ks + 1 : 0;
            const int t_slot = ahead_in_stage ? cur : nxt;
            // this K-step's scale bytes: byte 2 ks + lg of each row's eight
            int sc[MT + NT];
#pragma unroll
            for (int f = 0; f < MT + NT; ++f)
                sc[f] = (int)__builtin_amdgcn_ubfe(scl[f][ks >> 1], (ks & 1) ? sh_odd : sh_even, 8u);
            if (ks == KSTEPS4 - 1) read_scales(nxt);           // the next stage's, complete in LDS since this stage's barrier
#pragma unroll
            for (int m = 0; m < NM; ++m) {
                const int i = m / NT, j = m % NT;
                if (FIRST && ks == 0) {
                    const f32x16 zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
                    a.t[i][j] = mfma_32x32x64_mxfp4(fr[0][i], fr[0][MT + j], zero, sc[i], sc[MT + j]);
                } else {
                    a.t[i][j] = mfma_32x32x64_mxfp4(fr[ks & 1][i], fr[ks & 1][MT + j], a.t[i][j], sc[i], sc[MT + j]);
                }
#pragma unroll
                for (int f = m * (MT + NT) / NM; f < (m + 1) * (MT + NT) / NM; ++f)
                    read_frag_op(f, (ks + 1) & 1, t_slot, t_ks);   // this MFMA's share of the next K-step's fragments
                if (m == NM - 1) {                             // one part of the next stage's loads per K-step
                    if (ks == 0) issue_part(free_slot, Int<0>{});
                    if (ks == 1) issue_part(free_slot, Int<1>{});
                    if (ks == 2) issue_part(free_slot, Int<2>{});
                    if (ks == 3) issue_part(free_slot, Int<3>{});
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        cur = nxt;
    };

    auto superleaf = [&](Acc<MT, NT> &a) {
        stage(std::true_type{}, a);
#pragma nounroll
        for (int q = 1; q < p.stages_per_superleaf; ++q) stage(std::false_type{}, a);
    };

    for (int item = blockIdx.x; item < p.work; item += gridDim.x) {
        SubtreeWalker<LEVELS>::run(superleaf, acc, acc2, stash);

        const int tile = item % p.tiles, shard = item / p.tiles;
        const int m0 = (tile / p.tiles_n) * BM, n0 = (tile % p.tiles_n) * BN;
        float *part = p.partials ? p.partials + (int64_t)shard * p.M * p.N : nullptr;
        const bool interior = (m0 + BM <= p.M) && (n0 + BN <= p.N);
        if (interior && p.vector_stores) {
            // Each wavefront turns its 32 x 64 blocks around in its own region of the slot that was multiplied last
            // (nothing is loaded into it before the next stage's barrier; the barrier here is for the other wavefronts'
            // fragment reads), so that a lane stores 16 consecutive bytes.  A fixed number of store instructions.
            static_assert(REGION4 >= 32 * WCOLS * 4, "the output patch must fit a wavefront's region of a slot");
            const int last_slot = cur == 0 ? RING4 - 1 : cur - 1;
            float *patch = reinterpret_cast<float *>(smem + last_slot * STAGE4 + wave * REGION4);
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
            const bool to_bf16 = (part == nullptr) && p.y_bf16;
            const int wm_u = wave_u / WN, wn_u = wave_u % WN;
            const int col0 = n0 + wn_u * WCOLS;
            if (to_bf16) {
                constexpr int CPR = WCOLS / 8, RPI = 64 / CPR, N_IT = 32 / RPI;
                const int lrow = lane / CPR, lc = lane % CPR;
                const float *rd = patch + lrow * WCOLS + lc * 8;
                const unsigned lane_off = (unsigned)(lrow * (int)p.ldy + lc * 8) * 2u;
                const int64_t it_step = (int64_t)RPI * p.ldy * 2;
#pragma unroll
                for (int a = 0; a < MT; ++a) {
#pragma unroll
                    for (int b = 0; b < NT; ++b)
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            patch[(8 * (r >> 2) + 4 * lg + (r & 3)) * WCOLS + b * 32 + li] = acc.t[a][b][r];
                    f32x4 lo[N_IT], hi[N_IT];
#pragma unroll
                    for (int it = 0; it < N_IT; ++it) {
                        lo[it] = *reinterpret_cast<const f32x4 *>(rd + it * RPI * WCOLS);
                        hi[it] = *reinterpret_cast<const f32x4 *>(rd + it * RPI * WCOLS + 4);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                    char *base = reinterpret_cast<char *>(reinterpret_cast<uint16_t *>(p.Y) +
                                                          (int64_t)(m0 + (wm_u * MT + a) * 32) * p.ldy + col0);
#pragma unroll
                    for (int it = 0; it < N_IT; ++it) {
                        u32x4 o;
                        o[0] = pack_bf16x2(lo[it][0], lo[it][1]);
                        o[1] = pack_bf16x2(lo[it][2], lo[it][3]);
                        o[2] = pack_bf16x2(hi[it][0], hi[it][1]);
                        o[3] = pack_bf16x2(hi[it][2], hi[it][3]);
                        *reinterpret_cast<u32x4 *>(base + it * it_step + lane_off) = o;
                    }
                }
            } else {
                constexpr int CPR = WCOLS / 4, RPI = 64 / CPR, N_IT = 32 / RPI;
                float *dst = part ? part : reinterpret_cast<float *>(p.Y);
                const int64_t ld = part ? p.N : p.ldy;
                const int lrow = lane / CPR, lc = lane % CPR;
                const float *rd = patch + lrow * WCOLS + lc * 4;
                const unsigned lane_off = (unsigned)(lrow * (int)ld + lc * 4) * 4u;
                const int64_t it_step = (int64_t)RPI * ld * 4;
#pragma unroll
                for (int a = 0; a < MT; ++a) {
#pragma unroll
                    for (int b = 0; b < NT; ++b)
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            patch[(8 * (r >> 2) + 4 * lg + (r & 3)) * WCOLS + b * 32 + li] = acc.t[a][b][r];
                    f32x4 v[N_IT];
#pragma unroll
                    for (int it = 0; it < N_IT; ++it) v[it] = *reinterpret_cast<const f32x4 *>(rd + it * RPI * WCOLS);
                    __builtin_amdgcn_sched_barrier(0);
                    char *base = reinterpret_cast<char *>(dst + (int64_t)(m0 + (wm_u * MT + a) * 32) * ld + col0);
                    if (p.stream_stores) {
#pragma unroll
                        for (int it = 0; it < N_IT; ++it)
                            asm volatile("global_store_dwordx4 %0, %1, off nt" ::"v"(base + it * it_step + lane_off), "v"(v[it]) : "memory");
                    } else {
#pragma unroll
                        for (int it = 0; it < N_IT; ++it) *reinterpret_cast<f32x4 *>(base + it * it_step + lane_off) = v[it];
                    }
                }
            }
            stores_in_flight = to_bf16 ? STORES_BF16 : STORES_F32;
        } else {
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
            stores_in_flight = -1;
        }
    }
    wait_loads_and_barrier<0>();                          // no load may still be writing LDS when the workgroup ends
}

int levels_for(int ns_per_shard) {
    int l = 0;
    while ((1 << l) < ns_per_shard) ++l;
    return l;
}

int compute_units() {
    static int cus = 0;
    if (cus == 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
            cus = n;
        else
            cus = 256;
    }
    return cus;
}

}  // namespace

hipError_t launch_gemm_mxfp4_reference(const GemmArgs &a, const Mxfp4Scales &sc, hipStream_t s) {
    if (a.M <= 0 || a.N <= 0) return hipSuccess;
    if (a.superleaf % 64 != 0) return hipErrorInvalidValue;
    dim3 grid((a.N + 31) / 32, (a.M + 31) / 32, a.P);
    if (grid.y > 65535u || grid.z > 65535u) return hipErrorInvalidValue;
    void *Y = (a.P == 1) ? a.Y : nullptr;
    hipLaunchKernelGGL(gemm_mxfp4_reference_kernel, grid, dim3(64), 0, s, reinterpret_cast<const uint8_t *>(a.X), a.ldx,
                       sc.Xs, sc.ldxs, reinterpret_cast<const uint8_t *>(a.W), a.ldw, sc.Ws, sc.ldws, a.partials, Y, a.ldy,
                       a.y_dtype, a.M, a.N, a.superleaf, a.ns / a.P);
    return hipGetLastError();
}


bool gemm_mxfp4_tiled_supports(const GemmArgs &a, const Mxfp4Scales &sc) {
    if (a.superleaf % 256 != 0) return false;
    if (levels_for(a.ns / a.P) > 4) return false;
    if (a.ldx >= (1 << 22) || a.ldw >= (1 << 22) || sc.ldxs >= (1 << 22) || sc.ldws >= (1 << 22)) return false;   // 32-bit lane offsets
    const auto a8 = [](const void *q) { return (reinterpret_cast<uintptr_t>(q) & 7) == 0; };
    if (!a8(sc.Xs) || !a8(sc.Ws) || sc.ldxs % 8 != 0 || sc.ldws % 8 != 0) return false;   // a row's eight scale bytes per stage: two aligned dwords
    return true;
}

template <int WM, int WN, int MT, int NT, int RING4>
static hipError_t launch_mx4_shape(const GemmArgs &a, const Mxfp4Scales &sc, hipStream_t s) {
    constexpr int BM = 32 * MT * WM, BN = 32 * NT * WN;
    constexpr int STAGE4 = 4 * (BM / 32 + B_LOADS4) * 1024 + 2048;
    Mx4Params p;
    p.X = reinterpret_cast<const uint8_t *>(a.X); p.Wt = reinterpret_cast<const uint8_t *>(a.W);
    p.Xs = sc.Xs; p.Ws = sc.Ws;
    p.scales_packed = sc.packed;
    p.stages_total = a.K / 256;
    p.partials = a.partials; p.Y = (a.P == 1) ? a.Y : nullptr;
    p.ldx = a.ldx; p.ldw = a.ldw; p.ldxs = sc.ldxs; p.ldws = sc.ldws; p.ldy = a.ldy;
    p.M = a.M; p.N = a.N;
    p.y_bf16 = (a.y_dtype != TBIK_F32);
    p.stages_per_superleaf = a.superleaf / 256;
    p.ns_per_shard = a.ns / a.P;
    p.k_per_shard = (int64_t)a.K / a.P;
    p.tiles_n = (a.N + BN - 1) / BN;
    const int64_t tiles = (int64_t)p.tiles_n * ((a.M + BM - 1) / BM);
    if (tiles * a.P > 0x7fffffff) return hipErrorInvalidValue;
    p.tiles = (int)tiles;
    p.work = (int)(tiles * a.P);
    const int grid_x = p.work < compute_units() ? p.work : compute_units();
    dim3 grid((unsigned)grid_x), block(256);
    const size_t lds = (size_t)RING4 * STAGE4;
    const void *out = p.partials ? (const void *)p.partials : p.Y;
    const int64_t ld_bytes = p.partials ? (int64_t)a.N * 4 : a.ldy * (p.y_bf16 ? 2 : 4);
    p.vector_stores = ((reinterpret_cast<uintptr_t>(out) & 15) == 0) && (ld_bytes % 16 == 0);
    p.stream_stores = a.partials != nullptr && (int64_t)a.P * a.M * a.N * 4 > ((int64_t)192 << 20);
    const int levels = levels_for(p.ns_per_shard);
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 32) dev = 32;
#define TBIK_LAUNCH4(L)                                                                                  \
    case L: {                                                                                            \
        auto k = gemm_mxfp4_tiled_kernel<L, WM, WN, MT, NT, RING4>;                                      \
        static std::atomic<unsigned> lds_allowed{0};                                                     \
        if (dev >= 32 || !((lds_allowed.load(std::memory_order_relaxed) >> dev) & 1u)) {                 \
            hipError_t e = hipFuncSetAttribute((const void *)k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); \
            if (e != hipSuccess) return e;                                                               \
            if (dev < 32) lds_allowed.fetch_or(1u << dev, std::memory_order_relaxed);                    \
        }                                                                                                \
        hipLaunchKernelGGL(k, grid, block, lds, s, p);                                                   \
        break;                                                                                           \
    }
    switch (levels) {
        TBIK_LAUNCH4(0)
        TBIK_LAUNCH4(1)
        TBIK_LAUNCH4(2)
        TBIK_LAUNCH4(3)
        TBIK_LAUNCH4(4)
        default: return hipErrorInvalidValue;
    }
#undef TBIK_LAUNCH4
    return hipGetLastError();
}

size_t mxfp4_retiled_scales_bytes(int M, int N, int K) { return mx_retiled_scales_bytes<2>(M, N, K / 256); }

// packed_ws: nullptr, or mxfp4_retiled_scales_bytes(M, N, K) bytes (4-byte aligned) into which the scales are re-tiled
// first (one short launch), after which every scale load of the GEMM touches two cache lines instead of 32.
hipError_t launch_gemm_mxfp4_tiled(const GemmArgs &a, const Mxfp4Scales &sc, int rows, void *packed_ws, hipStream_t s) {
    if (a.M <= 0 || a.N <= 0) return hipSuccess;
    if (!gemm_mxfp4_tiled_supports(a, sc) || (rows != 32 && rows != 64 && rows != 128)) return hipErrorInvalidValue;
    Mxfp4Scales use = sc;
    if (packed_ws) {
        hipError_t e = launch_mx_scales_retile<2>(sc.Xs, sc.ldxs, a.M, rows, sc.Ws, sc.ldws, a.N, a.K / 256, packed_ws, &use.Xs, &use.Ws, s);
        if (e != hipSuccess) return e;
        use.packed = 1;
    }
    if (rows == 32) return launch_mx4_shape<1, 4, 1, 1, 7>(a, use, s);     // 7 x 22 KiB slots
    if (rows == 64) return launch_mx4_shape<1, 4, 2, 1, 6>(a, use, s);     // 6 x 26 KiB
    return launch_mx4_shape<2, 2, 2, 2, 4>(a, use, s);                     // 4 x 34 KiB
}

}  // namespace tbik
