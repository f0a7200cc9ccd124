// Tree-Based MatMul on OCP MXFP6 operands for gfx950: 6-bit E2M3 or E3M2 elements, 32 of them (one block) in 24
// bytes, one E8M0 (power-of-two) scale per block, for the activations and for the weight alike.
//
// The method is that of the other formats (Sec. 4.2, App. C, App. D.1, Alg. 1): a superleaf's products are accumulated
// in ascending k from +0, the superleaf sums are combined by the tree T.  A scaled 6-bit product has at most eight
// significant bits: exact in fp32.  The matrix instruction is v_mfma_scale_f32_32x32x64_f8f6f4 with both operands in
// a 6-bit format: 64 k per instruction; lane l carries row (or column) l % 32 and the 32 consecutive k of half l / 32
// of the step -- 24 bytes in six registers, exactly one block, whose scale the lane hands over in a byte of a register
// (measured with one element moved through all positions: a lane's 32 elements take the lane's own scale, as for 4-bit
// operands and unlike 8-bit ones; the elements are one little-endian bit stream, element e in bits 6 e .. 6 e + 5).
// The packing runs along k, so the weight is taken TRANSPOSED: Wt [N, 3 K / 4] bytes, Ws [N, K / 32] scales.
//
// Two kernels that must agree bit for bit: a reference (one wavefront per 32 x 32 tile and shard, operands straight
// from global memory) and the tiled kernel (128 x 128 tile, 4 wavefronts of 64 x 64, stages of 128 k = 96 bytes per
// row plus 4 scale bytes per row, a ring of 4 LDS slots of 33 KiB filled by direct global->LDS loads).
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
typedef int i32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// One MFMA: D = A(32 x 64) * B(64 x 32) + C, both operands in the 6-bit format FMT (2 = E2M3, 3 = E3M2) in the low
// six registers of the operand, each lane's 32 elements times 2^(scale - 127) with the lane's scale in the low byte of
// sa / sb.
template <int FMT>
__device__ __forceinline__ f32x16 mfma_32x32x64_mxfp6(i32x2 a0, i32x2 a1, i32x2 a2, i32x2 b0, i32x2 b1, i32x2 b2, f32x16 c, int sa, int sb) {
    const i32x8 a8 = {a0[0], a0[1], a1[0], a1[1], a2[0], a2[1], 0, 0}, b8 = {b0[0], b0[1], b1[0], b1[1], b2[0], b2[1], 0, 0};
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a8, b8, c, FMT, FMT, 0, sa, 0, sb);
}

constexpr int REF_MAX_LEVELS = 28;

template <int FMT>
__global__ __launch_bounds__(64) void gemm_mxfp6_reference_kernel(
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
            const int64_t blk = (k0 + kk) / 32 + g;                      // the lane's block of 32 k: 24 bytes, 8-byte aligned
            const i32x2 *a = reinterpret_cast<const i32x2 *>(X + xr * ldx + blk * 24);
            const i32x2 *b = reinterpret_cast<const i32x2 *>(Wt + wr * ldw + blk * 24);
            acc = mfma_32x32x64_mxfp6<FMT>(a[0], a[1], a[2], b[0], b[1], b[2], acc, Xs[xr * ldxs + blk], Ws[wr * ldws + blk]);
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
// Tiled kernel, 128 x 128.  A stage is 128 k: 96 bytes of each of the 128 rows of the X tile and of the Wt tile, and
// four scale bytes per row.  96 is not a power of two, so a row's stage is kept in two parts: its first 64 bytes
// (16-byte chunks 0 .. 3) in an area of 64-byte rows and its last 32 bytes (chunks 4, 5) in an area of 32-byte rows.
// A stage slot is cut into four regions of 8 KiB, one per loading wavefront, which brings 32 rows of each tile:
//   [X first parts, 2 KiB | X last parts, 1 KiB | 1 KiB unused | Wt first parts, 2 KiB | Wt last parts, 1 KiB | 1 KiB unused]
// (the unused KiB make the region as large as the output patch that the epilogue puts there), then 1 KiB of scales:
// 128 x 4 bytes of the X rows, then of the Wt rows.  Chunk c < 4 of row r sits at position c ^ ((r >> 2) & 3) of its
// 64-byte row, chunk 4 + c at position c ^ ((r >> 3) & 1) of its 32-byte row.  A lane's operand for one MFMA is block
// b = 2 ks + lg of its row, bytes 24 b .. 24 b + 23: three 8-byte reads (a block starts in the middle of a chunk when b
// is odd, and an 8-byte piece never straddles two chunks).
constexpr int BK6 = 128;               // k per stage
constexpr int ROWB6 = 96;              // bytes of a row per stage
constexpr int KSTEPS6 = 2;             // MFMA K-steps per stage
constexpr int REGION6 = 8192;
constexpr int SCALES_AT6 = 4 * REGION6;
constexpr int STAGE6 = SCALES_AT6 + 1024;

template <int N>
__device__ __forceinline__ void wait_loads_and_barrier() {
    static_assert(N >= 0 && N < 64, "vmcnt range");
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(N) : "memory");
}

struct Mx6Params {
    const uint8_t *X, *Xs, *Wt, *Ws;   // Xs, Ws: [rows, ld] scale bytes -- or, scales_packed, the re-tiled copies
    float *partials;
    void *Y;
    int64_t ldx, ldxs, ldw, ldws, ldy;
    int M, N;
    int y_bf16;
    int stages_per_superleaf;   // superleaf / 128
    int ns_per_shard;
    int64_t k_per_shard;
    int tiles_n, tiles, work;
    int vector_stores;
    int stream_stores;
    int scales_packed;          // the scales were re-tiled by mx_scales_retile_kernel<1> (blocks of 128 rows)
    int stages_total;           // K / 128
};

template <int LEVELS, int RING6, int FMT>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
void gemm_mxfp6_tiled_kernel(const Mx6Params p) {
    constexpr int WM = 2, WN = 2, MT = 2, NT = 2;
    constexpr int BM = 32 * MT * WM, BN = 32 * NT * WN;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int li = lane & 31, lg = lane >> 5;
    const int stages_per_item = p.ns_per_shard * p.stages_per_superleaf;
    const bool wave_is_x = __builtin_amdgcn_readfirstlane(wave) < 2;      // whose scales this wavefront fetches

    // ---- global -> LDS (global_load_lds_dwordx4: lane i's 16 bytes land at LDS base + 16 i) ----
    // Per wavefront and stage, for each of the two tiles: two loads of first parts (16 rows x 4 chunks each) and one of
    // last parts (32 rows x 2 chunks); the lane fetches the chunk that belongs at its position (the swizzle is applied
    // on the global side).  All six share one m0 (the start of the Wt half of the wavefront's region): instruction
    // offsets -4, -3, -2 KiB for X and 0, 1, 2 KiB for Wt; the lane offsets are biased so that the global side of the
    // instruction offset cancels.  Then one 256-byte load of scales (wavefronts 0, 1: rows 0 .. 63, 64 .. 127 of the X
    // tile; 2, 3: of the Wt tile).  Rows past M or N re-read the last valid row: theirs are never stored.
    constexpr int LOADS_PER_STAGE = 7;
    constexpr int WCOLS = 32 * NT;
    constexpr int STORES_F32 = MT * (32 * WCOLS / 4 / 64);
    constexpr int STORES_BF16 = MT * (32 * WCOLS / 8 / 64);
    static_assert(LOADS_PER_STAGE * (RING6 - 1) + STORES_F32 < 64 && STORES_F32 != STORES_BF16, "vmcnt range");
    static_assert(REGION6 >= 32 * WCOLS * 4, "the output patch must fit a wavefront's region of a slot");
    constexpr int LANE_BIAS = 4096;
    unsigned aoff[3], boff[3], soff = 0;
    const char *a_ptr = nullptr, *b_ptr = nullptr, *s_ptr = nullptr;

    auto point_loads_at = [&](int item) __attribute__((always_inline)) {
        const int tile = item % p.tiles, shard = item / p.tiles;
        const int m0 = (tile / p.tiles_n) * BM, n0 = (tile % p.tiles_n) * BN;
        const int64_t kbase = (int64_t)shard * p.k_per_shard;
        a_ptr = uniform_pointer(reinterpret_cast<const char *>(p.X + (int64_t)m0 * p.ldx + kbase / 4 * 3) - LANE_BIAS);
        b_ptr = uniform_pointer(reinterpret_cast<const char *>(p.Wt + (int64_t)n0 * p.ldw + kbase / 4 * 3) - LANE_BIAS);
#pragma unroll
        for (int j = 0; j < 3; ++j) {
            // j = 0, 1: first parts of rows 32 w + 16 j + lane / 4, position lane % 4; j = 2: last parts of rows 32 w + lane / 2
            const int r = wave * 32 + (j < 2 ? 16 * j + (lane >> 2) : (lane >> 1));
            const int c = j < 2 ? ((lane & 3) ^ ((r >> 2) & 3)) : 4 + ((lane & 1) ^ ((r >> 3) & 1));
            aoff[j] = (unsigned)(min(r, p.M - 1 - m0) * (int)p.ldx + c * 16) + (unsigned)(LANE_BIAS + (4 - j) * 1024);
            boff[j] = (unsigned)(min(r, p.N - 1 - n0) * (int)p.ldw + c * 16) + (unsigned)(LANE_BIAS - j * 1024);
        }
        const int rs = (wave & 1) * 64 + lane;
        if (p.scales_packed) {                         // a stage's scale bytes of a row block are consecutive: two cache lines per load
            const int64_t stage0 = kbase / BK6;
            const char *xs = reinterpret_cast<const char *>(p.Xs) + ((int64_t)(m0 / BM) * p.stages_total + stage0) * (BM * 4);
            const char *ws = reinterpret_cast<const char *>(p.Ws) + ((int64_t)(n0 / BN) * p.stages_total + stage0) * (BN * 4);
            s_ptr = uniform_pointer(wave_is_x ? xs : ws);
            soff = (unsigned)(4 * rs);
        } else {                                       // straight from the caller's [rows, K / 32] arrays: a cache line per lane
            const char *xs = reinterpret_cast<const char *>(p.Xs + (int64_t)m0 * p.ldxs + kbase / 32);
            const char *ws = reinterpret_cast<const char *>(p.Ws + (int64_t)n0 * p.ldws + kbase / 32);
            s_ptr = uniform_pointer(wave_is_x ? xs : ws);
            soff = wave_is_x ? (unsigned)(min(rs, p.M - 1 - m0) * (int)p.ldxs) : (unsigned)(min(rs, p.N - 1 - n0) * (int)p.ldws);
        }
    };

    const unsigned smem_lds = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const unsigned m0_in_stage = smem_lds + wave_u * REGION6 + 4096;
    const unsigned m0_scales = smem_lds + SCALES_AT6 + wave_u * 256;        // X rows 0 .. 127, then Wt rows 0 .. 127, four bytes each
    const int s_step = !p.scales_packed ? BK6 / 32 : (wave_u < 2 ? BM * 4 : BN * 4);     // scale bytes per stage
    int issue_item = blockIdx.x;
    int issue_stage = 0;
    // The loads of the next stage in four parts, which the caller spreads over the MFMAs of the stage it multiplies.
    auto issue_part = [&](int slot, auto part_c) __attribute__((always_inline)) {
        constexpr int PART = decltype(part_c)::value;
        if (PART == 0 && __builtin_expect(issue_stage == stages_per_item, 0)) {
            if (issue_item + (int)gridDim.x < p.work) {
                issue_item += gridDim.x;
                point_loads_at(issue_item);
                issue_stage = 0;
            } else {                                   // past the end: load the last stage again (nobody consumes it)
                issue_stage = stages_per_item - 1;
                a_ptr -= ROWB6;
                b_ptr -= ROWB6;
                s_ptr -= s_step;
            }
        }
        const unsigned m0v = m0_in_stage + slot * STAGE6;
        if constexpr (PART < 3) {
            load_16B_per_lane_to_lds<(PART - 4) * 1024, PART == 0>(a_ptr, aoff[PART], m0v);
            load_16B_per_lane_to_lds<PART * 1024, false>(b_ptr, boff[PART], m0v);
        } else {
            load_4B_per_lane_to_lds<0, true>(s_ptr, soff, m0_scales + slot * STAGE6);
            s_ptr += s_step;
            ++issue_stage;
            a_ptr += ROWB6;
            b_ptr += ROWB6;
        }
    };
    auto issue_next_stage = [&](int slot) {
        issue_part(slot, Int<0>{});
        issue_part(slot, Int<1>{});
        issue_part(slot, Int<2>{});
        issue_part(slot, Int<3>{});
    };

    // ---- LDS fragment addresses (bytes inside a stage) ----
    // Tile row R lies in region R / 32 at row R % 32 = li; the X half of a region starts at 0, the Wt half at 4 KiB.
    int f_off[MT + NT], s_off[MT + NT];
#pragma unroll
    for (int a = 0; a < MT; ++a) {
        f_off[a] = (wm * MT + a) * REGION6;
        s_off[a] = SCALES_AT6 + ((wm * MT + a) * 32 + li) * 4;
    }
#pragma unroll
    for (int b = 0; b < NT; ++b) {
        f_off[MT + b] = (wn * NT + b) * REGION6 + 4096;
        s_off[MT + b] = SCALES_AT6 + 512 + ((wn * NT + b) * 32 + li) * 4;
    }
    // piece q of block 2 ks + lg: bytes o = 24 (2 ks + lg) + 8 q of the row's stage, i.e. chunk o / 16 at o % 16
    int piece_off[KSTEPS6][3];
#pragma unroll
    for (int ks = 0; ks < KSTEPS6; ++ks)
#pragma unroll
        for (int q = 0; q < 3; ++q) {
            const int o = 24 * (2 * ks + lg) + 8 * q, c = o >> 4;
            piece_off[ks][q] = (c < 4 ? li * 64 + ((c ^ ((li >> 2) & 3)) << 4) : 2048 + li * 32 + (((c - 4) ^ ((li >> 3) & 1)) << 4)) + (o & 15);
        }

    // Fragment registers: one set per K-step of a stage; the reads run one K-step ahead.
    i32x2 fr[KSTEPS6][MT + NT][3];
    constexpr int READS_PER_KSTEP = 3 * (MT + NT);
    auto read_frag_op = [&](int r, int set, int slot, int ks) {
        const unsigned char *sb = smem + slot * STAGE6;
        const int f = r / 3, q = r % 3;
        fr[set][f][q] = *reinterpret_cast<const i32x2 *>(sb + f_off[f] + piece_off[ks][q]);
    };
    auto read_frags = [&](int set, int slot, int ks) {
#pragma unroll
        for (int r = 0; r < READS_PER_KSTEP; ++r) read_frag_op(r, set, slot, ks);
    };
    // The four scale bytes of each of the lane's rows, fetched once per stage (for the next stage after the last K-step's
    // bytes are taken out).
    unsigned scl[MT + NT];
    auto read_scales = [&](int slot) {
        const unsigned char *sb = smem + slot * STAGE6;
#pragma unroll
        for (int f = 0; f < MT + NT; ++f) scl[f] = *reinterpret_cast<const unsigned *>(sb + s_off[f]);
    };

    Acc<MT, NT> acc, acc2;
    TileStash<LEVELS - 1, MT, NT> stash;

    // Software pipeline over the ring, as in the other tiled kernels: at the top of stage s wait until this wavefront's
    // loads of stage s+1 have landed, meet the other wavefronts -- stage s+1 is complete, nobody reads the slot of stage
    // s-1 any more -- and start the loads of stage s+RING-1 into that slot.
    point_loads_at(issue_item);
#pragma unroll
    for (int i = 0; i < RING6 - 1; ++i) issue_next_stage(i);
    wait_loads_and_barrier<LOADS_PER_STAGE * (RING6 - 2)>();
    read_frags(0, 0, 0);
    read_scales(0);

    int cur = 0;
    int stores_in_flight = 0;          // output stores share the counter of the loads (see the 16-bit kernel)

    auto stage = [&](auto first, Acc<MT, NT> &a) {
        constexpr bool FIRST = decltype(first)::value;
        const int nxt = (cur + 1 == RING6) ? 0 : cur + 1;
        constexpr int ALLOW = LOADS_PER_STAGE * (RING6 - 3);
        if (__builtin_expect(stores_in_flight == 0, 1)) {
            wait_loads_and_barrier<ALLOW>();
        } else {
            if (stores_in_flight == STORES_F32) wait_loads_and_barrier<ALLOW + STORES_F32>();
            else if (stores_in_flight == STORES_BF16) wait_loads_and_barrier<ALLOW + STORES_BF16>();
            else wait_loads_and_barrier<0>();
            stores_in_flight = 0;
        }
        const int free_slot = cur == 0 ? RING6 - 1 : cur - 1;
        constexpr int NM = MT * NT;
#pragma unroll
        for (int ks = 0; ks < KSTEPS6; ++ks) {
            const bool ahead_in_stage = ks + 1 < KSTEPS6;
            const int t_set = ahead_in_stage ? ks + 1 : 0;
            const int t_slot = ahead_in_stage ? cur : nxt;
            int sc[MT + NT];
#pragma unroll
            for (int f = 0; f < MT + NT; ++f) sc[f] = (int)__builtin_amdgcn_ubfe(scl[f], 16u * ks + 8u * lg, 8u);
            if (ks == KSTEPS6 - 1) read_scales(nxt);           // the next stage's, complete in LDS since this stage's barrier
#pragma unroll
            for (int m = 0; m < NM; ++m) {
                const int i = m / NT, j = m % NT;
                const f32x16 zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
                const int set = (FIRST && ks == 0) ? 0 : ks;
                a.t[i][j] = mfma_32x32x64_mxfp6<FMT>(fr[set][i][0], fr[set][i][1], fr[set][i][2], fr[set][MT + j][0], fr[set][MT + j][1],
                                                     fr[set][MT + j][2], (FIRST && ks == 0) ? zero : a.t[i][j], sc[i], sc[MT + j]);
                // this MFMA's share of the LDS reads of the next K-step and of the loads of the stage being fetched
#pragma unroll
                for (int r = m * READS_PER_KSTEP / NM; r < (m + 1) * READS_PER_KSTEP / NM; ++r)
                    read_frag_op(r, t_set, t_slot, t_set);
                {
                    constexpr int G = KSTEPS6 * NM;
                    const int gi = ks * NM + m;
                    if (gi == (0 * G) / 4) issue_part(free_slot, Int<0>{});
                    if (gi == (1 * G) / 4) issue_part(free_slot, Int<1>{});
                    if (gi == (2 * G) / 4) issue_part(free_slot, Int<2>{});
                    if (gi == (3 * G) / 4) issue_part(free_slot, Int<3>{});
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
            static_assert(REGION6 >= 32 * WCOLS * 4, "the output patch must fit a wavefront's region of a slot");
            const int last_slot = cur == 0 ? RING6 - 1 : cur - 1;
            float *patch = reinterpret_cast<float *>(smem + last_slot * STAGE6 + wave * REGION6);
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

template <int FMT>
hipError_t launch_mx6(const GemmArgs &a, const Mxfp4Scales &sc, hipStream_t s) {
    constexpr int BM = 128, BN = 128, RING6 = 4;
    static_assert(RING6 * STAGE6 <= 160 * 1024, "LDS of a compute unit");
    Mx6Params p;
    p.X = reinterpret_cast<const uint8_t *>(a.X); p.Wt = reinterpret_cast<const uint8_t *>(a.W);
    p.Xs = sc.Xs; p.Ws = sc.Ws;
    p.scales_packed = sc.packed;
    p.stages_total = a.K / BK6;
    p.partials = a.partials; p.Y = (a.P == 1) ? a.Y : nullptr;
    p.ldx = a.ldx; p.ldw = a.ldw; p.ldxs = sc.ldxs; p.ldws = sc.ldws; p.ldy = a.ldy;
    p.M = a.M; p.N = a.N;
    p.y_bf16 = (a.y_dtype != TBIK_F32);
    p.stages_per_superleaf = a.superleaf / BK6;
    p.ns_per_shard = a.ns / a.P;
    p.k_per_shard = (int64_t)a.K / a.P;
    p.tiles_n = (a.N + BN - 1) / BN;
    const int64_t tiles = (int64_t)p.tiles_n * ((a.M + BM - 1) / BM);
    if (tiles * a.P > 0x7fffffff) return hipErrorInvalidValue;
    p.tiles = (int)tiles;
    p.work = (int)(tiles * a.P);
    const int grid_x = p.work < compute_units() ? p.work : compute_units();
    dim3 grid((unsigned)grid_x), block(256);
    const size_t lds = (size_t)RING6 * STAGE6;
    const void *out = p.partials ? (const void *)p.partials : p.Y;
    const int64_t ld_bytes = p.partials ? (int64_t)a.N * 4 : a.ldy * (p.y_bf16 ? 2 : 4);
    p.vector_stores = ((reinterpret_cast<uintptr_t>(out) & 15) == 0) && (ld_bytes % 16 == 0);
    p.stream_stores = a.partials != nullptr && (int64_t)a.P * a.M * a.N * 4 > ((int64_t)192 << 20);
    const int levels = levels_for(p.ns_per_shard);
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 32) dev = 32;
#define TBIK_LAUNCH6(L)                                                                                  \
    case L: {                                                                                            \
        auto k = gemm_mxfp6_tiled_kernel<L, RING6, FMT>;                                                 \
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
        TBIK_LAUNCH6(0)
        TBIK_LAUNCH6(1)
        TBIK_LAUNCH6(2)
        TBIK_LAUNCH6(3)
        TBIK_LAUNCH6(4)
        default: return hipErrorInvalidValue;
    }
#undef TBIK_LAUNCH6
    return hipGetLastError();
}

}  // namespace

// a.x_dtype names the element format: TBIK_FP6_E2M3 or TBIK_FP6_E3M2.
bool gemm_mxfp6_tiled_supports(const GemmArgs &a, const Mxfp4Scales &sc) {
    if (a.superleaf % BK6 != 0) return false;
    if (levels_for(a.ns / a.P) > 4) return false;
    if (a.ldx >= (1 << 22) || a.ldw >= (1 << 22) || sc.ldxs >= (1 << 24) || sc.ldws >= (1 << 24)) return false;   // 32-bit lane offsets
    const auto a4 = [](const void *q) { return (reinterpret_cast<uintptr_t>(q) & 3) == 0; };
    const auto a16 = [](const void *q) { return (reinterpret_cast<uintptr_t>(q) & 15) == 0; };
    if (!a16(a.X) || !a16(a.W) || a.ldx % 16 != 0 || a.ldw % 16 != 0) return false;       // 16-byte chunks
    if (!a4(sc.Xs) || !a4(sc.Ws) || sc.ldxs % 4 != 0 || sc.ldws % 4 != 0) return false;   // a row's four scale bytes per stage: one aligned dword
    return true;
}

size_t mxfp6_retiled_scales_bytes(int M, int N, int K) { return mx_retiled_scales_bytes<1>(M, N, K / BK6); }

// packed_ws: nullptr, or mxfp6_retiled_scales_bytes(M, N, K) bytes (4-byte aligned) into which the scales are re-tiled
// first (one short launch).
hipError_t launch_gemm_mxfp6_tiled(const GemmArgs &a, const Mxfp4Scales &sc, void *packed_ws, hipStream_t s) {
    if (a.M <= 0 || a.N <= 0) return hipSuccess;
    if (!gemm_mxfp6_tiled_supports(a, sc)) return hipErrorInvalidValue;
    Mxfp4Scales use = sc;
    if (packed_ws) {
        hipError_t e = launch_mx_scales_retile<1>(sc.Xs, sc.ldxs, a.M, 128, sc.Ws, sc.ldws, a.N, a.K / BK6, packed_ws, &use.Xs, &use.Ws, s);
        if (e != hipSuccess) return e;
        use.packed = 1;
    }
    return a.x_dtype == TBIK_FP6_E3M2 ? launch_mx6<3>(a, use, s) : launch_mx6<2>(a, use, s);
}

hipError_t launch_gemm_mxfp6_reference(const GemmArgs &a, const Mxfp4Scales &sc, hipStream_t s) {
    if (a.M <= 0 || a.N <= 0) return hipSuccess;
    if (a.superleaf % 64 != 0) return hipErrorInvalidValue;
    dim3 grid((a.N + 31) / 32, (a.M + 31) / 32, a.P);
    if (grid.y > 65535u || grid.z > 65535u) return hipErrorInvalidValue;
    void *Y = (a.P == 1) ? a.Y : nullptr;
    auto kernel = (a.x_dtype == TBIK_FP6_E3M2) ? gemm_mxfp6_reference_kernel<3> : gemm_mxfp6_reference_kernel<2>;
    hipLaunchKernelGGL(kernel, grid, dim3(64), 0, s, reinterpret_cast<const uint8_t *>(a.X), a.ldx, sc.Xs, sc.ldxs,
                       reinterpret_cast<const uint8_t *>(a.W), a.ldw, sc.Ws, sc.ldws, a.partials, Y, a.ldy, a.y_dtype, a.M, a.N,
                       a.superleaf, a.ns / a.P);
    return hipGetLastError();
}

}  // namespace tbik
