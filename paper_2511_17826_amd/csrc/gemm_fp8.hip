// Tree-Based MatMul on 8-bit floating-point operands (OCP E4M3 / E5M2) for gfx950.
//
// The method is that of the 16-bit kernels (Sec. 4.2, App. C, App. D.1, Alg. 1): a superleaf's products are accumulated
// in ascending k from +0, the superleaf sums are combined by the tree T.  A product of two 8-bit floats has at most
// eight significant bits, so it is exact in fp32 like a product of two bf16 numbers.  The matrix instruction is
// v_mfma_f32_32x32x64_f8f6f4 (64 k per instruction, both operands 8-bit): lane l carries row (or column) l % 32 and 32
// of the step's 64 k, for A and for B alike.  The instruction takes a lane's first 16 bytes (of either half of the
// wavefront) as positions 0..31 and its second 16 bytes as 32..63, and adds the 64 products as a chain of four rounded
// steps of 16 positions; the kernels give half l / 32 bytes 16 h .. 16 h + 15 of the step's first and of its second
// 32 k, so that the instruction meets k in ascending order.  Because both operands want k-contiguous bytes,
// the weight is taken TRANSPOSED, Wt [N, K] -- one row per output channel, the layout 8-bit weights are stored in --
// and the two operand tiles are staged, swizzled and read in exactly the same way.
//
// Two kernels that must agree bit for bit: a reference (one wavefront per 32 x 32 tile and shard, operands straight
// from global memory) and the tiled kernel (128 x 128 tile, 4 wavefronts of 64 x 64, K-steps of 128 bytes through a ring
// of 5 LDS slots of 32 KiB filled by direct global->LDS loads, the tree's stash in registers).
//
// MX = true: the same two kernels on OCP MXFP8 operands -- every block of 32 consecutive k of a row of X and of Wt
// carries an E8M0 scale byte (2^(s - 127)), which the instruction takes from a byte of a register of the lanes of one
// half of the wavefront; a lane then holds 16 bytes of each of the step's two blocks.  A stage (128 k) also holds four
// scale bytes per row.
#include <atomic>
#include <type_traits>

#include "tbik_device.hpp"
#include "mx_scales.hpp"
#include "tbik_internal.hpp"
#include "tree_walk.hpp"

namespace tbik {

namespace {

template <int V>
using Int = std::integral_constant<int, V>;

typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// One MFMA: D = A(32 x 64) * B(64 x 32) + C.  FMT: 0 = E4M3 ("fp8"), 1 = E5M2 ("bf8"), for both operands; the block
// scales of the instruction family are not used (the unscaled opcode is selected for zero scale operands).
template <int FMT>
__device__ __forceinline__ f32x16 mfma_32x32x64_8bit(i32x8 a, i32x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, FMT, FMT, 0, 0, 0, 0);
}
// The same with each lane's 32 elements times 2^(scale - 127), the lane's scale in the low byte of sa / sb.
template <int FMT>
__device__ __forceinline__ f32x16 mfma_32x32x64_8bit_scaled(i32x8 a, i32x8 b, f32x16 c, int sa, int sb) {
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, FMT, FMT, 0, sa, 0, sb);
}

constexpr int REF_MAX_LEVELS = 28;

template <int FMT, bool MX>
__global__ __launch_bounds__(64) void gemm_fp8_reference_kernel(
        const uint8_t *__restrict__ X, int64_t ldx, const uint8_t *__restrict__ Wt, int64_t ldw,
        const uint8_t *__restrict__ Xs, int64_t ldxs, const uint8_t *__restrict__ Ws, int64_t ldws,   // MX only
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
    const uint8_t *xrow = X + (int64_t)(row_ok ? m0 + i : 0) * ldx;
    const uint8_t *wrow = Wt + (int64_t)(col_ok ? n0 + i : 0) * ldw;
    const uint8_t *xsrow = MX ? Xs + (int64_t)(row_ok ? m0 + i : 0) * ldxs : nullptr;
    const uint8_t *wsrow = MX ? Ws + (int64_t)(col_ok ? n0 + i : 0) * ldws : nullptr;

    float stash[REF_MAX_LEVELS][16];
    f32x16 acc;
    for (int j = 0; j < ns_per_shard; ++j) {
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
        const int64_t k0 = kbase + (int64_t)j * superleaf;
        for (int kk = 0; kk < superleaf; kk += 64) {
            const int64_t k = k0 + kk + 32 * g;
            union { i32x4 h[2]; i32x8 v; } a, b;
            // rows past M and columns past N compute on a valid row's data and are never stored.
            // The instruction takes a lane's first 16 bytes (of either half of the wavefront) as positions 0..31 of the
            // step and its second 16 bytes as positions 32..63, scales them by what the lanes of half 0 resp. half 1 hand
            // over (measured: an element moved through the 64 positions shows which scale reaches it) and adds the
            // products as a chain of four rounded steps of 16 positions.  So half g holds bytes 16 g .. 16 g + 15 of the
            // step's first 32 k and of its second 32 k: the instruction then meets k in ascending order, and with block
            // scales half g hands over the scale of block g.
            const int64_t kq = k0 + kk;
            a.h[0] = *reinterpret_cast<const i32x4 *>(xrow + kq + 16 * g);
            a.h[1] = *reinterpret_cast<const i32x4 *>(xrow + kq + 32 + 16 * g);
            b.h[0] = *reinterpret_cast<const i32x4 *>(wrow + kq + 16 * g);
            b.h[1] = *reinterpret_cast<const i32x4 *>(wrow + kq + 32 + 16 * g);
            if (MX) acc = mfma_32x32x64_8bit_scaled<FMT>(a.v, b.v, acc, xsrow[k >> 5], wsrow[k >> 5]);
            else acc = mfma_32x32x64_8bit<FMT>(a.v, b.v, acc);
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
// Tiled kernel.  A stage is 128 k: a [128 rows x 128 bytes] tile of X and one of Wt.  A stage slot is cut into four
// regions of 8 KiB, one per loading wavefront: [32 rows of the X tile | 32 rows of the Wt tile].  Rows are 128 bytes;
// the 16-byte chunk c of row r sits at position c ^ ((r >> 1) & 7), so the 16 rows that a ds_read_b128 pass touches
// cover all banks.  A lane's operand for one MFMA is chunks 4*ks + lg and 4*ks + 2 + lg of its row (with block scales a
// slot carries 1 KiB of scales behind the four regions: four bytes per row of the X tile, then of the Wt tile).
// Three tile shapes, as for 16-bit operands: 128 x 128 (wave tile 64 x 64), 64 x 128 and 32 x 128 (four wavefronts side by
// side) for small batches, where the weight is the traffic and a deeper ring keeps more of it in flight.
constexpr int BK8 = 128;               // k (= bytes) per LDS stage row
constexpr int ROW8 = 128;              // bytes per LDS row
constexpr int KSTEPS8 = BK8 / 64;      // MFMA K-steps per stage
constexpr int B_LOADS8 = 4;            // 1 KiB loads of Wt rows per wavefront and stage (128 rows / 8 rows / 4 wavefronts)

template <int N>
__device__ __forceinline__ void wait_loads_and_barrier() {
    static_assert(N >= 0 && N < 64, "vmcnt range");
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(N) : "memory");
}

struct Fp8Params {
    const uint8_t *X;
    const uint8_t *Wt;
    const uint8_t *Xs, *Ws;     // MX: E8M0 scales [M, ldxs], [N, ldws], one per 32 k -- or, scales_packed, the re-tiled copies
    int64_t ldxs, ldws;
    int scales_packed;          // the scales were re-tiled by mx_scales_retile_kernel to the tile height of this launch
    int stages_total;           // K / 128
    float *partials;
    void *Y;
    int64_t ldx, ldw, ldy;
    int M, N;
    int y_bf16;
    int stages_per_superleaf;   // superleaf / 128
    int ns_per_shard;
    int64_t k_per_shard;
    int tiles_n, tiles, work;
    int vector_stores;
    int stream_stores;
};

template <int LEVELS, int WM, int WN, int MT, int NT, int RING8, int FMT, bool MX>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
void gemm_fp8_tiled_kernel(const Fp8Params p) {
    constexpr int BM = 32 * MT * WM, BN = 32 * NT * WN;
    static_assert(BN == 128 && WM * WN == 4, "tile shape");
    constexpr int A_LOADS8 = BM / 32;                           // 1 KiB loads of X rows per wavefront and stage
    constexpr int REGION8 = (A_LOADS8 + B_LOADS8) * 1024;       // [8 * A_LOADS8 rows of X | 32 rows of Wt] per loading wavefront
    constexpr int SCALES_AT = 4 * REGION8;                      // MX: 128 x 4 scale bytes of the X rows, then of the Wt rows
    constexpr int STAGE8 = 4 * REGION8 + (MX ? 1024 : 0);
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int li = lane & 31, lg = lane >> 5;
    const int stages_per_item = p.ns_per_shard * p.stages_per_superleaf;
    const bool wave_is_x = __builtin_amdgcn_readfirstlane(wave) < 2;      // MX: whose scales this wavefront fetches

    // ---- global -> LDS (global_load_lds_dwordx4: lane i's 16 bytes land at LDS base + 16 i) ----
    // Load j of wavefront w brings rows 32 w + 8 j + (lane >> 3) of a tile; the lane fetches the chunk that belongs at
    // its position (the swizzle is applied on the global side).  All eight loads of a wavefront and stage share one m0
    // (the start of the Wt part of its region): instruction offsets -4 .. -1 KiB for X and 0 .. 3 KiB for Wt; the lane
    // offsets are biased so that the global side of the instruction offset cancels.  Rows past M or N re-read the last
    // valid row: an output depends on its own row of X and of Wt only, and theirs are never stored.
    // MX: and one 256-byte load of scales per wavefront (4 bytes per lane = a row's four blocks of the stage): wavefronts
    // 0 and 1 bring rows 0 .. 63 and 64 .. 127 of the X tile (with fewer rows in the tile, rows again), 2 and 3 those of
    // the Wt tile.
    constexpr int LOADS_PER_STAGE = A_LOADS8 + B_LOADS8 + (MX ? 1 : 0);
    constexpr int WCOLS = 32 * NT;
    constexpr int STORES_F32 = MT * (32 * WCOLS / 4 / 64);
    constexpr int STORES_BF16 = MT * (32 * WCOLS / 8 / 64);
    static_assert(LOADS_PER_STAGE * (RING8 - 1) + STORES_F32 < 64 && STORES_F32 != STORES_BF16, "vmcnt range");
    constexpr int LANE_BIAS = 4096;
    unsigned aoff[A_LOADS8], boff[B_LOADS8], soff = 0;
    const char *a_ptr = nullptr, *b_ptr = nullptr, *s_ptr = nullptr;      // s_ptr, soff: this wavefront's scale rows (X's or Wt's)
    int issue_item = blockIdx.x;
    int issue_stage = 0;

    auto point_loads_at = [&](int item) __attribute__((always_inline)) {
        const int tile = item % p.tiles, shard = item / p.tiles;
        const int m0 = (tile / p.tiles_n) * BM, n0 = (tile % p.tiles_n) * BN;
        const int64_t kbase = (int64_t)shard * p.k_per_shard;
        a_ptr = uniform_pointer(reinterpret_cast<const char *>(p.X + (int64_t)m0 * p.ldx + kbase));
        b_ptr = uniform_pointer(reinterpret_cast<const char *>(p.Wt + (int64_t)n0 * p.ldw + kbase) - LANE_BIAS);
#pragma unroll
        for (int j = 0; j < A_LOADS8; ++j) {
            const int r = (wave * A_LOADS8 + j) * 8 + (lane >> 3);
            const int c = (lane & 7) ^ ((r >> 1) & 7);
            aoff[j] = (unsigned)(min(r, p.M - 1 - m0) * (int)p.ldx + c * 16) + (unsigned)((A_LOADS8 - j) * 1024);
        }
#pragma unroll
        for (int j = 0; j < B_LOADS8; ++j) {
            const int r = (wave * B_LOADS8 + j) * 8 + (lane >> 3);
            const int c = (lane & 7) ^ ((r >> 1) & 7);
            boff[j] = (unsigned)(min(r, p.N - 1 - n0) * (int)p.ldw + c * 16) + (unsigned)(LANE_BIAS - j * 1024);
        }
        if (MX) {
            const int rs = (wave & 1) * 64 + lane;
            const bool of_x = wave_is_x;               // uniform
            if (p.scales_packed) {                     // a stage's scale bytes of a row block are consecutive: two cache lines per load
                const int64_t stage0 = kbase / BK8;
                const char *xs = reinterpret_cast<const char *>(p.Xs) + ((int64_t)(m0 / BM) * p.stages_total + stage0) * (BM * 4);
                const char *ws = reinterpret_cast<const char *>(p.Ws) + ((int64_t)(n0 / BN) * p.stages_total + stage0) * (BN * 4);
                s_ptr = uniform_pointer(of_x ? xs : ws);
                soff = (unsigned)(4 * (of_x ? rs % BM : rs));
            } else {                                   // straight from the caller's [rows, K / 32] arrays: a cache line per lane
                const char *xs = reinterpret_cast<const char *>(p.Xs + (int64_t)m0 * p.ldxs + kbase / 32);
                const char *ws = reinterpret_cast<const char *>(p.Ws + (int64_t)n0 * p.ldws + kbase / 32);
                s_ptr = uniform_pointer(of_x ? xs : ws);
                soff = of_x ? (unsigned)(min(rs % BM, p.M - 1 - m0) * (int)p.ldxs) : (unsigned)(min(rs, p.N - 1 - n0) * (int)p.ldws);
            }
        }
    };

    const unsigned smem_lds = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const unsigned m0_in_stage = smem_lds + wave_u * REGION8 + A_LOADS8 * 1024;
    const unsigned m0_scales = smem_lds + SCALES_AT + wave_u * 256;         // X rows 0 .. 127, then Wt rows 0 .. 127, four bytes each
    const int s_step = !(MX && p.scales_packed) ? BK8 / 32 : (wave_u < 2 ? BM * 4 : BN * 4);      // scale bytes per stage
    auto issue_part = [&](int slot, auto part_c) __attribute__((always_inline)) {
        constexpr int PART = decltype(part_c)::value;
        if (PART == 0 && __builtin_expect(issue_stage == stages_per_item, 0)) {
            if (issue_item + (int)gridDim.x < p.work) {
                issue_item += gridDim.x;
                point_loads_at(issue_item);
                issue_stage = 0;
            } else {                                   // past the end: load the last stage again (nobody consumes it)
                issue_stage = stages_per_item - 1;
                a_ptr -= BK8;
                b_ptr -= BK8;
                s_ptr -= s_step;
            }
        }
        const unsigned m0v = m0_in_stage + slot * STAGE8;
        if constexpr (PART < A_LOADS8) load_16B_per_lane_to_lds<(PART - A_LOADS8) * 1024, PART == 0>(a_ptr, aoff[PART], m0v);
        load_16B_per_lane_to_lds<PART * 1024, false>(b_ptr, boff[PART], m0v);
        if (PART == B_LOADS8 - 1) {
            if (MX) {
                load_4B_per_lane_to_lds<0, true>(s_ptr, soff, m0_scales + slot * STAGE8);
                s_ptr += s_step;
            }
            ++issue_stage;
            a_ptr += BK8;
            b_ptr += BK8;
        }
    };
    auto issue_next_stage = [&](int slot) {
        issue_part(slot, Int<0>{});
        issue_part(slot, Int<1>{});
        issue_part(slot, Int<2>{});
        issue_part(slot, Int<3>{});
    };

    // ---- LDS fragment addresses (bytes inside a stage) ----
    // Row R of the X tile lies in region R / (8 A_LOADS8) at row R % (8 A_LOADS8); row n of the Wt tile in region n / 32
    // at row n % 32, behind the region's X rows.
    int a_off[MT], b_off[NT];
#pragma unroll
    for (int a = 0; a < MT; ++a) {
        const int R = (wm * MT + a) * 32 + li;
        a_off[a] = (R / (8 * A_LOADS8)) * REGION8 + (R % (8 * A_LOADS8)) * ROW8;
    }
#pragma unroll
    for (int b = 0; b < NT; ++b) b_off[b] = (wn * NT + b) * REGION8 + A_LOADS8 * 1024 + li * ROW8;
    // MX: where the four scale bytes of the lane's rows sit in a slot; block 2 ks + lg is the lane's in K-step ks
    int s_off[MT + NT];
#pragma unroll
    for (int a = 0; a < MT; ++a) s_off[a] = SCALES_AT + ((wm * MT + a) * 32 + li) * 4;
#pragma unroll
    for (int b = 0; b < NT; ++b) s_off[MT + b] = SCALES_AT + 512 + ((wn * NT + b) * 32 + li) * 4;
    const int sw = (li >> 1) & 7;
    // chunk positions of the lane's two 16-byte pieces in K-step ks: chunks 4 ks + lg and 4 ks + 2 + lg (the
    // instruction's first and second 32 positions are the first, and the second, 16 bytes of both halves of the
    // wavefront: see the reference kernel)
    int c_off[KSTEPS8][2];
#pragma unroll
    for (int ks = 0; ks < KSTEPS8; ++ks) {
        c_off[ks][0] = ((4 * ks + lg) ^ sw) << 4;
        c_off[ks][1] = ((4 * ks + 2 + lg) ^ sw) << 4;
    }

    // Fragment registers: one set per K-step of a stage; the reads run one K-step (four MFMAs of 16 passes) ahead.
    i32x4 fr[KSTEPS8][MT + NT][2];
    constexpr int READS_PER_KSTEP = 2 * (MT + NT);
    auto read_frag_op = [&](int r, int set, int slot, int ks) {
        const unsigned char *sb = smem + slot * STAGE8;
        const int f = r >> 1, h = r & 1;
        const int base = f < MT ? a_off[f] : b_off[f - MT];
        fr[set][f][h] = *reinterpret_cast<const i32x4 *>(sb + base + c_off[ks][h]);
    };
    auto read_frags = [&](int set, int slot, int ks) {
#pragma unroll
        for (int r = 0; r < READS_PER_KSTEP; ++r) read_frag_op(r, set, slot, ks);
    };
    auto frag = [&](int set, int f) {
        union { i32x4 h[2]; i32x8 v; } u;
        u.h[0] = fr[set][f][0];
        u.h[1] = fr[set][f][1];
        return u.v;
    };
    // MX: the four scale bytes of each of the lane's rows, fetched once per stage (for the next stage after the last
    // K-step's bytes are taken out).
    unsigned scl[MT + NT];
    auto read_scales = [&](int slot) {
        const unsigned char *sb = smem + slot * STAGE8;
#pragma unroll
        for (int f = 0; f < MT + NT; ++f) scl[f] = *reinterpret_cast<const unsigned *>(sb + s_off[f]);
    };

    Acc<MT, NT> acc, acc2;
    TileStash<LEVELS - 1, MT, NT> stash;

    // Software pipeline over the ring, as in the 16-bit kernel: at the top of stage s wait until this wavefront's loads
    // of stage s+1 have landed, meet the other wavefronts -- stage s+1 is complete, nobody reads the slot of stage s-1
    // any more -- and start the loads of stage s+RING-1 into that slot.
    point_loads_at(issue_item);
#pragma unroll
    for (int i = 0; i < RING8 - 1; ++i) issue_next_stage(i);
    wait_loads_and_barrier<LOADS_PER_STAGE * (RING8 - 2)>();
    read_frags(0, 0, 0);
    if (MX) read_scales(0);

    int cur = 0;
    int stores_in_flight = 0;          // output stores share the counter of the loads (see the 16-bit kernel)

    auto stage = [&](auto first, Acc<MT, NT> &a) {
        constexpr bool FIRST = decltype(first)::value;
        const int nxt = (cur + 1 == RING8) ? 0 : cur + 1;
        constexpr int ALLOW = LOADS_PER_STAGE * (RING8 - 3);
        if (__builtin_expect(stores_in_flight == 0, 1)) {
            wait_loads_and_barrier<ALLOW>();
        } else {
            if (stores_in_flight == STORES_F32) wait_loads_and_barrier<ALLOW + STORES_F32>();
            else if (stores_in_flight == STORES_BF16) wait_loads_and_barrier<ALLOW + STORES_BF16>();
            else wait_loads_and_barrier<0>();
            stores_in_flight = 0;
        }
        const int free_slot = cur == 0 ? RING8 - 1 : cur - 1;
        constexpr int NM = MT * NT;
#pragma unroll
        for (int ks = 0; ks < KSTEPS8; ++ks) {
            const bool ahead_in_stage = ks + 1 < KSTEPS8;
            const int t_set = ahead_in_stage ? ks + 1 : 0;
            const int t_slot = ahead_in_stage ? cur : nxt;
            int sc[MT + NT];
            if (MX) {
#pragma unroll
                for (int f = 0; f < MT + NT; ++f) sc[f] = (int)__builtin_amdgcn_ubfe(scl[f], 16u * ks + 8u * lg, 8u);
                if (ks == KSTEPS8 - 1) read_scales(nxt);       // the next stage's, complete in LDS since this stage's barrier
            }
#pragma unroll
            for (int m = 0; m < NM; ++m) {
                const int i = m / NT, j = m % NT;
                const f32x16 zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
                const int set = (FIRST && ks == 0) ? 0 : ks;
                const f32x16 c_in = (FIRST && ks == 0) ? zero : a.t[i][j];
                if (MX) a.t[i][j] = mfma_32x32x64_8bit_scaled<FMT>(frag(set, i), frag(set, MT + j), c_in, sc[i], sc[MT + j]);
                else a.t[i][j] = mfma_32x32x64_8bit<FMT>(frag(set, i), frag(set, MT + j), c_in);
                // this MFMA's share of the LDS reads of the next K-step and of the loads of the stage being fetched
#pragma unroll
                for (int r = m * READS_PER_KSTEP / NM; r < (m + 1) * READS_PER_KSTEP / NM; ++r)
                    read_frag_op(r, t_set, t_slot, t_set);
                {   // the four parts of the next stage's loads, spread evenly over the stage's KSTEPS8 * NM groups
                    constexpr int G = KSTEPS8 * NM;
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
            static_assert(REGION8 >= 32 * WCOLS * 4, "the output patch must fit a wavefront's region of a slot");
            const int last_slot = cur == 0 ? RING8 - 1 : cur - 1;
            float *patch = reinterpret_cast<float *>(smem + last_slot * STAGE8 + wave * REGION8);
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

template <int WM, int WN, int MT, int NT, int RING8, int FMT, bool MX>
hipError_t launch_tiled_fmt(const GemmArgs &a, const Mxfp4Scales *sc, hipStream_t s) {
    constexpr int BM = 32 * MT * WM, BN = 32 * NT * WN;
    constexpr int STAGE8 = 4 * (BM / 32 + B_LOADS8) * 1024 + (MX ? 1024 : 0);
    static_assert(RING8 * STAGE8 <= 160 * 1024, "LDS of a compute unit");
    Fp8Params p;
    p.X = reinterpret_cast<const uint8_t *>(a.X); p.Wt = reinterpret_cast<const uint8_t *>(a.W);
    p.Xs = MX ? sc->Xs : nullptr; p.Ws = MX ? sc->Ws : nullptr;
    p.ldxs = MX ? sc->ldxs : 0; p.ldws = MX ? sc->ldws : 0;
    p.scales_packed = MX ? sc->packed : 0;
    p.stages_total = a.K / BK8;
    p.partials = a.partials; p.Y = (a.P == 1) ? a.Y : nullptr;
    p.ldx = a.ldx; p.ldw = a.ldw; p.ldy = a.ldy;
    p.M = a.M; p.N = a.N;
    p.y_bf16 = (a.y_dtype != TBIK_F32);
    p.stages_per_superleaf = a.superleaf / BK8;
    p.ns_per_shard = a.ns / a.P;
    p.k_per_shard = (int64_t)a.K / a.P;
    p.tiles_n = (a.N + BN - 1) / BN;
    const int64_t tiles = (int64_t)p.tiles_n * ((a.M + BM - 1) / BM);
    if (tiles * a.P > 0x7fffffff) return hipErrorInvalidValue;
    p.tiles = (int)tiles;
    p.work = (int)(tiles * a.P);
    const int grid_x = p.work < compute_units() ? p.work : compute_units();
    dim3 grid((unsigned)grid_x), block(256);
    const size_t lds = (size_t)RING8 * STAGE8;
    const void *out = p.partials ? (const void *)p.partials : p.Y;
    const int64_t ld_bytes = p.partials ? (int64_t)a.N * 4 : a.ldy * (p.y_bf16 ? 2 : 4);
    p.vector_stores = ((reinterpret_cast<uintptr_t>(out) & 15) == 0) && (ld_bytes % 16 == 0);
    p.stream_stores = a.partials != nullptr && (int64_t)a.P * a.M * a.N * 4 > ((int64_t)192 << 20);
    const int levels = levels_for(p.ns_per_shard);
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 32) dev = 32;
#define TBIK_LAUNCH8(L)                                                                                  \
    case L: {                                                                                            \
        auto k = gemm_fp8_tiled_kernel<L, WM, WN, MT, NT, RING8, FMT, MX>;                               \
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
        TBIK_LAUNCH8(0)
        TBIK_LAUNCH8(1)
        TBIK_LAUNCH8(2)
        TBIK_LAUNCH8(3)
        TBIK_LAUNCH8(4)
        default: return hipErrorInvalidValue;
    }
#undef TBIK_LAUNCH8
    return hipGetLastError();
}

}  // namespace

// rows: 128, 64 or 32 rows per workgroup tile (the caller's choice; the bits do not depend on it)
template <int FMT>
static hipError_t launch_rows(const GemmArgs &a, int rows, hipStream_t s) {
    if (rows == 32) return launch_tiled_fmt<1, 4, 1, 1, 8, FMT, false>(a, nullptr, s);   // 8 x 20 KiB slots: deep prefetch for weight streaming
    if (rows == 64) return launch_tiled_fmt<1, 4, 2, 1, 6, FMT, false>(a, nullptr, s);   // 6 x 24 KiB
    return launch_tiled_fmt<2, 2, 2, 2, 5, FMT, false>(a, nullptr, s);                   // 5 x 32 KiB
}
// With block scales a slot is 1 KiB larger: one slot fewer where the ring filled LDS.
template <int FMT>
static hipError_t launch_rows_mx(const GemmArgs &a, const Mxfp4Scales &sc, int rows, hipStream_t s) {
    if (rows == 32) return launch_tiled_fmt<1, 4, 1, 1, 7, FMT, true>(a, &sc, s);        // 7 x 21 KiB
    if (rows == 64) return launch_tiled_fmt<1, 4, 2, 1, 6, FMT, true>(a, &sc, s);        // 6 x 25 KiB
    return launch_tiled_fmt<2, 2, 2, 2, 4, FMT, true>(a, &sc, s);                        // 4 x 33 KiB
}

bool gemm_fp8_tiled_supports(const GemmArgs &a) {
    if (a.superleaf % BK8 != 0) return false;
    if (levels_for(a.ns / a.P) > 4) return false;
    if (a.ldx >= (1 << 22) || a.ldw >= (1 << 22)) return false;     // per-lane byte offsets of a tile stay below 2^31
    return true;
}

hipError_t launch_gemm_fp8_tiled(const GemmArgs &a, int rows, hipStream_t s) {
    if (a.M <= 0 || a.N <= 0) return hipSuccess;
    if (!gemm_fp8_tiled_supports(a) || (rows != 32 && rows != 64 && rows != 128)) return hipErrorInvalidValue;
    return a.x_dtype == TBIK_FP8_E5M2 ? launch_rows<1>(a, rows, s) : launch_rows<0>(a, rows, s);
}

hipError_t launch_gemm_fp8_reference(const GemmArgs &a, hipStream_t s) {
    if (a.M <= 0 || a.N <= 0) return hipSuccess;
    if (a.superleaf % 64 != 0) return hipErrorInvalidValue;
    dim3 grid((a.N + 31) / 32, (a.M + 31) / 32, a.P);
    if (grid.y > 65535u || grid.z > 65535u) return hipErrorInvalidValue;
    void *Y = (a.P == 1) ? a.Y : nullptr;
    auto kernel = (a.x_dtype == TBIK_FP8_E5M2) ? gemm_fp8_reference_kernel<1, false> : gemm_fp8_reference_kernel<0, false>;
    hipLaunchKernelGGL(kernel, grid, dim3(64), 0, s, reinterpret_cast<const uint8_t *>(a.X), a.ldx,
                       reinterpret_cast<const uint8_t *>(a.W), a.ldw, nullptr, 0, nullptr, 0, a.partials, Y, a.ldy, a.y_dtype,
                       a.M, a.N, a.superleaf, a.ns / a.P);
    return hipGetLastError();
}

// MXFP8: x_dtype names the element format (TBIK_FP8_E4M3 or TBIK_FP8_E5M2); sc carries the E8M0 scales.
bool gemm_mxfp8_tiled_supports(const GemmArgs &a, const Mxfp4Scales &sc) {
    if (!gemm_fp8_tiled_supports(a)) return false;
    auto a4 = [](const void *q) { return (reinterpret_cast<uintptr_t>(q) & 3) == 0; };
    if (!a4(sc.Xs) || !a4(sc.Ws) || sc.ldxs % 4 != 0 || sc.ldws % 4 != 0) return false;   // a row's four scale bytes per stage: one aligned dword
    if (sc.ldxs >= (1 << 24) || sc.ldws >= (1 << 24)) return false;                       // per-lane byte offsets of a tile's scales stay below 2^31
    return true;
}

size_t mxfp8_retiled_scales_bytes(int M, int N, int K) { return mx_retiled_scales_bytes<1>(M, N, K / BK8); }

// packed_ws: nullptr, or mxfp8_retiled_scales_bytes(M, N, K) bytes (4-byte aligned) into which the scales are re-tiled
// first (one short launch), after which every scale load of the GEMM touches two cache lines instead of 64.
hipError_t launch_gemm_mxfp8_tiled(const GemmArgs &a, const Mxfp4Scales &sc, int rows, void *packed_ws, hipStream_t s) {
    if (a.M <= 0 || a.N <= 0) return hipSuccess;
    if (!gemm_mxfp8_tiled_supports(a, sc) || (rows != 32 && rows != 64 && rows != 128)) return hipErrorInvalidValue;
    Mxfp4Scales use = sc;
    if (packed_ws) {
        hipError_t e = launch_mx_scales_retile<1>(sc.Xs, sc.ldxs, a.M, rows, sc.Ws, sc.ldws, a.N, a.K / BK8, packed_ws, &use.Xs, &use.Ws, s);
        if (e != hipSuccess) return e;
        use.packed = 1;
    }
    return a.x_dtype == TBIK_FP8_E5M2 ? launch_rows_mx<1>(a, use, rows, s) : launch_rows_mx<0>(a, use, rows, s);
}

hipError_t launch_gemm_mxfp8_reference(const GemmArgs &a, const Mxfp4Scales &sc, hipStream_t s) {
    if (a.M <= 0 || a.N <= 0) return hipSuccess;
    if (a.superleaf % 64 != 0) return hipErrorInvalidValue;
    dim3 grid((a.N + 31) / 32, (a.M + 31) / 32, a.P);
    if (grid.y > 65535u || grid.z > 65535u) return hipErrorInvalidValue;
    void *Y = (a.P == 1) ? a.Y : nullptr;
    auto kernel = (a.x_dtype == TBIK_FP8_E5M2) ? gemm_fp8_reference_kernel<1, true> : gemm_fp8_reference_kernel<0, true>;
    hipLaunchKernelGGL(kernel, grid, dim3(64), 0, s, reinterpret_cast<const uint8_t *>(a.X), a.ldx,
                       reinterpret_cast<const uint8_t *>(a.W), a.ldw, sc.Xs, sc.ldxs, sc.Ws, sc.ldws, a.partials, Y, a.ldy,
                       a.y_dtype, a.M, a.N, a.superleaf, a.ns / a.P);
    return hipGetLastError();
}

}  // namespace tbik
