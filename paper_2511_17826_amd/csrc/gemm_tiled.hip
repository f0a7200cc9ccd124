// Tiled Tree-Based MatMul kernels (App. D.1, Alg. 1) for gfx950.
//
// A workgroup of 4 wavefronts owns one BM x 128 output tile of one K-shard and walks the shard's
// superleaves in ascending k.  Per superleaf each wavefront chains v_mfma_f32_32x32x16_bf16 over
// ascending groups of 16 k into accumulators that start at +0 (the same opcode and k -> (step,
// slot) map as the reference kernel, which is what makes all variants bit-identical); when a
// superleaf ends, the carry-over step folds the accumulators into the stash of waiting subtrees,
// which lives in registers (one wavefront per SIMD, up to 512 VGPR+AGPR per lane).
//
// Operands are staged through LDS in K-steps of 64 (a ring of stage slots filled by direct global->LDS
// loads), both in their global orientation.  A stage slot is cut into four regions, one per wavefront
// (the wavefront that loads it): [BM/4 rows of the X tile | 16 rows of the W tile].
//   X rows are 128 B; the 16-byte chunk c of row r sits at position c ^ ((r>>1)&7), so the 16 rows
//                    of a fragment read (ds_read_b128) hit all 64 banks once;
//   W rows are 256 B; chunk c of row k sits at position c ^ (4*(k&3)); the MFMA's B operand (8
//                    consecutive k of one column per lane) is fetched with the transposing LDS read
//                    ds_read_b64_tr_b16, whose 16-lane groups read 4 rows x 16 columns: with the
//                    swizzle the 4 rows fall into different banks.
#include <atomic>
#include <type_traits>

#include "tbik_device.hpp"
#include "tbik_internal.hpp"
#include "tree_walk.hpp"

namespace tbik {

template <int V>
using Int = std::integral_constant<int, V>;

constexpr int BK = 64;                 // K-elements per LDS stage
constexpr int BN_TILE = 128;           // columns per workgroup tile
#ifndef TBIK_FRAG_AHEAD
#define TBIK_FRAG_AHEAD 2
#endif
constexpr int FRAG_AHEAD = TBIK_FRAG_AHEAD;   // K-steps between an LDS fragment read and its MFMAs (1..3)
constexpr int A_ROW = BK * 2;          // bytes per LDS row of the X tile
constexpr int B_ROW = BN_TILE * 2;     // bytes per LDS row of the W tile

typedef short v4i16 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// Waits until at most N of this wavefront's vector-memory loads are outstanding, then joins the workgroup
// barrier.  Deliberately not __syncthreads(): its fence would wait for all loads.
template <int N>
__device__ __forceinline__ void wait_loads_and_barrier() {
    static_assert(N >= 0 && N < 64, "vmcnt range");
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(N) : "memory");
}

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
    int tiles_n;                // column tiles
    int tiles;                  // output tiles per shard
    int work;                   // tiles * shards
    int vector_stores;          // outputs are 16-byte aligned with 16-byte aligned rows
    int stream_stores;          // fp32 outputs bypass the caches (partials too large to stay there until they are combined)
    int swiglu;                 // W is [gate | up] ([K, 2 I], N = 2 I); Y is act [M, I] = SiLU(gate) * up, 16-bit
};

// ---------------------------------------------------------------------------------------------
// BM = 32*MT*WM rows, BN = 32*NT*WN columns, WM*WN = 4 wavefronts.
// Persistent workgroups: workgroup g handles work items g, g + gridDim.x, ... (item = tile + tiles * shard).
// The global->LDS load stream runs ahead of the MFMA stream across item boundaries, so the first stages
// of the next tile are already in flight while the current tile is finished and stored.
// RING: LDS stage slots; RING - 3 stages of loads are in flight at a stage's entry, one more is issued during it.
// F16: the operands (and a 16-bit output) are IEEE binary16 instead of bf16; only the MFMA opcode and the output
// conversion differ.
template <int LEVELS, int WM, int WN, int MT, int NT, int RING, bool F16>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
void gemm_tiled_kernel(const TiledParams p) {
    constexpr int BM = 32 * MT * WM, BN = 32 * NT * WN;
    static_assert(BN == BN_TILE && WM * WN == 4, "tile shape");
    constexpr int A_LOADS = BM / 32;          // 1 KiB loads per wavefront and stage: BM rows / 8 rows / 4 wavefronts
    constexpr int B_LOADS = BK / 16;          // 64 rows / 4 rows / 4 wavefronts
    static_assert(B_LOADS == 4 && A_LOADS <= 4, "one W load and at most one X load per K-step");
    constexpr int REGION_BYTES = (A_LOADS + B_LOADS) * 1024;   // stage layout: one region per loading wavefront,
    constexpr int STAGE_BYTES = 4 * REGION_BYTES;               // [8*A_LOADS rows of X | 16 rows of W]

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int li = lane & 31, lg = lane >> 5;
    const int stages_per_item = p.ns_per_shard * p.stages_per_superleaf;

    // ---- global -> LDS, without passing through registers (global_load_lds_dwordx4) ----
    // One such instruction moves 64 x 16 bytes: lane i's chunk lands at LDS base + 16*i, so a
    // wavefront fills 1 KiB of consecutive LDS = 8 rows of the X tile or 4 rows of the W tile, and
    // the swizzle is applied on the global side (which chunk a lane fetches).  Rows past M and
    // columns past N are never stored, and an output element depends only on its own row of X and
    // column of W, so out-of-range lanes simply re-read the last valid row / column block.
    // All loads of a wavefront and stage share one m0 (the start of the W part of its region) and differ in
    // their instruction offsets, -A_LOADS KiB .. -1 KiB for X and 0 .. 3 KiB for W; the lane offsets are biased
    // so that the global side of the instruction offset cancels.
    constexpr int LOADS_PER_STAGE = A_LOADS + B_LOADS;
    constexpr int WCOLS = 32 * NT;                         // columns of a wavefront's tile
    constexpr int STORES_F32 = MT * (32 * WCOLS / 4 / 64);   // 16-byte store instructions per wavefront and tile
    constexpr int STORES_BF16 = MT * (32 * WCOLS / 8 / 64);
    constexpr int STORES_ACT = NT == 2 ? MT * 2 : -2;         // gated activation (NT == 2 only): 32 x 32 values of 16 bits per block
    static_assert(LOADS_PER_STAGE * (RING - 3) + STORES_F32 < 64 && STORES_F32 != STORES_BF16 && STORES_BF16 != STORES_ACT,
                  "vmcnt range");
    constexpr int LANE_BIAS = 4096;            // keeps every biased lane offset non-negative
    unsigned aoff[A_LOADS], boff[B_LOADS];     // per-lane byte offsets from the uniform stage pointers
    const char *a_ptr = nullptr, *b_ptr = nullptr;   // stage pointers of the stage to load next (b_ptr: minus LANE_BIAS)
    const int64_t b_stage_bytes = (int64_t)BK * p.ldw * 2;
    int issue_item = blockIdx.x;               // work item whose stages are being loaded
    int issue_stage = 0;                       // next stage of that item to load

    auto point_loads_at = [&](int item) __attribute__((always_inline)) {
        const int tile = item % p.tiles, shard = item / p.tiles;
        const int m0 = (tile / p.tiles_n) * BM, n0 = (tile % p.tiles_n) * BN;
        const int64_t kbase = (int64_t)shard * p.k_per_shard;
        a_ptr = uniform_pointer(reinterpret_cast<const char *>(p.X + (int64_t)m0 * p.ldx + kbase));
        // Gated activation: the 128 columns of a tile are, per wavefront column, 32 gate channels and the same 32 up
        // channels (a lane then holds gate and up of one channel in its two column blocks), taken from the two halves
        // of W; the tile starts at channel n0 / 2.
        b_ptr = uniform_pointer(reinterpret_cast<const char *>(p.W + kbase * p.ldw + (p.swiglu ? n0 / 2 : n0)) - LANE_BIAS);
#pragma unroll
        for (int j = 0; j < A_LOADS; ++j) {
            const int r = (wave * A_LOADS + j) * 8 + (lane >> 3);
            const int c = (lane & 7) ^ ((r >> 1) & 7);
            aoff[j] = (unsigned)(min(r, p.M - 1 - m0) * (int)p.ldx + c * 8) * 2u + (unsigned)((A_LOADS - j) * 1024);
        }
#pragma unroll
        for (int j = 0; j < B_LOADS; ++j) {
            const int kk = (wave * B_LOADS + j) * 4 + (lane >> 4);
            const int c = (lane & 15) ^ ((lane >> 4) << 2);
            const int col = p.swiglu ? ((c >> 2) & 1) * (p.N / 2) + (c >> 3) * 32 + (c & 3) * 8 : min(c * 8, p.N - 8 - n0);
            boff[j] = (unsigned)(kk * (int)p.ldw + col) * 2u + (unsigned)(LANE_BIAS - j * 1024);
        }
    };

    const unsigned smem_lds = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const unsigned m0_in_stage = smem_lds + wave_u * REGION_BYTES + A_LOADS * 1024;
    // Loads the next stage of the stream into ring slot `slot`, in BK/16 parts that the caller spreads over the
    // K-steps of the stage it is multiplying (part 0 first; a burst of loads would keep the LDS write port busy
    // while fragment reads wait).  Past the last stage of the last item the last stage is simply loaded again
    // (nobody consumes it).
    auto issue_part = [&](int slot, auto part_c) __attribute__((always_inline)) {
        constexpr int PART = decltype(part_c)::value;
        if (PART == 0 && __builtin_expect(issue_stage == stages_per_item, 0)) {
            if (issue_item + (int)gridDim.x < p.work) {
                issue_item += gridDim.x;
                point_loads_at(issue_item);
                issue_stage = 0;
            } else {
                issue_stage = stages_per_item - 1;
                a_ptr -= BK * 2;
                b_ptr -= b_stage_bytes;
            }
        }
        const unsigned m0v = m0_in_stage + slot * STAGE_BYTES;
        if constexpr (PART < A_LOADS) load_16B_per_lane_to_lds<(PART - A_LOADS) * 1024, PART == 0>(a_ptr, aoff[PART], m0v);
        load_16B_per_lane_to_lds<PART * 1024, (PART == 0 && A_LOADS == 0)>(b_ptr, boff[PART], m0v);
        if (PART == BK / 16 - 1) {
            ++issue_stage;
            a_ptr += BK * 2;
            b_ptr += b_stage_bytes;
        }
    };
    auto issue_next_stage = [&](int slot) {
        issue_part(slot, Int<0>{});
        issue_part(slot, Int<1>{});
        issue_part(slot, Int<2>{});
        issue_part(slot, Int<3>{});
    };

    // ---- LDS fragment addresses (bytes inside a stage) ----
    // X fragment a: row R = wm*MT*32 + a*32 + li lies in region R / (8*A_LOADS); chunk 2*ks + lg of it sits at
    // position (2*ks) ^ (lg ^ ((li>>1)&7)).
    int a_off[MT];
#pragma unroll
    for (int a = 0; a < MT; ++a) {
        const int R = (wm * MT + a) * 32 + li;
        a_off[a] = (R / (8 * A_LOADS)) * REGION_BYTES + (R % (8 * A_LOADS)) * A_ROW;
    }
    const int a_sw = (lg ^ ((li >> 1) & 7)) << 4;
    // W fragment b, half h, K-step ks: region ks holds rows 16*ks .. 16*ks+15; a 16-lane group reads rows
    // 8*lg + 4*h + (0..3) of it, 16 columns.
    const int l16 = lane & 15, e = l16 >> 2;
    int b_off[NT];
#pragma unroll
    for (int b = 0; b < NT; ++b) {
        const int col = (wn * NT + b) * 32 + ((lane >> 4) & 1) * 16 + (l16 & 3) * 4;
        b_off[b] = A_LOADS * 1024 + (lg * 8 + e) * B_ROW + ((((col >> 3) ^ (e << 2))) << 4) + ((col >> 2) & 1) * 8;
    }

    // Fragment registers: the LDS reads run FRAG_AHEAD K-steps ahead of the MFMAs that consume them (into the
    // next stage's slot near the end of a stage: that slot is complete since the barrier at the top of this stage).
    constexpr int KSTEPS = BK / 16;
    bf16x8 af[KSTEPS][MT];                        // one register set per K-step of a stage
    v4i16 bh[KSTEPS][NT][2];                      // W fragments arrive as two transposed 8-byte halves
    constexpr int READS_PER_KSTEP = MT + 2 * NT;  // LDS read instructions per K-step
    // LDS read number r of a K-step: the X fragments first, then the halves of the W fragments.
    auto read_frag_op = [&](int r, int set, int slot, int ks) {
        const unsigned char *sb = smem + slot * STAGE_BYTES;
        if (r < MT) {
            af[set][r] = *reinterpret_cast<const bf16x8 *>(sb + a_off[r] + (a_sw ^ (ks << 5)));
        } else {
            const int b = (r - MT) >> 1, h = (r - MT) & 1;
            bh[set][b][h] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (__attribute__((address_space(3))) v4i16 *)(sb + b_off[b] + ks * REGION_BYTES + h * 4 * B_ROW));
        }
    };
    auto read_frags = [&](int set, int slot, int ks) {
#pragma unroll
        for (int r = 0; r < READS_PER_KSTEP; ++r) read_frag_op(r, set, slot, ks);
    };
    auto w_frag = [&](int set, int b) {
        union { v4i16 h[2]; bf16x8 v; } u;
        u.h[0] = bh[set][b][0];
        u.h[1] = bh[set][b][1];
        return u.v;
    };

    Acc<MT, NT> acc, acc2;
    TileStash<LEVELS - 1, MT, NT> stash;

    // Software pipeline over a ring of RING LDS stage slots.  At the top of stage s: wait until this
    // wavefront's loads of stage s+1 have landed (those of later stages may still be in flight), meet the
    // other wavefronts at a barrier -- now stage s+1 is complete in LDS and nobody reads the slot of
    // stage s-1 any more -- and start the loads of stage s+RING-1 into that slot.  The barrier is written
    // in assembly on purpose: a fence would make the compiler drain every outstanding load.
    point_loads_at(issue_item);
#pragma unroll
    for (int i = 0; i < RING - 1; ++i) issue_next_stage(i);
    wait_loads_and_barrier<LOADS_PER_STAGE * (RING - 2)>();      // stage 0 landed everywhere
#pragma unroll
    for (int i = 0; i < FRAG_AHEAD; ++i) read_frags(i, 0, i);

    int cur = 0;             // ring slot of the stage being multiplied
    // Output stores share the load counter (vmcnt counts loads and stores in issue order).  -1: an unknown number of
    // stores was issued (edge tile): wait for everything once.  n >= 0: exactly n store instructions follow the loads
    // that are in flight, so they are simply added to the allowance of the next wait.
    int stores_in_flight = 0;

    // One LDS stage of MFMA chains into `a`.  FIRST: the accumulators start at +0 (zero C operand).
    auto stage = [&](auto first, Acc<MT, NT> &a) {
        constexpr bool FIRST = decltype(first)::value;
        const int nxt = (cur + 1 == RING) ? 0 : cur + 1;
        constexpr int ALLOW = LOADS_PER_STAGE * (RING - 3);  // loads of stage s+2.. may still be in flight
        if (__builtin_expect(stores_in_flight == 0, 1)) {
            wait_loads_and_barrier<ALLOW>();                         // stage s+1 landed; the slot of stage s-1 is free
        } else {                                                     // first stage after an epilogue
            if (stores_in_flight == STORES_F32) wait_loads_and_barrier<ALLOW + STORES_F32>();
            else if (stores_in_flight == STORES_BF16) wait_loads_and_barrier<ALLOW + STORES_BF16>();
            else if (stores_in_flight == STORES_ACT) wait_loads_and_barrier<ALLOW + STORES_ACT>();
            else wait_loads_and_barrier<0>();
            stores_in_flight = 0;
        }
        const int free_slot = cur == 0 ? RING - 1 : cur - 1;  // the slot of stage s-1
        // A wavefront issues in order, one instruction per four cycles at best, and it is alone on its SIMD: every
        // non-MFMA instruction that is not placed between two MFMAs leaves the matrix pipe idle.  So the K-step is
        // written as one group per MFMA -- the MFMA, then its share of the LDS reads (FRAG_AHEAD steps ahead) and of
        // the global->LDS loads of the stage being fetched -- and the scheduler may not move anything across groups.
        constexpr int NM = MT * NT;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
            const bool ahead_in_stage = ks + FRAG_AHEAD < KSTEPS;
            const int t_set = ahead_in_stage ? ks + FRAG_AHEAD : ks + FRAG_AHEAD - KSTEPS;
            const int t_slot = ahead_in_stage ? cur : nxt;
#pragma unroll
            for (int m = 0; m < NM; ++m) {
                const int i = m / NT, j = m % NT;
                if (FIRST && ks == 0) {
                    const f32x16 zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
                    a.t[i][j] = mfma_32x32x16<F16>(af[0][i], w_frag(0, j), zero);
                } else {
                    a.t[i][j] = mfma_32x32x16<F16>(af[ks][i], w_frag(ks, j), a.t[i][j]);
                }
#pragma unroll
                for (int r = m * READS_PER_KSTEP / NM; r < (m + 1) * READS_PER_KSTEP / NM; ++r)
                    read_frag_op(r, t_set, t_slot, t_set);
                if (m == 1 % NM) {
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

    // One superleaf: stages_per_superleaf stages chained in ascending k.
    auto superleaf = [&](Acc<MT, NT> &a) {
        stage(std::true_type{}, a);
#pragma nounroll
        for (int q = 1; q < p.stages_per_superleaf; ++q) stage(std::false_type{}, a);
    };

    for (int item = blockIdx.x; item < p.work; item += gridDim.x) {
        SubtreeWalker<LEVELS>::run(superleaf, acc, acc2, stash);

        // ---- acc holds T(superleaves of this shard) for this tile: store it ----
        const int tile = item % p.tiles, shard = item / p.tiles;
        const int m0 = (tile / p.tiles_n) * BM, n0 = (tile % p.tiles_n) * BN;
        float *part = p.partials ? p.partials + (int64_t)shard * p.M * p.N : nullptr;
        const bool interior = (m0 + BM <= p.M) && (n0 + BN <= p.N);
        if (interior && p.vector_stores) {
            // Full tile, 16-byte aligned rows: each wavefront turns its 32 x (32*NT) blocks around in its private LDS
            // patch, so that a lane holds 4 (fp32) or 8 (bf16) consecutive columns and stores 16 bytes.  The number of
            // store instructions is fixed (no lane masks, no branches), which the load accounting above relies on.
            // The patch is the wavefront's own region of the stage slot that was multiplied last: nothing is loaded
            // into that slot before the next stage's barrier, but the other wavefronts may still be reading it.
            static_assert(REGION_BYTES >= 32 * WCOLS * 4, "the output patch must fit a wavefront's region of a slot");
            const int last_slot = cur == 0 ? RING - 1 : cur - 1;
            float *patch = reinterpret_cast<float *>(smem + last_slot * STAGE_BYTES + wave * REGION_BYTES);
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
            const bool to_bf16 = (part == nullptr) && p.y_bf16;
            // All patch reads of a 32-row block are issued before its first store (one LDS latency per block, not one
            // per store), and a store's address is a wave-uniform base plus a 32-bit lane offset.
            const int wm_u = wave_u / WN, wn_u = wave_u % WN;          // the same numbers as wm, wn, known to be uniform
            const int col0 = n0 + wn_u * WCOLS;
            if (NT == 2 && p.swiglu) {
                // Gate and up of a channel sit in the lane's two column blocks: both are rounded as the 16-bit outputs
                // of two separate GEMMs would be, the activation is applied, and the 32 x 32 block goes through the patch.
                constexpr int CPR = 4, RPI = 16, N_IT = 2;
                const int lrow = lane / CPR, lc = lane % CPR;
                const float *rd = patch + lrow * 32 + lc * 8;
                const unsigned lane_off = (unsigned)(lrow * (int)p.ldy + lc * 8) * 2u;
                const int64_t it_step = (int64_t)RPI * p.ldy * 2;
#pragma unroll
                for (int a = 0; a < MT; ++a) {
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        patch[(8 * (r >> 2) + 4 * lg + (r & 3)) * 32 + li] =
                            silu_mul(through_16_bits<F16>(acc.t[a][0][r]), through_16_bits<F16>(acc.t[a][NT - 1][r]));
                    f32x4 lo[N_IT], hi[N_IT];
#pragma unroll
                    for (int it = 0; it < N_IT; ++it) {
                        lo[it] = *reinterpret_cast<const f32x4 *>(rd + it * RPI * 32);
                        hi[it] = *reinterpret_cast<const f32x4 *>(rd + it * RPI * 32 + 4);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                    char *base = reinterpret_cast<char *>(reinterpret_cast<uint16_t *>(p.Y) +
                                                          (int64_t)(m0 + (wm_u * MT + a) * 32) * p.ldy + n0 / 2 + wn_u * 32);
#pragma unroll
                    for (int it = 0; it < N_IT; ++it) {
                        u32x4 o;
                        o[0] = pack_16x2<F16>(lo[it][0], lo[it][1]);
                        o[1] = pack_16x2<F16>(lo[it][2], lo[it][3]);
                        o[2] = pack_16x2<F16>(hi[it][0], hi[it][1]);
                        o[3] = pack_16x2<F16>(hi[it][2], hi[it][3]);
                        *reinterpret_cast<u32x4 *>(base + it * it_step + lane_off) = o;
                    }
                }
            } else if (to_bf16) {
                constexpr int CPR = WCOLS / 8, RPI = 64 / CPR, N_IT = 32 / RPI;      // 16-byte chunks per row, rows per store
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
                        o[0] = pack_16x2<F16>(lo[it][0], lo[it][1]);
                        o[1] = pack_16x2<F16>(lo[it][2], lo[it][3]);
                        o[2] = pack_16x2<F16>(hi[it][0], hi[it][1]);
                        o[3] = pack_16x2<F16>(hi[it][2], hi[it][3]);
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
                    if (p.stream_stores) {                 // uniform; the same number of store instructions either way
                        // (in assembly: written as two branches of ordinary code the compiler merges them and drops the hint)
#pragma unroll
                        for (int it = 0; it < N_IT; ++it)
                            asm volatile("global_store_dwordx4 %0, %1, off nt" ::"v"(base + it * it_step + lane_off), "v"(v[it]) : "memory");
                    } else {
#pragma unroll
                        for (int it = 0; it < N_IT; ++it) *reinterpret_cast<f32x4 *>(base + it * it_step + lane_off) = v[it];
                    }
                }
            }
            stores_in_flight = (NT == 2 && p.swiglu) ? STORES_ACT : to_bf16 ? STORES_BF16 : STORES_F32;
        } else if (NT == 2 && p.swiglu) {                    // ragged last row tile
            const int col = n0 / 2 + wn * 32 + li;
#pragma unroll
            for (int a = 0; a < MT; ++a) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = m0 + (wm * MT + a) * 32 + 8 * (r >> 2) + 4 * lg + (r & 3);
                    if (row >= p.M) continue;
                    const float v = silu_mul(through_16_bits<F16>(acc.t[a][0][r]), through_16_bits<F16>(acc.t[a][NT - 1][r]));
                    reinterpret_cast<uint16_t *>(p.Y)[(int64_t)row * p.ldy + col] = (uint16_t)f32_to_16_bits<F16>(v);
                }
            }
            stores_in_flight = -1;
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
                            if (p.y_bf16) reinterpret_cast<uint16_t *>(p.Y)[(int64_t)row * p.ldy + col] = (uint16_t)f32_to_16_bits<F16>(v);
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

// ---------------------------------------------------------------------------------------------

static int levels_for(int ns_per_shard) {
    int l = 0;
    while ((1 << l) < ns_per_shard) ++l;
    return l;
}

bool gemm_tiled_supports(const GemmArgs &a, int variant) {
    if (variant != VARIANT_T128 && variant != VARIANT_T32 && variant != VARIANT_T64) return false;
    if (a.N % 8 != 0 || a.superleaf % BK != 0) return false;
    if (levels_for(a.ns / a.P) > 4) return false;
    if (a.ldx >= (1 << 22) || a.ldw >= (1 << 22)) return false;   // per-lane byte offsets of a tile stay below 2^31
    if (a.swiglu && (variant != VARIANT_T128 || a.P != 1 || a.partials || a.N % 128 != 0 || a.y_dtype != a.x_dtype)) return false;
    return true;
}

static int compute_units() {
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

template <int WM, int WN, int MT, int NT, int RING, bool F16>
static hipError_t launch_shape(const GemmArgs &a, hipStream_t s) {
    constexpr int BM = 32 * MT * WM, BN = 32 * NT * WN;
    TiledParams p;
    p.X = a.X; p.W = a.W; p.partials = a.partials; p.Y = (a.P == 1) ? a.Y : nullptr;
    p.ldx = a.ldx; p.ldw = a.ldw; p.ldy = a.ldy;
    p.M = a.M; p.N = a.N;
    p.swiglu = (NT == 2) ? a.swiglu : 0;
    p.y_bf16 = (a.y_dtype != TBIK_F32);                  // 16-bit output, in the operands' format
    p.stages_per_superleaf = a.superleaf / BK;
    p.ns_per_shard = a.ns / a.P;
    p.k_per_shard = (int64_t)a.K / a.P;
    p.tiles_n = (a.N + BN - 1) / BN;
    const int64_t tiles = (int64_t)p.tiles_n * ((a.M + BM - 1) / BM);
    if (tiles * a.P > 0x7fffffff) return hipErrorInvalidValue;
    p.tiles = (int)tiles;
    p.work = (int)(tiles * a.P);
    const int grid_x = p.work < compute_units() ? p.work : compute_units();
    dim3 grid((unsigned)grid_x), block(256);
    const size_t lds = RING * ((size_t)BM * A_ROW + (size_t)BK * B_ROW);   // the output patch reuses a stage slot
    {
        const void *out = p.partials ? (const void *)p.partials : p.Y;
        const int64_t ld_bytes = p.partials ? (int64_t)a.N * 4 : a.ldy * (p.y_bf16 ? 2 : 4);   // act: 16-byte chunks of 8 channels
        p.vector_stores = ((reinterpret_cast<uintptr_t>(out) & 15) == 0) && (ld_bytes % 16 == 0);
        // Partials of many shards exceed the 256 MiB memory-side cache before the combine reads them: written around
        // the caches they do not evict the operands (P = 8 at 4096^2: 257 -> 170 us).  Fewer planes stay cached for
        // their reader, so those keep ordinary stores.
        p.stream_stores = a.partials != nullptr && (int64_t)a.P * a.M * a.N * 4 > ((int64_t)192 << 20);
    }
    const int levels = levels_for(p.ns_per_shard);
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 32) dev = 32;   // 32: not remembered, set every time
#define TBIK_LAUNCH(L)                                                                                   \
    case L: {                                                                                            \
        auto k = gemm_tiled_kernel<L, WM, WN, MT, NT, RING, F16>;                                            \
        static std::atomic<unsigned> lds_allowed{0};   /* bit d: the attribute is set on device d */     \
        if (dev >= 32 || !((lds_allowed.load(std::memory_order_relaxed) >> dev) & 1u)) {                 \
            hipError_t e = hipFuncSetAttribute((const void *)k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); \
            if (e != hipSuccess) return e;                                                               \
            if (dev < 32) lds_allowed.fetch_or(1u << dev, std::memory_order_relaxed);                    \
        }                                                                                                \
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
    const bool f16 = (a.x_dtype == TBIK_F16);
    // 128 x 128, wave tile 64 x 64, 5 x 32 KiB stage slots = all of LDS
    if (variant == VARIANT_T128) return f16 ? launch_shape<2, 2, 2, 2, 5, true>(a, s) : launch_shape<2, 2, 2, 2, 5, false>(a, s);
    // 64 x 128, wave tile 64 x 32, 6 x 24 KiB: batches of 33..64 rows without the idle upper half of a 128-row tile
    if (variant == VARIANT_T64) return f16 ? launch_shape<1, 4, 2, 1, 6, true>(a, s) : launch_shape<1, 4, 2, 1, 6, false>(a, s);
    // 32 x 128, wave tile 32 x 32, 6 x 20 KiB: deep prefetch for weight streaming
    return f16 ? launch_shape<1, 4, 1, 1, 6, true>(a, s) : launch_shape<1, 4, 1, 1, 6, false>(a, s);
}

}  // namespace tbik
