// Tree-Based MatMul on fp32 operands (the FP32 row of the paper's kernel table; App. D.1, Alg. 1) for gfx950.
//
// The product of two fp32 numbers is not an fp32 number, so a leaf's accumulation needs a definition: one fused
// multiply-add per k, ascending k, from +0.  That is what v_mfma_f32_32x32x2_f32 computes: its two k-slots (lanes
// 0..31 hold k, lanes 32..63 hold k + 1) are applied as D = fma(a1, b1, fma(a0, b0, C)), each a single rounding.
// Chained over ascending pairs of k this is the sequential chain, whatever the tile shape, so the reference kernel
// (operands straight from global memory) and the tiled kernel give the same bits, and so does any CPU with fmaf.
// Above the superleaves the tree is the one of the 16-bit kernels (tree_walk.hpp).
#include <atomic>
#include <type_traits>

#include "tbik_device.hpp"
#include "tbik_internal.hpp"
#include "tree_walk.hpp"

namespace tbik {

__device__ __forceinline__ f32x16 mfma_f32(float a, float b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

// ---------------------------------------------------------------------------------------------------------------
// Reference: one wavefront per 32x32 output tile and shard, no LDS.
// ---------------------------------------------------------------------------------------------------------------
constexpr int F32_REF_MAX_LEVELS = 28;

__global__ __launch_bounds__(64) void gemm_f32_reference_kernel(
        const float *__restrict__ X, int64_t ldx, const float *__restrict__ W, int64_t ldw,
        float *__restrict__ partials, float *__restrict__ Y, int64_t ldy,
        int M, int N, int superleaf, int ns_per_shard) {
    const int lane = threadIdx.x;
    const int i = lane & 31, g = lane >> 5;
    const int m0 = blockIdx.y * 32, n0 = blockIdx.x * 32;
    const int p = blockIdx.z;
    const int64_t kbase = (int64_t)p * ns_per_shard * superleaf;
    const bool row_ok = (m0 + i) < M, col_ok = (n0 + i) < N;
    const float *xrow = X + (int64_t)(m0 + i) * ldx;
    const float *wcol = W + (n0 + i);

    float stash[F32_REF_MAX_LEVELS][16];
    f32x16 acc;
    for (int j = 0; j < ns_per_shard; ++j) {
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
        const int64_t k0 = kbase + (int64_t)j * superleaf;
        for (int kk = 0; kk < superleaf; kk += 2) {
            const int64_t k = k0 + kk + g;
            const float a = row_ok ? xrow[k] : 0.0f;
            const float b = col_ok ? wcol[k * ldw] : 0.0f;
            acc = mfma_f32(a, b, acc);
        }
        const int t = __builtin_ctz(~(unsigned)j);         // carry-over: as many finished subtrees as trailing one bits
        for (int l = 0; l < t; ++l) {
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = stash[l][r] + acc[r];
        }
        if (j + 1 < ns_per_shard) {
#pragma unroll
            for (int r = 0; r < 16; ++r) stash[t][r] = acc[r];
        }
    }
    if (!col_ok) return;
    const int col = n0 + i;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int row = m0 + 8 * (r >> 2) + 4 * g + (r & 3);   // D layout of the 32x32 MFMA
        if (row >= M) continue;
        if (partials) partials[((int64_t)p * M + row) * N + col] = acc[r];
        if (Y) Y[(int64_t)row * ldy + col] = acc[r];
    }
}

// ---------------------------------------------------------------------------------------------------------------
// Tiled: a workgroup of 4 wavefronts (2 x 2, each 64 x 64 = 2 x 2 MFMA tiles) owns a 128 x 128 output tile of one
// K-shard.  K-steps of 32 go through a ring of 4 LDS slots filled by direct global->LDS loads issued three steps
// ahead and needed two steps later (about 8000 cycles: a K-step is 64 MFMAs of 64 cycles per wavefront), so memory latency stays hidden with
// one wavefront per SIMD and no staging registers.  The fp32 MFMA is slow enough that neither the LDS fill (8 B/clk)
// nor the fragment reads (one 4-byte read per MFMA) come near a limit; what does cost is every instruction of the
// wavefront's own vector ALU between MFMAs, so the K-loop is kept free of them.
//   Slot = [X tile: 128 rows x 32 k, 128 B per row][W tile: 32 k x 128 columns, 512 B per row], no padding (a direct
//   load writes 1 KiB of consecutive LDS); bank conflicts are kept low by swizzles applied on the global side:
//   X: the 16-byte chunk c of row r sits at position c ^ (r & 7)             (4-byte fragment reads: 4 lanes per bank)
//   W: chunk c of row k sits at position c ^ (8 (k & 1))                     (the two k-slots of a step: other banks)
// Wavefront w loads X rows 32 w .. 32 w + 31 (4 loads of 8 rows) and W rows 8 w .. 8 w + 7 (4 loads of 2 rows).
// Rows past M repeat row M - 1 and column chunks past N repeat the last chunk (such outputs are never stored).
// ---------------------------------------------------------------------------------------------------------------
constexpr int F32_BN = 128, F32_BK = 32;
constexpr int F32_RING = 4;
constexpr int F32_B_BYTES = F32_BK * F32_BN * 4;           // 16 KiB
constexpr unsigned F32_BIAS = 4096;                        // keeps the biased lane offsets non-negative

struct F32Params {
    const float *X, *W;
    float *partials, *Y;
    int64_t ldx, ldw, ldy;
    int M, N;
    int stages_per_superleaf;   // superleaf / 32
    int ns_per_shard;
    int64_t k_per_shard;
    int tiles_m, tiles_n;       // output tiles
    int blocks_n, blocks;       // blocks of 8 x 4 tiles: per row of blocks, in all (large tile only)
    int shards;
};

template <int N>
__device__ __forceinline__ void f32_wait_loads_and_barrier() {
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(N) : "memory");
}

// MT x NT MFMA tiles per wavefront, WN wavefronts side by side (4 / WN on top of each other):
//   <2, 2, 2>  128 x 128 tile, for batches that fill it;
//   <1, 1, 4>   32 x 128 tile, for small batches: a quarter of the MFMA work per weight byte, so that streaming W
//               (not multiplying rows that do not exist) sets the time.
// Same instructions on the same k in the same order per output element, hence the same bits.
template <int LEVELS, int MT, int NT, int WN>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
void gemm_f32_tiled_kernel(const F32Params p) {
    constexpr int WM = 4 / WN;
    constexpr int BM = 32 * MT * WM;
    static_assert(32 * NT * WN == F32_BN && (BM == 128 || BM == 32), "tile shape");
    constexpr int A_BYTES = BM * F32_BK * 4;
    constexpr int SLOT_BYTES = A_BYTES + F32_B_BYTES;
    constexpr int A_LOADS = BM / 32;                       // per wavefront and K-step: BM / 4 rows, 8 rows per load
    constexpr int LOADS = A_LOADS + 4;
    extern __shared__ __attribute__((aligned(16))) float smem_f32[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int li = lane & 31, lg = lane >> 5;

    int shard, tile_m, tile_n;
    if (BM == 128) {
        // Consecutive workgroups go round the 8 XCDs, and the 32 workgroups that an XCD (32 compute units, one workgroup
        // each) runs at a time should share operand panels in its L2.  Tiles are grouped into blocks of 8 x 4 (12 panels
        // for 32 tiles); block q runs on XCD q % 8 as that XCD's round q / 8.  Workgroups whose slot falls outside the
        // matrix (ragged block, padding of the grid to whole rounds) leave at once.
        const int id = blockIdx.x;
        const int slot_in_block = (id >> 3) & 31;
        const int q = ((id >> 8) << 3) + (id & 7);
        shard = q / p.blocks;
        const int blk = q % p.blocks;
        tile_m = (blk / p.blocks_n) * 8 + (slot_in_block >> 2);
        tile_n = (blk % p.blocks_n) * 4 + (slot_in_block & 3);
        if (shard >= p.shards || tile_m >= p.tiles_m || tile_n >= p.tiles_n) return;      // uniform
    } else {
        // Few rows: every workgroup streams its own panel of W; the grid is exactly tiles x shards.
        const int id = blockIdx.x;
        tile_n = id % p.tiles_n;
        tile_m = (id / p.tiles_n) % p.tiles_m;
        shard = id / (p.tiles_n * p.tiles_m);
    }
    const int m0 = tile_m * BM, n0 = tile_n * F32_BN;
    const int64_t kbase = (int64_t)shard * p.k_per_shard;

    // ---- direct loads: per-lane byte offsets from the wave-uniform stage pointers (minus the instruction offset) ----
    // Wavefront w loads X rows (BM / 4) w .. (A_LOADS loads of 8 rows) and W rows 8 w .. 8 w + 7 (4 loads of 2 rows).
    unsigned a_lo[A_LOADS], b_lo[4];
#pragma unroll
    for (int i = 0; i < A_LOADS; ++i) {
        const int r = (BM / 4) * wave + 8 * i + (lane >> 3);                 // row of the X tile
        const int rg = min(m0 + r, p.M - 1) - m0;                            // row fetched into its place; >= 0 since m0 < M
        const int c = (lane & 7) ^ (r & 7);                                  // chunk that belongs at this lane's position
        a_lo[i] = (unsigned)((int64_t)rg * p.ldx * 4 + c * 16 + (int64_t)F32_BIAS) - 1024u * i;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int kr = 8 * wave + 2 * i + (lane >> 5);                       // row of the W tile
        const int cb = (lane & 31) ^ ((kr & 1) << 3);
        const int cg = min(n0 / 4 + cb, p.N / 4 - 1);                        // absolute chunk column, clamped
        b_lo[i] = (unsigned)((int64_t)kr * p.ldw * 4 + cg * 16 + (int64_t)F32_BIAS) - 1024u * i;
    }
    const char *a_ptr = reinterpret_cast<const char *>(p.X + (int64_t)m0 * p.ldx + kbase) - F32_BIAS;
    const char *b_ptr = reinterpret_cast<const char *>(p.W + kbase * p.ldw) - F32_BIAS;
    const int64_t b_stage_bytes = (int64_t)F32_BK * p.ldw * 4;
    const unsigned smem_lds = (unsigned)(uintptr_t)(__attribute__((address_space(3))) float *)smem_f32;
    const unsigned a_m0 = smem_lds + wave * (A_LOADS * 1024), b_m0 = smem_lds + A_BYTES + wave * 4096;

    const int total_stages = p.ns_per_shard * p.stages_per_superleaf;
    int issued = 0;                                        // K-steps whose loads have been started
    // One of the direct loads of a K-step (pointers and m0 values of that step in scalar registers).
    auto load_one = [&](int i, const char *ap, const char *bp, unsigned am, unsigned bm) __attribute__((always_inline)) {
        if (i < A_LOADS) {
            switch (i) {
                case 0: load_16B_per_lane_to_lds<0, true>(ap, a_lo[0], am); break;
                case 1: load_16B_per_lane_to_lds<1024, true>(ap, a_lo[1 % A_LOADS], am); break;
                case 2: load_16B_per_lane_to_lds<2048, true>(ap, a_lo[2 % A_LOADS], am); break;
                default: load_16B_per_lane_to_lds<3072, true>(ap, a_lo[3 % A_LOADS], am); break;
            }
        } else {
            switch (i - A_LOADS) {
                case 0: load_16B_per_lane_to_lds<0, true>(bp, b_lo[0], bm); break;
                case 1: load_16B_per_lane_to_lds<1024, true>(bp, b_lo[1], bm); break;
                case 2: load_16B_per_lane_to_lds<2048, true>(bp, b_lo[2], bm); break;
                default: load_16B_per_lane_to_lds<3072, true>(bp, b_lo[3], bm); break;
            }
        }
    };
    auto issue_stage = [&]() __attribute__((always_inline)) {
        const unsigned slot = (unsigned)(issued & (F32_RING - 1)) * SLOT_BYTES;
        const char *ap = uniform_pointer(a_ptr), *bp = uniform_pointer(b_ptr);
        const unsigned am = __builtin_amdgcn_readfirstlane(a_m0 + slot), bm = __builtin_amdgcn_readfirstlane(b_m0 + slot);
#pragma unroll
        for (int i = 0; i < LOADS; ++i) load_one(i, ap, bp, am, bm);
        a_ptr += F32_BK * 4;
        b_ptr += b_stage_bytes;
        ++issued;
    };

    // ---- fragment reads ----
    // Any vector-ALU instruction between two MFMAs of this wavefront costs 8-15 cycles of the matrix pipe (measured), so
    // the K-loop holds none but the address updates, once per K-step: every read address is a register prepared here
    // (the swizzle included) plus an immediate offset, and the registers move from ring slot to ring slot by one add each.
    // X: lane (row li, slot lg) reads k = 2 ks + lg of its row, i.e. element 2 (ks & 1) + lg of chunk ks / 2: one
    // two-address read per chunk and row block serves MFMA steps 2 c and 2 c + 1.  (4 lanes share a bank: with rows of 32
    // floats and 16-byte placement no better is possible; the reads run a group ahead and are not waited for.)
    unsigned a_at[MT][F32_BK / 4], b_at[NT];               // LDS byte addresses, of the slot that is read next
#pragma unroll
    for (int x = 0; x < MT; ++x) {
        const int r = wm * (32 * MT) + x * 32 + li;
#pragma unroll
        for (int c = 0; c < F32_BK / 4; ++c) a_at[x][c] = smem_lds + (unsigned)(r * 32 + 4 * (c ^ (r & 7)) + lg) * 4u;
    }
#pragma unroll
    for (int y = 0; y < NT; ++y) {
        const int col = wn * (32 * NT) + y * 32 + li;
        b_at[y] = smem_lds + (unsigned)(A_BYTES / 4 + lg * 128 + 4 * ((col >> 2) ^ (lg << 3)) + (col & 3)) * 4u;   // + 1024 ks
    }
    auto lds_f32 = [&](unsigned lds_address) __attribute__((always_inline)) {
        return *reinterpret_cast<const __attribute__((address_space(3))) float *>((uintptr_t)lds_address);
    };

    // Fragments of a group of 4 MFMA steps (8 k), two register sets: a group is read while the one before it is
    // multiplied, also across the K-step boundary.
    constexpr int GROUP = 4, GROUPS = F32_BK / 2 / GROUP;
    constexpr int PER_GROUP = GROUP * MT * NT;             // MFMAs of a group
    constexpr int READS = 2 * MT + 2 * NT;                 // memory instructions of a group's fragment reads
    static_assert(GROUPS % 2 == 0 && PER_GROUP % READS == 0, "group 0 of every K-step uses register set 0; reads spread evenly");
    float fa[2][GROUP][MT], fb[2][GROUP][NT];
    auto read_one = [&](int set, int g, int r) __attribute__((always_inline)) {
        if (r < 2 * MT) {
            const int h = r / MT, x = r % MT;
            fa[set][2 * h][x] = lds_f32(a_at[x][g * (GROUP / 2) + h]);
            fa[set][2 * h + 1][x] = lds_f32(a_at[x][g * (GROUP / 2) + h] + 8);
        } else {
            const int q = 2 * ((r - 2 * MT) / NT), y = (r - 2 * MT) % NT, ks = g * GROUP + q;
            fb[set][q][y] = lds_f32(b_at[y] + 1024 * ks);
            fb[set][q + 1][y] = lds_f32(b_at[y] + 1024 * (ks + 1));
        }
    };
    // Moves the read addresses to the next ring slot (wave-uniform step, negative at the wrap).
    auto advance_reads = [&](int from_slot) __attribute__((always_inline)) {
        const unsigned step = (from_slot == F32_RING - 1) ? (unsigned)(-(F32_RING - 1) * SLOT_BYTES) : (unsigned)SLOT_BYTES;
#pragma unroll
        for (int x = 0; x < MT; ++x)
#pragma unroll
            for (int c = 0; c < F32_BK / 4; ++c) a_at[x][c] += step;
#pragma unroll
        for (int y = 0; y < NT; ++y) b_at[y] += step;
    };

    int s = 0;                                             // K-step being multiplied
    // One K-step of 32: 16 MFMA steps of 2 k on each of the wavefront's tiles (64 cycles per MFMA).  A memory instruction
    // keeps the issue port for tens of cycles, so they are spread one by one between the MFMAs (which run on while the
    // port is busy): the fragment reads of the next group at even distances, and the direct loads of K-step s + 3 after
    // other MFMAs (large tile: two per group; small tile: one per group and a fifth in group 0).
    // FIRST: first K-step of a superleaf, the accumulators start at +0.
    auto stage = [&](auto first, Acc<MT, NT> &a) __attribute__((always_inline)) {
        constexpr bool FIRST = decltype(first)::value;
        // Top of K-step s: this wavefront's loads of step s + 1 have landed when at most those of step s + 2 are in
        // flight; after the barrier step s + 1 is whole in LDS (its first fragments are read during this step) and
        // nobody reads the slot of step s - 1 any more, which step s + 3 takes.
        if (issued >= s + 3) f32_wait_loads_and_barrier<LOADS>();
        else f32_wait_loads_and_barrier<0>();
        const bool fetch = issued < total_stages;          // uniform
        const unsigned slot = (unsigned)(issued & (F32_RING - 1)) * SLOT_BYTES;
        const char *ap = uniform_pointer(a_ptr), *bp = uniform_pointer(b_ptr);
        const unsigned am = __builtin_amdgcn_readfirstlane(a_m0 + slot), bm = __builtin_amdgcn_readfirstlane(b_m0 + slot);
        f32x16 zero;
        if (FIRST) {
#pragma unroll
            for (int r = 0; r < 16; ++r) zero[r] = 0.0f;
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < GROUPS * PER_GROUP; ++j) {
            const int g = j / PER_GROUP, jj = j % PER_GROUP;
            const int q = jj / (MT * NT), x = (jj / NT) % MT, y = jj % NT;
            // The last group reads the first fragments of K-step s + 1 (after the last step: of a slot nobody needs).
            if (g == GROUPS - 1 && jj == 0) advance_reads(s & (F32_RING - 1));
            a.t[x][y] = mfma_f32(fa[g & 1][q][x], fb[g & 1][q][y], (FIRST && j < MT * NT) ? zero : a.t[x][y]);
            if (jj % (PER_GROUP / READS) == 0) read_one((g + 1) & 1, (g + 1) % GROUPS, jj / (PER_GROUP / READS));
            if (BM == 128) {                               // which direct load follows this MFMA, if any
                if (jj == 5 || jj == 11) {
                    if (fetch) load_one(2 * g + (jj == 11), ap, bp, am, bm);
                }
            } else {
                if (jj == 1) {
                    if (fetch) load_one(g, ap, bp, am, bm);
                }
                if (jj == 3 && g == 0) {
                    if (fetch) load_one(4, ap, bp, am, bm);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        if (fetch) {
            a_ptr += F32_BK * 4;
            b_ptr += b_stage_bytes;
            ++issued;
        }
        ++s;
    };
    // One superleaf: chains its K-steps in ascending k.
    auto superleaf = [&](Acc<MT, NT> &a) {
        stage(std::true_type{}, a);
#pragma nounroll
        for (int q = 1; q < p.stages_per_superleaf; ++q) stage(std::false_type{}, a);
    };

#pragma unroll
    for (int i = 0; i < F32_RING - 1; ++i)
        if (issued < total_stages) issue_stage();
    if (issued >= 3) f32_wait_loads_and_barrier<2 * LOADS>();          // K-step 0 has landed everywhere
    else if (issued == 2) f32_wait_loads_and_barrier<LOADS>();
    else f32_wait_loads_and_barrier<0>();
#pragma unroll
    for (int r = 0; r < READS; ++r) read_one(0, 0, r);

    Acc<MT, NT> acc, acc2;
    TileStash<LEVELS - 1, MT, NT> stash;
    SubtreeWalker<LEVELS>::run(superleaf, acc, acc2, stash);

    // acc = T(superleaves of this shard).  D layout: register r of lane l is row 8 (r / 4) + 4 (l / 32) + r % 4, column l % 32.
    float *dst = p.partials ? p.partials + (int64_t)shard * p.M * p.N : p.Y;
    const int64_t ld = p.partials ? (int64_t)p.N : p.ldy;
#pragma unroll
    for (int x = 0; x < MT; ++x)
#pragma unroll
        for (int y = 0; y < NT; ++y) {
            const int col = n0 + wn * (32 * NT) + y * 32 + li;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + wm * (32 * MT) + x * 32 + 8 * (r >> 2) + 4 * lg + (r & 3);
                if (row < p.M && col < p.N) __builtin_nontemporal_store(acc.t[x][y][r], dst + (int64_t)row * ld + col);   // read by a later kernel, if at all
            }
        }
}

bool gemm_f32_tiled_supports(const GemmArgs &a) {
    const int per = a.ns / a.P;
    // Whole 16-byte chunks of a row of W are fetched, so N has to be a multiple of 4; a lane's byte offset inside a
    // K-step (up to 127 rows of X, 31 rows of W) has to fit 32 bits.
    return a.superleaf % F32_BK == 0 && per >= 1 && per <= 16 && a.N % 4 == 0 && a.ldx < (1 << 23) && a.ldw < (1 << 23);
}

hipError_t launch_gemm_f32_reference(const GemmArgs &a, hipStream_t s) {
    if (a.M <= 0 || a.N <= 0) return hipSuccess;
    dim3 grid((a.N + 31) / 32, (a.M + 31) / 32, a.P);
    if (grid.y > 65535u || grid.z > 65535u) return hipErrorInvalidValue;
    float *Y = (a.P == 1) ? reinterpret_cast<float *>(a.Y) : nullptr;
    hipLaunchKernelGGL(gemm_f32_reference_kernel, grid, dim3(64), 0, s, reinterpret_cast<const float *>(a.X), a.ldx,
                       reinterpret_cast<const float *>(a.W), a.ldw, a.partials, Y, a.ldy, a.M, a.N, a.superleaf, a.ns / a.P);
    return hipGetLastError();
}

template <int LEVELS, int MT, int NT, int WN>
static hipError_t launch_f32_levels(const F32Params &p, unsigned grid, hipStream_t s) {
    constexpr int LDS_BYTES = F32_RING * (32 * MT * (4 / WN) * F32_BK * 4 + F32_B_BYTES);
    static std::atomic<unsigned> done{0};                 // bit d: the LDS attribute is set on device d
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 32) dev = 32;
    if (dev >= 32 || !((done.load(std::memory_order_relaxed) >> dev) & 1u)) {
        hipError_t e = hipFuncSetAttribute((const void *)gemm_f32_tiled_kernel<LEVELS, MT, NT, WN>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
        if (e != hipSuccess) return e;
        if (dev < 32) done.fetch_or(1u << dev, std::memory_order_relaxed);
    }
    hipLaunchKernelGGL((gemm_f32_tiled_kernel<LEVELS, MT, NT, WN>), dim3(grid), dim3(256), LDS_BYTES, s, p);
    return hipGetLastError();
}

template <int MT, int NT, int WN>
static hipError_t launch_f32_shape(const GemmArgs &a, hipStream_t s) {
    constexpr int BM = 32 * MT * (4 / WN);
    F32Params p;
    p.X = reinterpret_cast<const float *>(a.X);
    p.W = reinterpret_cast<const float *>(a.W);
    p.partials = a.partials;
    p.Y = reinterpret_cast<float *>(a.Y);
    p.ldx = a.ldx; p.ldw = a.ldw; p.ldy = a.ldy;
    p.M = a.M; p.N = a.N;
    p.stages_per_superleaf = a.superleaf / F32_BK;
    p.ns_per_shard = a.ns / a.P;
    p.k_per_shard = (int64_t)p.ns_per_shard * a.superleaf;
    p.tiles_n = (a.N + F32_BN - 1) / F32_BN;
    p.tiles_m = (a.M + BM - 1) / BM;
    p.blocks_n = (p.tiles_n + 3) / 4;
    p.blocks = p.blocks_n * ((p.tiles_m + 7) / 8);
    p.shards = a.P;
    int64_t work;
    if (BM == 128) work = (((int64_t)p.blocks * a.P + 7) / 8) * 256;     // rounds of 8 blocks of 32 tiles, one block per XCD
    else work = (int64_t)p.tiles_m * p.tiles_n * a.P;
    if (work > 0x7fffffff) return hipErrorInvalidValue;
    int levels = 0;
    while ((1 << levels) < p.ns_per_shard) ++levels;
    switch (levels) {
        case 0: return launch_f32_levels<0, MT, NT, WN>(p, (unsigned)work, s);
        case 1: return launch_f32_levels<1, MT, NT, WN>(p, (unsigned)work, s);
        case 2: return launch_f32_levels<2, MT, NT, WN>(p, (unsigned)work, s);
        case 3: return launch_f32_levels<3, MT, NT, WN>(p, (unsigned)work, s);
        case 4: return launch_f32_levels<4, MT, NT, WN>(p, (unsigned)work, s);
        default: return hipErrorInvalidValue;
    }
}

// variant: VARIANT_T128 forces the 128-row tile, VARIANT_T32 / VARIANT_T64 the 32-row tile; otherwise by the batch.
hipError_t launch_gemm_f32_tiled(const GemmArgs &a, int variant, hipStream_t s) {
    if (a.M <= 0 || a.N <= 0) return hipSuccess;
    if (!gemm_f32_tiled_supports(a)) return hipErrorInvalidValue;
    const bool small = (variant == VARIANT_T32 || variant == VARIANT_T64) || (variant != VARIANT_T128 && a.M <= 64);
    return small ? launch_f32_shape<1, 1, 4>(a, s) : launch_f32_shape<2, 2, 2>(a, s);
}

}  // namespace tbik
