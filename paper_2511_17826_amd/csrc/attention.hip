// Batch-invariant attention for gfx950: one kernel for prefill, decode and anything between, with a FIXED key tile
// (the attention rule of the paper's implementation appendix, "Framework Modifications": fix the tile size, run
// prefill and decode through the same kernel; Sec. 2.1: fp32 accumulators).
//
// A workgroup of 4 wavefronts owns 128 query rows of one sequence that share ONE key/value head, so that a key tile
// is fetched once for all of them: with `pack` query heads per key/value head packed into a workgroup, row slot s
// is query (128 / pack) * block + s % (128 / pack) of query head pack * kvhead + s / (128 / pack).  (pack = the size
// of a head group when that is a power of two up to 128, else 1.)  A decode step (one query per sequence) then
// costs one pass over the keys per key/value head instead of one per query head.  Which slot a query lands in has
// no influence on its bits.
// The keys of the sequence are visited in tiles of ATT_KV = 64 at absolute positions [64 t, 64 t + 64), in
// ascending order, with the streaming-softmax recurrence per query row:
//     s_j = (q . k_j) * c            c = scale * log2(e), fp32
//     m'  = max(m, max_j s_j);  a = exp2(m - m');  p_j = exp2(s_j - m')
//     l   = l a + sum_j p_j;    o = o a + sum_j r16(p_j) v_j;    m = m'
// and O = o / l, rounded once to 16 bits (r16: to the tensors' format, bf16 or with F16 IEEE binary16; the MFMA
// opcode and the two conversions are all that depends on the format).  Nothing in a row's arithmetic depends on the other rows of the block, on
// the number of queries in the call or on the batch: a tile that is masked for a row leaves that row's (m, l, o)
// unchanged bit for bit (a = 1, p = 0), so the number of tiles a block walks does not matter either.
//
// Beyond ATT_SPLIT = 64 tiles (4096 keys) the key axis is cut into splits at absolute tile numbers: each split runs
// the recurrence from the empty state, and the splits' states are folded in ascending order (state_fold below; an
// empty split is skipped exactly).  This is an extension of the paper's rule, which keeps decode and prefill on one
// order by leaving the key axis unsplit: a split that is fixed, and used in every phase, keeps them on one order as
// well, and the splits of a long sequence can run at the same time.  Two forms, same bits: a workgroup walks all its
// tiles and folds at every 64th through a state kept in the workspace (calls with many workgroups), or one workgroup
// per split writes its state and attention_merge_kernel folds them (decode steps on few long sequences).
//
// Everything is computed transposed, so that a lane owns ONE query (column lane % 32 of every MFMA result) and
// the per-query state m, l, a lives in one register per lane:
//     S^T (keys x queries)  = K (A operand, 16-byte LDS reads)        x Q^T (B operand, in registers for the whole block)
//     O^T (channels x queries) = V^T (A operand, transposing LDS read) x P^T (B operand = the S^T registers, rounded to 16 bits)
// The MFMA's k-slot (g, t) of step s stands for key 32 kb + 16 h + 8 (t / 4) + 4 g + t % 4 (kb = s / 2, h = s % 2): the
// order in which the result layout of S^T hands the keys to a lane; V^T is fetched in the same order.
#include <algorithm>
#include <atomic>
#include <cstdint>
#include <type_traits>

#include "tbik_device.hpp"
#include "tbik_internal.hpp"

namespace tbik {

constexpr int ATT_D = 128;    // head dimension
constexpr int ATT_BQ = 128;   // queries per workgroup
constexpr int ATT_KV = 64;    // keys per tile: part of the result, never tuned per call
constexpr int ATT_TILE_BYTES = ATT_KV * ATT_D * 2;
#ifndef TBIK_ATT_SPLIT
#define TBIK_ATT_SPLIT 64     // other values: timing experiments only (the bits change, the oracle's tests fail)
#endif
constexpr int ATT_SPLIT = TBIK_ATT_SPLIT;   // key tiles per split (4096 keys): part of the result as well
constexpr int ATT_THREAD_STATE = 4 + ATT_D / 32 * 16;            // floats of one thread's softmax state: m, l, two unused, o
constexpr int ATT_STATE_FLOATS = ATT_THREAD_STATE * 256;         // one workgroup's

typedef short att_v4i16 __attribute__((ext_vector_type(4)));
typedef unsigned int att_u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int att_u32x2 __attribute__((ext_vector_type(2)));

struct AttnParams {
    const uint16_t *Q, *K, *V;
    uint16_t *O;
    const int32_t *cu_q, *cu_k;
    int64_t q_stride, k_stride, v_stride, o_stride;   // token strides, elements
    int total_q, total_k;
    int group;                                        // query heads per key/value head
    int pack;                                         // query heads per workgroup (group or 1)
    int rows;                                         // queries per head and workgroup: 128 / pack
    float c;                                          // scale * log2(e)
    int ny, nz;                                       // head groups, sequences
    int nb;                                           // bound on the query blocks of the call: block ids 0 .. nb - 1 (see attention_work_item)
    int chunk, nchunks;                               // block ids are dealt to the XCDs in chunks of this many
    int chunk_lo, chunk_hi;                           // this launch covers chunks chunk_lo .. chunk_hi - 1 (a long call is
                                                      // launched in several pieces that take turns at one capped scratch area)
    int n_splits;                                     // 1: an item walks all key tiles (folding its splits as it goes);
                                                      // > 1: an item is one split of those, its state goes to `states`
    int max_tiles;                                    // key tiles of a sequence of max_seqlen_k keys: no workgroup walks further
    float *states;                                    // n_splits == 1: one state per item, scratch of the fold between splits;
                                                      // n_splits > 1: [item][split] states for attention_merge_kernel
};

__device__ __forceinline__ int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

// Query blocks are numbered over the whole call without a table: sequence b owns the ids G(b) .. G(b) + blocks(b) - 1
// with G(b) = cu_q[b] / R + b (R queries per block; G(b + 1) - G(b) >= ceil(Lq_b / R), so the ranges do not overlap,
// and all ids are below total_q / R + batch).  A few ids between the ranges belong to nobody.  The host needs no
// sequence length for this (the launch is sized from total_q), and a call of one long chunk and many decode steps
// launches about as many workgroups as it has blocks -- not batch x blocks of the longest.
// Returns the sequence of block id g: the largest b with G(b) <= g, by a 64-way search (one or two rounds for any
// realistic batch); the same value in every lane.  Offsets that do not ascend give some sequence in range, no more.
__device__ __forceinline__ int sequence_of_block(const AttnParams &p, int R, int g, int lane) {
    int lo = 0, n = p.nz;
    while (n > 1) {
        const int step = (n + 63) >> 6;
        const int b = lo + lane * step;
        const bool ok = b < lo + n && clampi(p.cu_q[min(b, p.nz - 1)], 0, p.total_q) / R + b <= g;
        const int k = max(__builtin_popcountll(__builtin_amdgcn_ballot_w64(ok)) - 1, 0);
        n = min(step, lo + n - (lo + k * step));
        lo += k * step;
    }
    return __builtin_amdgcn_readfirstlane(lo);
}

// Work item of this workgroup; false if it has none.  Consecutive workgroups go round the 8 XCDs.  A run is a chunk
// of consecutive block ids of one head group and split -- mostly query blocks of one sequence, which read the same
// keys and values -- and run u goes to XCD u % 8 as a whole, so that the workgroups an XCD runs at a time find their
// keys in that XCD's L2 (consecutive query blocks on different XCDs: every XCD walks every head's keys, 3.4 times the
// algorithmic fetch); with a multiple of 8 head groups a head group stays on one XCD.  Late chunks, and in a chunk late
// blocks, come first: under a causal mask they are the long ones.
__device__ __forceinline__ bool attention_work_item(const AttnParams &p, int R, int lane, int &qb, int &by, int &seq, int &split, int &base) {
    const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
    const int bx = j % p.chunk;
    int t = xcd + 8 * (j / p.chunk);
    split = t % p.n_splits;
    t /= p.n_splits;
    by = t % p.ny;
    const int ch = p.chunk_hi - 1 - t / p.ny;
    if (ch < p.chunk_lo) return false;                // the launch is padded to a multiple of 8 runs
    const int g = ch * p.chunk + (p.chunk - 1 - bx);
    if (g >= p.nb) return false;
    seq = sequence_of_block(p, R, g, lane);
    qb = g - (clampi(p.cu_q[seq], 0, p.total_q) / R + seq);
    base = g * p.ny + by;                             // number of the (block id, head group) pair
    return true;
}

// The softmax state of one split of the keys, (m, l, o) per thread, and the fold of two of them (the accumulated one
// A and the next split's B):  M = max(mA, mB);  a = exp2(mA - M), b = exp2(mB - M);  l = fl(lA a) + fl(lB b);
// o = fl(oA a) + fl(oB b).  A split in which the query saw no key (l == 0) is skipped: the other state is taken as it
// is, bit for bit.  The function is symmetric in its two arguments, and every multiplication and addition is a single
// rounded operation (no contraction), so that the fold gives the same bits wherever it runs.
// Layout in memory, in units of 16 bytes: chunk c of thread t at [c * 256 + t] -- chunk 0 is (m, l, -, -), chunk
// 1 + 4 db + q holds o[db][4 q .. 4 q + 3] -- so that the lanes of a wavefront touch consecutive memory (a thread's 272
// bytes side by side cost 25 us per fold on a full chip: 64 cache lines per instruction).  The workgroup's base is
// uniform and the pointer says "global" (it went through scalar registers as integers, which made it a generic one),
// so the accesses take the scalar base + lane offset form: one address register.
typedef __attribute__((address_space(1))) f32x4 global_f32x4;

// Chunk c of thread tid: a uniform base (scalar registers) plus an unsigned 32-bit lane offset.
__device__ __forceinline__ global_f32x4 *state_chunk(const f32x4 *wg, int c, int tid) {
    typedef __attribute__((address_space(1))) char global_char;
    global_char *base = (global_char *)const_cast<f32x4 *>(wg + c * 256);
    return (global_f32x4 *)(base + (uint64_t)((uint32_t)tid * 16u));
}

__device__ __forceinline__ void state_store(f32x4 *wg, int tid, float m, float l, const f32x16 (&o)[ATT_D / 32]) {
    *state_chunk(wg, 0, tid) = f32x4{m, l, 0.0f, 0.0f};
#pragma unroll
    for (int db = 0; db < ATT_D / 32; ++db)
#pragma unroll
        for (int q = 0; q < 4; ++q) *state_chunk(wg, 1 + 4 * db + q, tid) = f32x4{o[db][4 * q], o[db][4 * q + 1], o[db][4 * q + 2], o[db][4 * q + 3]};
}

// (m, l, o) <- fold(the state stored at `wg`, (m, l, o))
__device__ __forceinline__ void state_fold(const f32x4 *wg, int tid, float &m, float &l, f32x16 (&o)[ATT_D / 32]) {
    const f32x4 h = *state_chunk(wg, 0, tid);
    const float m2 = h[0], l2 = h[1];
    const float M = fmaxf(m2, m);
    const float m_use = (M == -INFINITY) ? 0.0f : M;
    const float a2 = __builtin_amdgcn_exp2f(m2 - m_use), a1 = __builtin_amdgcn_exp2f(m - m_use);
    const bool mine_empty = (l == 0.0f), other_empty = (l2 == 0.0f);
#pragma unroll
    for (int db = 0; db < ATT_D / 32; ++db) {
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) {                          // eight values at a time: the callers have few registers to spare
            const f32x4 x0 = *state_chunk(wg, 1 + 4 * db + 2 * hh, tid), x1 = *state_chunk(wg, 2 + 4 * db + 2 * hh, tid);
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                const float o2 = r < 4 ? x0[r] : x1[r - 4];
                const float t = __fadd_rn(__fmul_rn(o2, a2), __fmul_rn(o[db][8 * hh + r], a1));
                o[db][8 * hh + r] = mine_empty ? o2 : (other_empty ? o[db][8 * hh + r] : t);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    const float lt = __fadd_rn(__fmul_rn(l2, a2), __fmul_rn(l, a1));
    l = mine_empty ? l2 : (other_empty ? l : lt);
    m = mine_empty ? m2 : (other_empty ? m : M);
}

// O = o / l, one rounding to the 16-bit format; lane (query li, half lg) holds channels 32 db + 8 q + 4 lg + (0..3).
template <bool F16>
__device__ __forceinline__ void attention_store_output(uint16_t *optr, float l, const f32x16 (&o)[ATT_D / 32]) {
#pragma unroll
    for (int db = 0; db < ATT_D / 32; ++db)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            float v[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) v[i] = (l > 0.0f) ? o[db][4 * q + i] / l : 0.0f;
            att_u32x2 w;
            w[0] = pack_16x2<F16>(v[0], v[1]);
            w[1] = pack_16x2<F16>(v[2], v[3]);
            *reinterpret_cast<att_u32x2 *>(optr + db * 32 + 8 * q) = w;
        }
}

// A lane and its partner lane ^ 32 hold the two halves of one query's keys.  v_permlane32_swap exchanges the upper
// half of its first operand with the lower half of its second: from (v, v) it makes (lower half's values, upper
// half's values) in every lane, i.e. {mine, partner's} in some order -- enough for a maximum or a sum of the two.
__device__ __forceinline__ void both_halves(float v, float &a, float &b) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    a = __uint_as_float(r[0]);
    b = __uint_as_float(r[1]);
}

template <bool CAUSAL, bool F16>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
void attention_kernel(const AttnParams p) {
    // LDS: K tile [2][64 keys][256 B], then V tile [2][64 keys][256 B].
    //   K rows: 16-byte chunk c of key r sits at position c ^ (r & 15): the 16 rows of a fragment read hit all banks.
    //   V rows: chunk c of key r sits at position c ^ (4 (r & 3)): the 4 rows of a transposing read differ in banks.
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char *const k_lds = smem;
    unsigned char *const v_lds = smem + 2 * ATT_TILE_BYTES;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 31, lg = lane >> 5;
    int qb, by, seq, split, base_item;
    const int R = p.rows;
    if (!attention_work_item(p, R, lane, qb, by, seq, split, base_item)) return;     // uniform
    const bool one_split_each = p.n_splits > 1;                   // uniform: this workgroup computes one split's state
    f32x4 *const my_state = reinterpret_cast<f32x4 *>(const_cast<char *>(uniform_pointer(           // the workgroup's, in scalar registers
        reinterpret_cast<const char *>(p.states + ((size_t)(base_item - p.chunk_lo * p.chunk * p.ny) * p.n_splits + split) * ATT_STATE_FLOATS))));

    // Sequence bounds, clamped so that no value of the offset arrays can lead outside the tensors.
    const int q0 = clampi(p.cu_q[seq], 0, p.total_q), q1 = clampi(p.cu_q[seq + 1], q0, p.total_q);
    const int k0 = clampi(p.cu_k[seq], 0, p.total_k), k1 = clampi(p.cu_k[seq + 1], k0, p.total_k);
    const int Lq = q1 - q0, Lk = k1 - k0;
    if (qb < 0 || qb * R >= Lq) return;                                     // uniform: nothing of this sequence in the block
    const int shift = Lk - Lq;                                    // the queries are the last Lq positions
    const int slot = wave * 32 + li;
    const int head = by * p.pack + slot / R;
    const int hk = (by * p.pack) / p.group;

    const int q_last = min(Lq - 1, qb * R + R - 1);
    const int lim_block = CAUSAL ? min(Lk - 1, q_last + shift) : Lk - 1;
    const int n_tiles = lim_block >= 0 ? min(p.max_tiles, lim_block / ATT_KV + 1) : 0;   // keys past max_seqlen_k are left out

    // This lane's query (rows past the sequence repeat its last query; they are never stored).
    const int qrow = qb * R + slot % R;
    const int qpos = min(qrow, Lq - 1);
    const int lim = CAUSAL ? min(Lk - 1, qpos + shift) : Lk - 1; // last visible key of this query; < 0: none
    // The wavefront as a whole: tiles it has to multiply, and the keys that every one of its rows sees.
    const int wave_first = qb * R + (wave * 32) % R;              // R >= 32: 32 consecutive queries; R < 32: all R of the block
    const int wave_lim = CAUSAL ? min(Lk - 1, min(Lq - 1, wave_first + min(R, 32) - 1) + shift) : Lk - 1;
    const int wave_tiles = (wave_first < Lq && wave_lim >= 0) ? wave_lim / ATT_KV + 1 : 0;
    const int wave_full = CAUSAL ? min(Lk - 1, min(Lq - 1, wave_first) + shift) : Lk - 1;

    // Q^T fragments: lane (query li, half lg) holds channels 16 ks + 8 lg .. + 7 of its query.
    bf16x8 bq[ATT_D / 16];
    {
        const uint16_t *qptr = p.Q + (int64_t)(q0 + qpos) * p.q_stride + (int64_t)head * ATT_D + lg * 8;
#pragma unroll
        for (int ks = 0; ks < ATT_D / 16; ++ks) bq[ks] = *reinterpret_cast<const bf16x8 *>(qptr + ks * 16);
        // A use the compiler can see: it waits for these loads here, once, and not later among the direct loads whose
        // counter values it does not know.
#pragma unroll
        for (int ks = 0; ks < ATT_D / 16; ++ks) asm volatile("" ::"v"(bq[ks]));
    }

    // Tile loader: direct global->LDS loads (no staging registers).  Wavefront w fills key rows 16 w .. 16 w + 15 of a
    // tile with 4 loads for K and 4 for V; load i covers rows 16 w + 4 i .. + 3: lane -> row r = 16 w + 4 i + lane / 16
    // and chunk POSITION lane % 16 of that row in LDS, which holds chunk (lane % 16) ^ (r & 15) of the key's channels for K
    // and (lane % 16) ^ 4 (r & 3) for V (the swizzle is applied on the global side).  Keys past the sequence repeat its
    // last key (they are masked).  Token strides are below 2^24 elements, so a lane's byte offset fits 32 bits.
    const int ld_pos = lane & 15, ld_sub = lane >> 4;
    const uint16_t *kbase = p.K + (int64_t)k0 * p.k_stride + (int64_t)hk * ATT_D;     // wave-uniform
    const uint16_t *vbase = p.V + (int64_t)k0 * p.v_stride + (int64_t)hk * ATT_D;
    unsigned k_ld[4], v_ld[4];                                   // minus the instruction offset 1024 i, which the load adds back
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const unsigned r = 16 * wave + 4 * i + ld_sub;
        k_ld[i] = (r * (unsigned)p.k_stride + ((ld_pos ^ (r & 15)) << 3)) * 2u - 1024u * i;
        v_ld[i] = (r * (unsigned)p.v_stride + ((ld_pos ^ ((r & 3) << 2)) << 3)) * 2u - 1024u * i;
    }
    const unsigned smem_lds = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;
    const unsigned k_m0 = smem_lds + wave * 4096;                // + buffer offset
    const unsigned v_m0 = smem_lds + 2 * ATT_TILE_BYTES + wave * 4096;
    // Starts the loads of tile t into the K buffer at k_off and the V buffer at v_off; they are complete (for this
    // wavefront) after an s_waitcnt vmcnt(0).
    auto fetch = [&](int t, int k_off, int v_off) __attribute__((always_inline)) {
        const char *kt = uniform_pointer(reinterpret_cast<const char *>(kbase + (int64_t)t * ATT_KV * p.k_stride));
        const char *vt = uniform_pointer(reinterpret_cast<const char *>(vbase + (int64_t)t * ATT_KV * p.v_stride));
        const unsigned km = __builtin_amdgcn_readfirstlane(k_m0 + k_off), vm = __builtin_amdgcn_readfirstlane(v_m0 + v_off);
        if (__builtin_expect(t * ATT_KV + ATT_KV <= Lk, 1)) {      // uniform: the whole tile lies inside the sequence
            load_16B_per_lane_to_lds<0, true>(kt, k_ld[0], km);
            load_16B_per_lane_to_lds<1024, false>(kt, k_ld[1], km);
            load_16B_per_lane_to_lds<2048, false>(kt, k_ld[2], km);
            load_16B_per_lane_to_lds<3072, false>(kt, k_ld[3], km);
            load_16B_per_lane_to_lds<0, true>(vt, v_ld[0], vm);
            load_16B_per_lane_to_lds<1024, false>(vt, v_ld[1], vm);
            load_16B_per_lane_to_lds<2048, false>(vt, v_ld[2], vm);
            load_16B_per_lane_to_lds<3072, false>(vt, v_ld[3], vm);
        } else {
            const int last = Lk - 1 - t * ATT_KV;                  // >= 0: the tile holds at least one key
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const unsigned r = 16 * wave + 4 * i + ld_sub;
                const unsigned rg = min((int)r, last);           // row fetched; it still lands in row r's place
                load_16B_per_lane_to_lds<0, true>(kt, (rg * (unsigned)p.k_stride + ((ld_pos ^ (r & 15)) << 3)) * 2u, km + 1024 * i);
                load_16B_per_lane_to_lds<0, true>(vt, (rg * (unsigned)p.v_stride + ((ld_pos ^ ((r & 3) << 2)) << 3)) * 2u, vm + 1024 * i);
            }
        }
    };

    // Fragment addresses inside a tile.
    //   K, block kb, step ks: key 32 kb + li, chunk 2 ks + lg.
    const int k_rd = li * 256;                                   // + kb * 8192; chunk swizzled per step: (2 ks + lg) ^ (li & 15)
    //   V^T, channel block db, step s (kb = s / 2, h = s % 2), half hh: rows 32 kb + 16 h + 8 hh + 4 lg + e, e = l16 / 4,
    //   columns 32 db + 16 ((lane / 16) % 2) + 4 (l16 % 4) .. + 3 before the transpose.
    const int l16 = lane & 15, e = l16 >> 2;
    int v_rd[ATT_D / 32];
#pragma unroll
    for (int db = 0; db < ATT_D / 32; ++db) {
        const int col = db * 32 + ((lane >> 4) & 1) * 16 + (l16 & 3) * 4;
        v_rd[db] = (4 * lg + e) * 256 + ((((col >> 3) ^ (e << 2))) << 4) + ((col >> 2) & 1) * 8;
    }

    f32x16 o[ATT_D / 32];
#pragma unroll
    for (int db = 0; db < ATT_D / 32; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[db][r] = 0.0f;
    float m = -INFINITY, l = 0.0f;

    // Tiles of this workgroup: all of them, or those of its split.
    const int t_begin = one_split_each ? split * ATT_SPLIT : 0;
    const int t_end = one_split_each ? min(n_tiles, t_begin + ATT_SPLIT) : n_tiles;
    if (t_begin >= t_end) {                                       // uniform: no query of the block sees a key (of this split)
        if (one_split_each) {
            *state_chunk(my_state, 0, tid) = f32x4{-INFINITY, 0.0f, 0.0f, 0.0f};   // an empty state: only m and l are looked at
        } else if (qrow < Lq) {
            uint16_t *optr = p.O + (int64_t)(q0 + qrow) * p.o_stride + (int64_t)head * ATT_D + lg * 64;
#pragma unroll
            for (int i = 0; i < 8; ++i) *reinterpret_cast<att_u32x4 *>(optr + 8 * i) = att_u32x4{0, 0, 0, 0};
        }
        return;
    }
    fetch(t_begin, 0, 0);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    // One key tile out of LDS buffer BUF; the next tile is fetched meanwhile and parked in the other buffer.
    auto tile = [&](auto buf_tag, int t) {
        constexpr int BUF = decltype(buf_tag)::value;
        const bool more = t + 1 < t_end;
        if (more) fetch(t + 1, (BUF ^ 1) * ATT_TILE_BYTES, (BUF ^ 1) * ATT_TILE_BYTES);   // lands while this tile is multiplied;
                                                                  // that buffer was last read before the previous barrier

        if (t < wave_tiles) {
            const unsigned char *kt = k_lds + BUF * ATT_TILE_BYTES;
            const unsigned char *vt = v_lds + BUF * ATT_TILE_BYTES;
            // ---- S^T = K Q^T ----
            f32x16 s[2];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) s[kb][r] = 0.0f;
#pragma unroll
            for (int ks = 0; ks < ATT_D / 16; ++ks)               // the two key blocks alternate: consecutive MFMAs are independent
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) {
                    const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(kt + kb * 8192 + k_rd + (((2 * ks + lg) ^ (li & 15)) << 4));
                    s[kb] = mfma_32x32x16<F16>(kf, bq[ks], s[kb]);
                }
            // ---- scale, mask, running maximum ----
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) s[kb][r] = s[kb][r] * p.c;
            if (t * ATT_KV + ATT_KV - 1 > wave_full) {            // uniform: some row of the wavefront does not see the whole tile
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int key = t * ATT_KV + kb * 32 + 8 * (r >> 2) + 4 * lg + (r & 3);
                        if (key > lim) s[kb][r] = -INFINITY;
                    }
            }
            float tmax = s[0][0];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) tmax = fmaxf(tmax, s[kb][r]);
            {
                float a, b;
                both_halves(tmax, a, b);
                tmax = fmaxf(a, b);                               // with the other half of this query's keys
            }
            const float m_new = fmaxf(m, tmax);
            const float m_use = (m_new == -INFINITY) ? 0.0f : m_new;   // a query that has seen no key yet
            const float alpha = __builtin_amdgcn_exp2f(m - m_use);
            float psum = 0.0f;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    s[kb][r] = __builtin_amdgcn_exp2f(s[kb][r] - m_use);
                    psum = psum + s[kb][r];
                }
            {
                float a, b;
                both_halves(psum, a, b);
                psum = a + b;                                     // lower half's sum + upper half's sum, in both lanes
            }
            l = l * alpha + psum;
            m = m_new;
            if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {   // uniform: o * 1 is o, so skipping changes no bit
#pragma unroll
                for (int db = 0; db < ATT_D / 32; ++db)
#pragma unroll
                    for (int r = 0; r < 16; ++r) o[db][r] = o[db][r] * alpha;
            }
            // ---- O^T += V^T P^T ----
#pragma unroll
            for (int st = 0; st < 4; ++st) {
                const int kb = st >> 1, h = st & 1;
                union { uint32_t u[4]; bf16x8 v; } pb;
#pragma unroll
                for (int i = 0; i < 4; ++i) pb.u[i] = pack_16x2<F16>(s[kb][8 * h + 2 * i], s[kb][8 * h + 2 * i + 1]);
#pragma unroll
                for (int db = 0; db < ATT_D / 32; ++db) {
                    union { att_v4i16 h2[2]; bf16x8 v; } vf;
#pragma unroll
                    for (int hh = 0; hh < 2; ++hh)
                        vf.h2[hh] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                            (__attribute__((address_space(3))) att_v4i16 *)(vt + (32 * kb + 16 * h + 8 * hh) * 256 + v_rd[db]));
                    o[db] = mfma_32x32x16<F16>(vf.v, pb.v, o[db]);
                }
            }
        }


        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");          // this wavefront's part of the next tile has landed
        __syncthreads();
    };
    bool folded = false;                                          // uniform: an accumulated state waits in my_state
    for (int t = t_begin; t < t_end; t += 2) {
        if (t > t_begin && (t & (ATT_SPLIT - 1)) == 0) {          // uniform: a split ends here (only when one workgroup walks them all)
            // No direct load is in flight at this point (the tile before waited for its successor), so ordinary
            // loads and stores, which the compiler counts itself, can be used.
            int me = tid;
            asm volatile("" : "+v"(me));                          // the addresses are formed here, not kept in registers across the tiles
            if (folded) state_fold(my_state, me, m, l, o);
            state_store(my_state, me, m, l, o);
            folded = true;
            m = -INFINITY;
            l = 0.0f;
#pragma unroll
            for (int db = 0; db < ATT_D / 32; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) o[db][r] = 0.0f;
        }
        tile(std::integral_constant<int, 0>{}, t);
        if (t + 1 < t_end) tile(std::integral_constant<int, 1>{}, t + 1);
    }

    int me = tid;
    asm volatile("" : "+v"(me));
    if (one_split_each) {                                         // the state as it is; attention_merge_kernel folds and divides
        state_store(my_state, me, m, l, o);
        return;
    }
    if (folded) state_fold(my_state, me, m, l, o);
    if (qrow < Lq) attention_store_output<F16>(p.O + (int64_t)(q0 + qrow) * p.o_stride + (int64_t)head * ATT_D + 4 * lg, l, o);
}

// Folds the states of the splits of each (query block, head group, sequence) triple in ascending order and writes the
// output: the second kernel of a launch in which every split had its own workgroup.  Thread t of a workgroup here
// stands for thread t of those workgroups (same query); blockIdx.y picks one of the four blocks of 32 channels, of
// which the thread folds its 16.  The loads do not depend on the fold, so the states of four splits are fetched at a
// time (one trip to memory per four splits instead of several per split); the fold itself runs split by split, with
// the operations of state_fold.
template <bool F16>
__global__ __launch_bounds__(256) void attention_merge_kernel(const AttnParams p) {
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, lg = lane >> 5;
    const int db = blockIdx.y;
    const int by = blockIdx.x % p.ny, g = blockIdx.x / p.ny;     // g: the block id, as in attention_work_item
    const int R = p.rows;
    const int seq = sequence_of_block(p, R, g, lane);
    const int qb = g - (clampi(p.cu_q[seq], 0, p.total_q) / R + seq);
    const int base_item = blockIdx.x;
    const int q0 = clampi(p.cu_q[seq], 0, p.total_q), q1 = clampi(p.cu_q[seq + 1], q0, p.total_q);
    const int Lq = q1 - q0;
    if (qb < 0 || qb * R >= Lq) return;
    const int slot = wave * 32 + li;
    const int head = by * p.pack + slot / R;
    const int qrow = qb * R + slot % R;
    if (qrow >= Lq) return;
    const f32x4 *states = reinterpret_cast<const f32x4 *>(uniform_pointer(
        reinterpret_cast<const char *>(p.states + (size_t)base_item * p.n_splits * ATT_STATE_FLOATS)));
    float m = -INFINITY, l = 0.0f;                                // the empty state
    float o[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) o[r] = 0.0f;
    constexpr int AHEAD = 4;
    for (int j0 = 0; j0 < p.n_splits; j0 += AHEAD) {
        f32x4 h[AHEAD], x[AHEAD][4];
#pragma unroll
        for (int u = 0; u < AHEAD; ++u) {
            const int j = min(j0 + u, p.n_splits - 1);            // past the end: the last one again, not used
            const f32x4 *st = states + (size_t)j * (ATT_STATE_FLOATS / 4);
            h[u] = *state_chunk(st, 0, tid);
#pragma unroll
            for (int q = 0; q < 4; ++q) x[u][q] = *state_chunk(st, 1 + 4 * db + q, tid);
        }
#pragma unroll
        for (int u = 0; u < AHEAD; ++u) {
            const float m2 = h[u][0], l2 = h[u][1];
            if (j0 + u >= p.n_splits || l2 == 0.0f) continue;     // an empty split (its o was never written) changes nothing
            const float M = fmaxf(m2, m);
            const float m_use = (M == -INFINITY) ? 0.0f : M;
            const float a2 = __builtin_amdgcn_exp2f(m2 - m_use), a1 = __builtin_amdgcn_exp2f(m - m_use);
            const bool mine_empty = (l == 0.0f);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float o2 = x[u][r >> 2][r & 3];
                const float f = __fadd_rn(__fmul_rn(o2, a2), __fmul_rn(o[r], a1));
                o[r] = mine_empty ? o2 : f;
            }
            const float lt = __fadd_rn(__fmul_rn(l2, a2), __fmul_rn(l, a1));
            l = mine_empty ? l2 : lt;
            m = mine_empty ? m2 : M;
        }
    }
    uint16_t *optr = p.O + (int64_t)(q0 + qrow) * p.o_stride + (int64_t)head * ATT_D + 4 * lg + db * 32;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        float v[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = (l > 0.0f) ? o[4 * q + i] / l : 0.0f;
        att_u32x2 w;
        w[0] = pack_16x2<F16>(v[0], v[1]);
        w[1] = pack_16x2<F16>(v[2], v[3]);
        *reinterpret_cast<att_u32x2 *>(optr + 8 * q) = w;
    }
}

// ---------------------------------------------------------------------------------------------
// The same arithmetic with two groups of wavefronts taking turns at the two pipes of a SIMD.
//
// A workgroup of 8 wavefronts (two per SIMD) owns 256 row slots that share one key/value head; wavefronts 0-3 are group
// A, 4-7 group B, so each SIMD holds one wavefront of each group.  Per key tile a wavefront has an MFMA half -- the
// product P_{t-1} V_{t-1} of the tile before, then the scores S_t = K_t Q^T -- and a vector half -- the softmax step
// of tile t (scale, mask, maximum, exponentials, sums, rescale of o, weights rounded to 16 bits).  The two groups run
// these halves in opposite phase, with a workgroup barrier between half-slots:
//     half-slot 2t      A: MFMA half t          B: vector half t - 1
//     half-slot 2t + 1  A: vector half t        B: MFMA half t
// so the matrix pipe and the vector ALU of a SIMD are both busy all the time instead of whenever two independent
// workgroups happen to be out of phase.  K_t is read in half-slots 2t and 2t + 1, V_t in 2t + 2 and 2t + 3; tile t lives
// in slot t % RING of a ring of (K, V) pairs that direct global->LDS loads fill RING - 2 tiles ahead.  A row's
// arithmetic is exactly that of attention_kernel (the order of its operations is unchanged), so are its bits.
template <bool CAUSAL, int RING, bool F16>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2)))
void attention_pingpong_kernel(const AttnParams p) {
    static_assert(RING == 3 || RING == 4, "the prologue and the load counting below are written for these depths");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char *const k_lds = smem;                            // [RING][64 keys][256 B], swizzled as in attention_kernel
    unsigned char *const v_lds = smem + RING * ATT_TILE_BYTES;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);    // 0..7
    const int group = wave >> 2;
    const int li = lane & 31, lg = lane >> 5;
    int qb, by, seq;
    int split_unused, base_unused;
    const int R = 2 * p.rows;                                     // queries per head and workgroup: 256 / pack
    if (!attention_work_item(p, R, lane, qb, by, seq, split_unused, base_unused)) return;      // uniform; launched with n_splits == 1 only

    const int q0 = clampi(p.cu_q[seq], 0, p.total_q), q1 = clampi(p.cu_q[seq + 1], q0, p.total_q);
    const int k0 = clampi(p.cu_k[seq], 0, p.total_k), k1 = clampi(p.cu_k[seq + 1], k0, p.total_k);
    const int Lq = q1 - q0, Lk = k1 - k0;
    if (qb < 0 || qb * R >= Lq) return;                                     // uniform: nothing of this sequence in the block
    const int shift = Lk - Lq;
    const int slot = wave * 32 + li;
    const int head = by * p.pack + slot / R;
    const int hk = (by * p.pack) / p.group;

    const int q_last = min(Lq - 1, qb * R + R - 1);
    const int lim_block = CAUSAL ? min(Lk - 1, q_last + shift) : Lk - 1;
    const int n_tiles = lim_block >= 0 ? min(p.max_tiles, lim_block / ATT_KV + 1) : 0;   // keys past max_seqlen_k are left out

    const int qrow = qb * R + slot % R;
    const int qpos = min(qrow, Lq - 1);
    const int lim = CAUSAL ? min(Lk - 1, qpos + shift) : Lk - 1;
    const int wave_first = qb * R + (wave * 32) % R;
    const int wave_lim = CAUSAL ? min(Lk - 1, min(Lq - 1, wave_first + min(R, 32) - 1) + shift) : Lk - 1;
    const int wave_tiles = (wave_first < Lq && wave_lim >= 0) ? wave_lim / ATT_KV + 1 : 0;
    const int wave_full = CAUSAL ? min(Lk - 1, min(Lq - 1, wave_first) + shift) : Lk - 1;

    bf16x8 bq[ATT_D / 16];
    {
        const uint16_t *qptr = p.Q + (int64_t)(q0 + qpos) * p.q_stride + (int64_t)head * ATT_D + lg * 8;
#pragma unroll
        for (int ks = 0; ks < ATT_D / 16; ++ks) bq[ks] = *reinterpret_cast<const bf16x8 *>(qptr + ks * 16);
        // A use the compiler can see: it waits for these loads here, once, and not later among the direct loads whose
        // counter values it does not know.
#pragma unroll
        for (int ks = 0; ks < ATT_D / 16; ++ks) asm volatile("" ::"v"(bq[ks]));
    }

    f32x16 o[ATT_D / 32];
#pragma unroll
    for (int db = 0; db < ATT_D / 32; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[db][r] = 0.0f;
    float m = -INFINITY, l = 0.0f;

    if (n_tiles == 0) {                                           // uniform: no query of the block sees a key
        if (qrow < Lq) {
            uint16_t *optr = p.O + (int64_t)(q0 + qrow) * p.o_stride + (int64_t)head * ATT_D + lg * 64;
#pragma unroll
            for (int i = 0; i < 8; ++i) *reinterpret_cast<att_u32x4 *>(optr + 8 * i) = att_u32x4{0, 0, 0, 0};
        }
        return;
    }

    // Tile loader: wavefront w fills key rows 8 w .. 8 w + 7 of a tile with 2 direct loads for K and 2 for V.
    const int ld_pos = lane & 15, ld_sub = lane >> 4;
    const uint16_t *kbase = p.K + (int64_t)k0 * p.k_stride + (int64_t)hk * ATT_D;
    const uint16_t *vbase = p.V + (int64_t)k0 * p.v_stride + (int64_t)hk * ATT_D;
    unsigned k_ld[2], v_ld[2];                                   // minus the instruction offset 1024 i, which the load adds back
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const unsigned r = 8 * wave + 4 * i + ld_sub;
        k_ld[i] = (r * (unsigned)p.k_stride + ((ld_pos ^ (r & 15)) << 3)) * 2u - 1024u * i;
        v_ld[i] = (r * (unsigned)p.v_stride + ((ld_pos ^ ((r & 3) << 2)) << 3)) * 2u - 1024u * i;
    }
    const unsigned smem_lds = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;
    const unsigned k_m0 = smem_lds + wave * 2048;
    const unsigned v_m0 = smem_lds + RING * ATT_TILE_BYTES + wave * 2048;
    constexpr int LOADS_PER_TILE = 4;                             // per wavefront: these and nothing else count in vmcnt inside the loop
    auto fetch = [&](int t) __attribute__((always_inline)) {      // tile t -> ring slot t % RING
        const int off = (t % RING) * ATT_TILE_BYTES;
        const char *kt = uniform_pointer(reinterpret_cast<const char *>(kbase + (int64_t)t * ATT_KV * p.k_stride));
        const char *vt = uniform_pointer(reinterpret_cast<const char *>(vbase + (int64_t)t * ATT_KV * p.v_stride));
        const unsigned km = __builtin_amdgcn_readfirstlane(k_m0 + off), vm = __builtin_amdgcn_readfirstlane(v_m0 + off);
        if (__builtin_expect(t * ATT_KV + ATT_KV <= Lk, 1)) {      // uniform: the whole tile lies inside the sequence
            load_16B_per_lane_to_lds<0, true>(kt, k_ld[0], km);
            load_16B_per_lane_to_lds<1024, false>(kt, k_ld[1], km);
            load_16B_per_lane_to_lds<0, true>(vt, v_ld[0], vm);
            load_16B_per_lane_to_lds<1024, false>(vt, v_ld[1], vm);
        } else {
            const int last = Lk - 1 - t * ATT_KV;                  // >= 0: the tile holds at least one key
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const unsigned r = 8 * wave + 4 * i + ld_sub;
                const unsigned rg = min((int)r, last);           // row fetched; it still lands in row r's place
                load_16B_per_lane_to_lds<0, true>(kt, (rg * (unsigned)p.k_stride + ((ld_pos ^ (r & 15)) << 3)) * 2u, km + 1024 * i);
                load_16B_per_lane_to_lds<0, true>(vt, (rg * (unsigned)p.v_stride + ((ld_pos ^ ((r & 3) << 2)) << 3)) * 2u, vm + 1024 * i);
            }
        }
    };

    const int k_rd = li * 256 + ((lg ^ (li & 15)) << 4);         // ^ (ks << 5), + kb * 8192: ((2 ks + lg) ^ (li & 15)) << 4
    const int l16 = lane & 15, e = l16 >> 2;
    int v_rd[ATT_D / 32];
#pragma unroll
    for (int db = 0; db < ATT_D / 32; ++db) {
        const int col = db * 32 + ((lane >> 4) & 1) * 16 + (l16 & 3) * 4;
        v_rd[db] = (4 * lg + e) * 256 + ((((col >> 3) ^ (e << 2))) << 4) + ((col >> 2) & 1) * 8;
    }

    f32x16 s[2];                                                  // S_t between the two halves of tile t
    bf16x8 pw[4];                                                 // P_t^T rounded to bf16, from the vector half of t to the MFMA half of t + 1

    // MFMA half of tile t: o += V_{t-1}^T P_{t-1}^T, then S_t = K_t Q^T.  The fragments of a group of MFMAs are read
    // while earlier groups are multiplied, and nothing is allowed to move across the groups, which bounds the fragment
    // registers in flight (the register budget is 256 per lane: two wavefronts per SIMD).  Product: 4 groups of 4 MFMAs
    // (one k-step each), fragments read two groups ahead; scores: 8 groups of 2 MFMAs, fragments read three groups
    // ahead, the first ones already during the product.  (Reading the very first fragments before the barrier that
    // opens the half, which the residency of the tiles would allow, was tried and did not pay.)
    typedef union { att_v4i16 h2[2]; bf16x8 v; } vfrag;
    vfrag vf[2][ATT_D / 32];
    bf16x8 kf[4][2];
    auto read_v = [&](vfrag (&f)[ATT_D / 32], int t, int st) __attribute__((always_inline)) {
        const unsigned char *vt = v_lds + ((t + RING - 1) % RING) * ATT_TILE_BYTES;      // V_{t-1}
        const int kb = st >> 1, h = st & 1;
#pragma unroll
        for (int db = 0; db < ATT_D / 32; ++db)
#pragma unroll
            for (int hh = 0; hh < 2; ++hh)
                f[db].h2[hh] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) att_v4i16 *)(vt + (32 * kb + 16 * h + 8 * hh) * 256 + v_rd[db]));
    };
    auto read_k = [&](bf16x8 (&f)[2], int k_rd_here, int ks) __attribute__((always_inline)) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) f[kb] = *reinterpret_cast<const bf16x8 *>(k_lds + kb * 8192 + (k_rd_here ^ (ks << 5)));
    };
    auto k_base = [&](int t) __attribute__((always_inline)) {
        int k_rd_here = k_rd + (t % RING) * ATT_TILE_BYTES;      // the tile offset leaves the bits of the swizzle alone
        asm volatile("" : "+v"(k_rd_here));                       // per-step addresses are formed where they are used, not kept
        return k_rd_here;
    };
    auto mfma_prefetch = [&](int t) __attribute__((always_inline)) {
        const bool do_product = t >= 1 && t - 1 < wave_tiles, do_scores = t < wave_tiles;
        if (do_product) {
            read_v(vf[0], t, 0);
            read_v(vf[1], t, 1);
        } else if (do_scores) {
            const int kr = k_base(t);
            read_k(kf[0], kr, 0);
            read_k(kf[1], kr, 1);
            read_k(kf[2], kr, 2);
        }
    };
    auto mfma_half = [&](int t) __attribute__((always_inline)) {
        const bool do_product = t >= 1 && t - 1 < wave_tiles, do_scores = t < wave_tiles;
        const int kr = k_base(t);
        mfma_prefetch(t);
        if (do_product) {
#pragma unroll
            for (int st = 0; st < 4; ++st) {
#pragma unroll
                for (int db = 0; db < ATT_D / 32; ++db)
                    o[db] = mfma_32x32x16<F16>(vf[st & 1][db].v, pw[st], o[db]);
                if (st + 2 < 4) read_v(vf[st & 1], t, st + 2);
                if (st >= 1 && do_scores) read_k(kf[st - 1], kr, st - 1);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        if (do_scores) {
            const f32x16 zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
            for (int ks = 0; ks < ATT_D / 16; ++ks) {
                if (ks + 3 < ATT_D / 16) read_k(kf[(ks + 3) & 3], kr, ks + 3);
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
                    s[kb] = mfma_32x32x16<F16>(kf[ks & 3][kb], bq[ks], ks == 0 ? zero : s[kb]);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };

    // Vector half of tile t: the softmax step on S_t; o is rescaled here (it holds everything up to tile t - 1).
    auto vector_half = [&](int t) __attribute__((always_inline)) {
        if (t < 0 || t >= wave_tiles) return;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) s[kb][r] = s[kb][r] * p.c;
        if (t * ATT_KV + ATT_KV - 1 > wave_full) {                // uniform: some row of the wavefront does not see the whole tile
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = t * ATT_KV + kb * 32 + 8 * (r >> 2) + 4 * lg + (r & 3);
                    if (key > lim) s[kb][r] = -INFINITY;
                }
        }
        float tmax = s[0][0];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) tmax = fmaxf(tmax, s[kb][r]);
        {
            float a, b;
            both_halves(tmax, a, b);
            tmax = fmaxf(a, b);                                   // with the other half of this query's keys
        }
        const float m_new = fmaxf(m, tmax);
        const float m_use = (m_new == -INFINITY) ? 0.0f : m_new;   // a query that has seen no key yet
        const float alpha = __builtin_amdgcn_exp2f(m - m_use);
        if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {     // uniform: o * 1 is o, so skipping changes no bit
#pragma unroll
            for (int db = 0; db < ATT_D / 32; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) o[db][r] = o[db][r] * alpha;
        }
        // Weights in key order, eight at a time: summed in fp32 and rounded to 16 bits as they are formed, so that only a
        // few of them are in registers at once (k-step st of the product takes elements 8 st .. 8 st + 7).
        float psum = 0.0f;
#pragma unroll
        for (int st = 0; st < 4; ++st) {
            union { uint32_t u[4]; bf16x8 v; } pb;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float p0 = __builtin_amdgcn_exp2f(s[st >> 1][8 * (st & 1) + 2 * i] - m_use);
                const float p1 = __builtin_amdgcn_exp2f(s[st >> 1][8 * (st & 1) + 2 * i + 1] - m_use);
                psum = psum + p0;
                psum = psum + p1;
                pb.u[i] = pack_16x2<F16>(p0, p1);
            }
            pw[st] = pb.v;
            __builtin_amdgcn_sched_barrier(0);
        }
        {
            float a, b;
            both_halves(psum, a, b);
            psum = a + b;                                         // lower half's sum + upper half's sum, in both lanes
        }
        l = l * alpha + psum;
        m = m_new;
    };

    // Every wavefront of the workgroup passes the same barriers: 1 + 2 n_tiles + 1, whatever its own number of tiles.
    // The two groups run separate copies of the loop (one branch at the top, none inside), which differ only in which
    // half comes first.
    fetch(0);
    if (RING > 3 && n_tiles > 1) fetch(1);
    if (RING > 3 && n_tiles > 1) asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(LOADS_PER_TILE) : "memory");
    else asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
    // End of iteration t: tile t + 1 must have landed before half-slot 2t + 2; tiles t + 2 .. t + RING - 2 may still be
    // on their way.
    auto end_of_iteration = [&](int t) __attribute__((always_inline)) {
        if (RING > 3 && t + 2 < n_tiles) asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"((RING - 3) * LOADS_PER_TILE) : "memory");
        else asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
    };
    if (group == 0) {
        for (int t = 0; t < n_tiles; ++t) {
            // The slot of tile t - 2 was last read in half-slot 2t - 1: free since the barrier that ended it.
            if (t + RING - 2 < n_tiles) fetch(t + RING - 2);
            mfma_half(t);
            asm volatile("s_barrier" ::: "memory");
            vector_half(t);
            end_of_iteration(t);
        }
        mfma_half(n_tiles);                                       // the product of the last tile (no scores: n_tiles >= wave_tiles)
        asm volatile("s_barrier" ::: "memory");
    } else {
        for (int t = 0; t < n_tiles; ++t) {
            if (t + RING - 2 < n_tiles) fetch(t + RING - 2);
            vector_half(t - 1);
            asm volatile("s_barrier" ::: "memory");
            mfma_half(t);
            end_of_iteration(t);
        }
        vector_half(n_tiles - 1);
        asm volatile("s_barrier" ::: "memory");
        mfma_half(n_tiles);
    }

    if (qrow < Lq) {
        uint16_t *optr = p.O + (int64_t)(q0 + qrow) * p.o_stride + (int64_t)head * ATT_D + 4 * lg;
#pragma unroll
        for (int db = 0; db < ATT_D / 32; ++db)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float v[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) v[i] = (l > 0.0f) ? o[db][4 * q + i] / l : 0.0f;
                att_u32x2 w;
                w[0] = pack_16x2<F16>(v[0], v[1]);
                w[1] = pack_16x2<F16>(v[2], v[3]);
                *reinterpret_cast<att_u32x2 *>(optr + db * 32 + 8 * q) = w;
            }
    }
}

static std::atomic<int> g_attention_variant{0};
int set_attention_variant(int v) {
    if (v < 0 || v > 2) return -1;
    return g_attention_variant.exchange(v);
}

template <class Kernel>
static hipError_t launch_with_lds(Kernel kernel, std::atomic<unsigned> &done, dim3 grid, dim3 block, int lds, const AttnParams &p,
                                  hipStream_t s) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 32) dev = 32;      // 32: not remembered, set every time
    if (dev >= 32 || !((done.load(std::memory_order_relaxed) >> dev) & 1u)) {  // bit d: the attribute is set on device d
        hipError_t e = hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
        if (dev < 32) done.fetch_or(1u << dev, std::memory_order_relaxed);
    }
    hipLaunchKernelGGL(kernel, grid, block, lds, s, p);
    return hipGetLastError();
}

// How a call is cut into work items: a pure function of the host-side arguments, shared by the launcher and by the
// workspace size the caller is told.
struct AttnPlan {
    int pack, rows;          // query heads per workgroup, queries per head and workgroup
    bool pingpong;
    int ny;                  // head groups
    int64_t nb;              // bound on the query blocks of the call (block ids 0 .. nb - 1)
    int64_t items;           // (block id, head group) pairs: a bound on the workgroups that find work, per split
    int chunk;               // block ids per run (runs are dealt to the XCDs in turn)
    int64_t nchunks;
    int splits_max;          // splits a sequence of max_seqlen_k keys has
    int n_splits;            // 1: every workgroup walks all its tiles; else one workgroup per split, then a merge kernel
    size_t state_bytes;      // workspace: fold scratch (one state per item of a launch) or the states of all splits
    int64_t chunks_per_launch;   // walking form: chunks (of block ids) per launch, so that a launch's items fit the capped scratch
};

// The scratch area never exceeds this many states (68 KiB each: 306 MiB; 16384 queries of 32 heads over 8 are 4104
// items and still go in one launch).  A call with more items that fold as they walk is launched in equal pieces of at
// most this many, one after the other on the stream, all using the same area; the form with one workgroup per split
// is only chosen when all its states fit.
constexpr int64_t ATT_MAX_STATES = 4608;

// total_q: tokens in Q (or a bound on them); workspace_bytes: what the caller brought (SIZE_MAX: as much as is wanted).
static AttnPlan plan_attention(int batch, int64_t total_q, int max_seqlen_k, int heads_q, int heads_kv, int variant, size_t workspace_bytes) {
    AttnPlan pl;
    const int group = heads_q / heads_kv;
    pl.pack = (group <= ATT_BQ && (group & (group - 1)) == 0) ? group : 1;
    pl.rows = ATT_BQ / pl.pack;
    pl.ny = heads_q / pl.pack;
    pl.splits_max = max_seqlen_k > 0 ? (max_seqlen_k + ATT_SPLIT * ATT_KV - 1) / (ATT_SPLIT * ATT_KV) : 1;
    // The kernel whose wavefront groups take turns keeps one state per workgroup in two groups of wavefronts and has no
    // fold: it serves sequences of one split (where it is a differently scheduled cross-check of the other kernel).
    pl.pingpong = (variant == 2) && pl.splits_max == 1;
    const int rows = pl.pingpong ? 2 * pl.rows : pl.rows;
    pl.nb = total_q / rows + batch;
    pl.items = pl.nb * pl.ny;
    const size_t state = ATT_STATE_FLOATS * sizeof(float);
    // Few items and long sequences (decode steps on long contexts, alone or beside a chunk of a prefill): one
    // workgroup per split, all at once, then the fold in a second kernel.  Same bits as one workgroup walking the
    // splits, so the choice is free; below two workgroups per compute unit the parallel form wins -- if the caller's
    // workspace holds its states (sized from a bound on total_q it may not; walking needs less and always fits).
    pl.n_splits = (pl.splits_max > 1 && pl.items < 512 && pl.items * pl.splits_max <= ATT_MAX_STATES &&
                   (size_t)pl.items * pl.splits_max * state <= workspace_bytes) ? pl.splits_max : 1;
    // Enough runs to keep every XCD busy (64 or more where the call has that many blocks), chunks of at most 128 blocks.
    const int64_t spread = (pl.items * pl.n_splits + 63) / 64;
    pl.chunk = (int)std::max<int64_t>(1, std::min<int64_t>(spread, std::min<int64_t>(128, pl.nb)));   // no chunk longer than the call: its idle
                                                                  // workgroups would pair the busy ones up on half the compute units
    pl.nchunks = (pl.nb + pl.chunk - 1) / pl.chunk;
    pl.chunks_per_launch = pl.nchunks;
    if (pl.splits_max > 1 && pl.n_splits == 1) {
        const int64_t most = std::max<int64_t>(1, std::min<int64_t>(pl.nchunks, ATT_MAX_STATES / ((int64_t)pl.chunk * pl.ny)));
        const int64_t pieces = (pl.nchunks + most - 1) / most;
        pl.chunks_per_launch = (pl.nchunks + pieces - 1) / pieces;
    }
    const int64_t launch_items = std::min<int64_t>(pl.items, pl.chunks_per_launch * pl.chunk * pl.ny);
    pl.state_bytes = pl.splits_max > 1 ? (size_t)(pl.n_splits > 1 ? pl.items * pl.n_splits : launch_items) * state : 0;
    return pl;
}

// From the arguments a caller has before the call: batch x max_seqlen_q bounds total_q.
size_t attention_workspace(int batch, int max_seqlen_q, int max_seqlen_k, int heads_q, int heads_kv) {
    if (batch <= 0 || max_seqlen_q <= 0 || heads_q <= 0 || heads_kv <= 0 || heads_q % heads_kv) return 0;
    // the variant switch may only move a call to the other kernel where no workspace is involved, so it does not matter here
    return plan_attention(batch, (int64_t)batch * max_seqlen_q, max_seqlen_k, heads_q, heads_kv, 0, SIZE_MAX).state_bytes;
}

template <bool F16>
static hipError_t launch_of(const AttnArgs &a, AttnParams p, const AttnPlan &pl, hipStream_t s) {
    static std::atomic<unsigned> done[4] = {{0}, {0}, {0}, {0}};     // one set per operand format
    hipError_t e = hipSuccess;
    // Late chunks first, as inside a launch (under a causal mask they are the long ones).
    for (int64_t hi = pl.nchunks; hi > 0 && e == hipSuccess; hi -= pl.chunks_per_launch) {
        p.chunk_hi = (int)hi;
        p.chunk_lo = (int)std::max<int64_t>(0, hi - pl.chunks_per_launch);
        const int64_t runs = (int64_t)(p.chunk_hi - p.chunk_lo) * pl.ny * pl.n_splits;   // (chunk of block ids, head group, split) triples, dealt to the 8 XCDs in turn
        const dim3 grid((unsigned)((runs + 7) / 8 * 8 * pl.chunk));
        if (pl.pingpong) {
            constexpr int RING = 4;
            if (a.causal) e = launch_with_lds(attention_pingpong_kernel<true, RING, F16>, done[0], grid, dim3(512), 2 * RING * ATT_TILE_BYTES, p, s);
            else e = launch_with_lds(attention_pingpong_kernel<false, RING, F16>, done[1], grid, dim3(512), 2 * RING * ATT_TILE_BYTES, p, s);
        } else if (a.causal) {
            e = launch_with_lds(attention_kernel<true, F16>, done[2], grid, dim3(256), 4 * ATT_TILE_BYTES, p, s);
        } else {
            e = launch_with_lds(attention_kernel<false, F16>, done[3], grid, dim3(256), 4 * ATT_TILE_BYTES, p, s);
        }
    }
    if (e != hipSuccess || pl.pingpong || pl.n_splits == 1) return e;
    hipLaunchKernelGGL(attention_merge_kernel<F16>, dim3((unsigned)pl.items, ATT_D / 32), dim3(256), 0, s, p);
    return hipGetLastError();
}

hipError_t launch_attention(const AttnArgs &a, hipStream_t s) {
    if (a.batch <= 0 || a.max_seqlen_q <= 0 || a.total_q <= 0) return hipSuccess;
    // Blocks past batch x max_seqlen_q tokens are not launched (the workspace was sized from that bound): with
    // max_seqlen_q below the largest Lq the last queries of the call stay unwritten.
    const int64_t tokens = std::min<int64_t>(a.total_q, (int64_t)a.batch * a.max_seqlen_q);
    const AttnPlan pl = plan_attention(a.batch, tokens, a.max_seqlen_k, a.heads_q, a.heads_kv, g_attention_variant.load(),
                                       a.workspace ? a.workspace_bytes : 0);
    if (pl.state_bytes > (a.workspace ? a.workspace_bytes : 0)) return hipErrorInvalidValue;
    if ((pl.nchunks * pl.ny * pl.n_splits + 8) * pl.chunk > 0x7fffffff || pl.items > 0x7fffffff) return hipErrorInvalidValue;
    AttnParams p;
    p.Q = a.Q; p.K = a.K; p.V = a.V; p.O = a.O;
    p.cu_q = a.cu_q; p.cu_k = a.cu_k;
    p.q_stride = a.q_stride; p.k_stride = a.k_stride; p.v_stride = a.v_stride; p.o_stride = a.o_stride;
    p.total_q = a.total_q; p.total_k = a.total_k;
    p.group = a.heads_q / a.heads_kv;
    p.pack = pl.pack;
    p.rows = pl.rows;
    p.c = a.scale * 1.44269504088896340736f;
    p.ny = pl.ny;
    p.nb = (int)pl.nb;
    p.chunk = pl.chunk;
    p.nchunks = (int)pl.nchunks;
    p.nz = a.batch;
    p.n_splits = pl.n_splits;
    p.max_tiles = pl.splits_max * ATT_SPLIT;
    p.states = reinterpret_cast<float *>(a.workspace);
    return a.dtype == TBIK_F16 ? launch_of<true>(a, p, pl, s) : launch_of<false>(a, p, pl, s);
}

}  // namespace tbik
