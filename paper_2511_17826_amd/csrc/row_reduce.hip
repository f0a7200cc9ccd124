// Batch-invariant row reductions (App. B) in the tree order of App. C: sum, max, log-softmax.
//
// A row is cut into blocks of 2048 leaves (one leaf = one 16-byte chunk = 4 fp32 or 8 bf16 or
// fp16 elements).  One workgroup of 256 threads reduces one block of one row: leaf number
// 256*seg + tid (seg = 0..7) of the block belongs to thread tid, so tree levels 0..5 are lane-pair
// additions, levels 6..7 combine the four wavefronts, levels 8..10 the eight segments; the block
// sums of a row are then combined by the same tree (blocks past the end of the row count as +0).
// Which workgroup handles which (row, block) depends only on the row length, never on M, so a
// row's bits cannot depend on the batch.  Log-softmax keeps the plain two-pass definition:
// exact max first, then TreeSum(exp(x - max)).  Rows of several blocks are handled by one launch in which every
// workgroup keeps its block in registers and the blocks of a row exchange their maxima and sums through memory
// (bounded waits; a row whose wait runs out is redone by a second, normally idle, kernel), so a row is read once.
#include <atomic>

#include "tbik_device.hpp"
#include "tbik_internal.hpp"

namespace tbik {

constexpr int RR_THREADS = 256;
constexpr int RR_SEGS = 8;
constexpr int RR_BLOCK_LEAVES = RR_THREADS * RR_SEGS;   // 2048

enum { MODE_SUM = 0, MODE_MAX = 1, MODE_EXPSUM = 2 };

// XT: the rows' element type, a tbik_dtype (TBIK_F32, TBIK_BF16 or TBIK_F16).
template <int XT> struct Elem {
    static constexpr int EPL = 8;   // elements per leaf
    static constexpr int BYTES = 2;
    __device__ static __forceinline__ void load(const void *row, int64_t leaf, float (&f)[8]) {
        unpack8<XT == TBIK_F16>(reinterpret_cast<const uint4 *>(row)[leaf], f);
    }
};
template <> struct Elem<TBIK_F32> {
    static constexpr int EPL = 4;
    static constexpr int BYTES = 4;
    __device__ static __forceinline__ void load(const void *row, int64_t leaf, float (&f)[8]) {
        const float4 v = reinterpret_cast<const float4 *>(row)[leaf];
        f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
    }
};

// T over n2 (power of two) values of which the first n are stored at p and the rest are +0.
// Executed by one whole wavefront; every lane returns the result.
__device__ __forceinline__ float wave_tree_of_array(const float *p, int n, int n2, int lane) {
    TreeStash<26> st;
    float tot = 0.0f;
    const int nseg = n2 < 64 ? 1 : n2 >> 6;
    for (int seg = 0; seg < nseg; ++seg) {
        const int i = seg * 64 + lane;
        const float v = (i < n) ? p[i] : 0.0f;
        tot = st.push(wave_tree_sum(v), (unsigned)seg);
    }
    return tot;
}

__device__ __forceinline__ float wave_max_of_array(const float *p, int n, int lane) {
    float m = -INFINITY;
    for (int i = lane; i < n; i += 64) m = fmaxf(m, p[i]);
    return wave_max(m);
}

// Combines the per-thread leaf values L[seg] of a block in tree order; result valid in every thread.
__device__ __forceinline__ float block_tree_sum(float (&L)[RR_SEGS], float *lds) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int seg = 0; seg < RR_SEGS; ++seg) {
        const float w = wave_tree_sum(L[seg]);                      // levels 0..5
        if (lane == 0) lds[seg * 4 + wave] = w;
    }
    __syncthreads();
    float t[RR_SEGS];
#pragma unroll
    for (int seg = 0; seg < RR_SEGS; ++seg)                          // levels 6..7: the four wavefronts
        t[seg] = (lds[seg * 4 + 0] + lds[seg * 4 + 1]) + (lds[seg * 4 + 2] + lds[seg * 4 + 3]);
    const float r = ((t[0] + t[1]) + (t[2] + t[3])) + ((t[4] + t[5]) + (t[6] + t[7]));   // levels 8..10
    __syncthreads();
    return r;
}

__device__ __forceinline__ float block_max(float m, float *lds) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    m = wave_max(m);
    if (lane == 0) lds[wave] = m;
    __syncthreads();
    const float r = fmaxf(fmaxf(lds[0], lds[1]), fmaxf(lds[2], lds[3]));
    __syncthreads();
    return r;
}

// Pass over one (row, block): MODE_SUM -> block tree sum; MODE_MAX -> block max;
// MODE_EXPSUM -> block tree sum of exp(x - rowmax), rowmax taken from the block maxima in wsmax.
template <int XT, int MODE>
__global__ __launch_bounds__(RR_THREADS) void row_block_kernel(const void *__restrict__ x, int64_t V, int nb,
                                                               const float *__restrict__ wsmax, float *__restrict__ wsout) {
    __shared__ float lds[RR_SEGS * 4];
    constexpr int EPL = Elem<XT>::EPL;
    // The second pass of log-softmax walks the (row, block) grid backwards: what the first pass read last is
    // what the caches still hold.  Which workgroup handles a (row, block) never affects its arithmetic.
    const int b = (MODE == MODE_EXPSUM) ? (int)(gridDim.x - 1 - blockIdx.x) : (int)blockIdx.x;
    const int row = (MODE == MODE_EXPSUM) ? (int)(gridDim.y - 1 - blockIdx.y) : (int)blockIdx.y;
    const int lane = threadIdx.x & 63;
    const int64_t nleaves = V / EPL;
    const char *rowp = reinterpret_cast<const char *>(x) + (int64_t)row * V * Elem<XT>::BYTES;

    float rowmax = 0.0f;
    if (MODE == MODE_EXPSUM) rowmax = wave_max_of_array(wsmax + (int64_t)row * nb, nb, lane);

    float L[RR_SEGS];
    float mx = -INFINITY;
#pragma unroll
    for (int seg = 0; seg < RR_SEGS; ++seg) {
        const int64_t leaf = (int64_t)b * RR_BLOCK_LEAVES + seg * RR_THREADS + threadIdx.x;
        float acc = 0.0f;
        if (leaf < nleaves) {
            float f[8];
            Elem<XT>::load(rowp, leaf, f);
#pragma unroll
            for (int e = 0; e < EPL; ++e) {
                if (MODE == MODE_SUM) acc = acc + f[e];
                else if (MODE == MODE_MAX) mx = fmaxf(mx, f[e]);
                else acc = acc + expf(f[e] - rowmax);
            }
        }
        L[seg] = acc;
    }
    float r;
    if (MODE == MODE_MAX) r = block_max(mx, lds);
    else r = block_tree_sum(L, lds);
    if (threadIdx.x == 0) wsout[(int64_t)row * nb + b] = r;
}

// out[row] = tree (or max) over the nb block results of the row.  One wavefront per row.
template <int MODE>
__global__ __launch_bounds__(64) void row_finish_kernel(const float *__restrict__ ws, int nb, int nb2, float *__restrict__ out) {
    const int row = blockIdx.x, lane = threadIdx.x;
    const float *p = ws + (int64_t)row * nb;
    const float r = (MODE == MODE_MAX) ? wave_max_of_array(p, nb, lane) : wave_tree_of_array(p, nb, nb2, lane);
    if (lane == 0) out[row] = r;
}

// out[row, i] = (x[row, i] - rowmax) - log(S), S = tree over the row's block sums.
template <int XT>
__global__ __launch_bounds__(RR_THREADS) void logsoftmax_write_kernel(const void *__restrict__ x, int64_t V, int nb, int nb2,
                                                                     const float *__restrict__ wsmax,
                                                                     const float *__restrict__ wssum, float *__restrict__ out) {
    constexpr int EPL = Elem<XT>::EPL;
    const int b = blockIdx.x, row = blockIdx.y;
    const int lane = threadIdx.x & 63;
    const int64_t nleaves = V / EPL;
    const char *rowp = reinterpret_cast<const char *>(x) + (int64_t)row * V * Elem<XT>::BYTES;
    float *orow = out + (int64_t)row * V;
    const float rowmax = wave_max_of_array(wsmax + (int64_t)row * nb, nb, lane);
    const float S = wave_tree_of_array(wssum + (int64_t)row * nb, nb, nb2, lane);
    const float lg = logf(S);
#pragma unroll
    for (int seg = 0; seg < RR_SEGS; ++seg) {
        const int64_t leaf = (int64_t)b * RR_BLOCK_LEAVES + seg * RR_THREADS + threadIdx.x;
        if (leaf < nleaves) {
            float f[8];
            Elem<XT>::load(rowp, leaf, f);
            float o[8];
#pragma unroll
            for (int e = 0; e < EPL; ++e) o[e] = (f[e] - rowmax) - lg;
            float4 *dst = reinterpret_cast<float4 *>(orow + leaf * EPL);
            dst[0] = make_float4(o[0], o[1], o[2], o[3]);
            if (EPL == 8) dst[1] = make_float4(o[4], o[5], o[6], o[7]);
        }
    }
}

// Log-softmax of rows that fit one block: the row stays in registers between the three steps, so it is read once.
// Same leaves, same block tree and the same elementwise arithmetic as the three-kernel path (whose trees over a
// single block value add only +0), hence the same bits.
template <int XT>
__global__ __launch_bounds__(RR_THREADS) void logsoftmax_one_block_kernel(const void *__restrict__ x, int64_t V,
                                                                         float *__restrict__ out) {
    __shared__ float lds[RR_SEGS * 4];
    constexpr int EPL = Elem<XT>::EPL;
    const int row = blockIdx.x;
    const int64_t nleaves = V / EPL;
    const char *rowp = reinterpret_cast<const char *>(x) + (int64_t)row * V * Elem<XT>::BYTES;
    float *orow = out + (int64_t)row * V;

    float f[RR_SEGS][8];
    float mx = -INFINITY;
#pragma unroll
    for (int seg = 0; seg < RR_SEGS; ++seg) {
        const int64_t leaf = seg * RR_THREADS + threadIdx.x;
        if (leaf < nleaves) {
            Elem<XT>::load(rowp, leaf, f[seg]);
#pragma unroll
            for (int e = 0; e < EPL; ++e) mx = fmaxf(mx, f[seg][e]);
        }
    }
    const float rowmax = block_max(mx, lds);
    float L[RR_SEGS];
#pragma unroll
    for (int seg = 0; seg < RR_SEGS; ++seg) {
        const int64_t leaf = seg * RR_THREADS + threadIdx.x;
        float acc = 0.0f;
        if (leaf < nleaves) {
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc = acc + expf(f[seg][e] - rowmax);
        }
        L[seg] = acc;
    }
    const float S = block_tree_sum(L, lds);
    const float lg = logf(S);
#pragma unroll
    for (int seg = 0; seg < RR_SEGS; ++seg) {
        const int64_t leaf = seg * RR_THREADS + threadIdx.x;
        if (leaf < nleaves) {
            float o[8];
#pragma unroll
            for (int e = 0; e < EPL; ++e) o[e] = (f[seg][e] - rowmax) - lg;
            float4 *dst = reinterpret_cast<float4 *>(orow + leaf * EPL);
            dst[0] = make_float4(o[0], o[1], o[2], o[3]);
            if (EPL == 8) dst[1] = make_float4(o[4], o[5], o[6], o[7]);
        }
    }
}

// ---------------------------------------------------------------------------------------------------------
// Log-softmax of rows of 2..RR_MAX_COOP_BLOCKS blocks, one launch, one workgroup per (row, block), block index
// fastest.  Each workgroup loads its block once and keeps it in registers; the blocks of a row publish their
// maxima, wait for each other, publish their sums of exp(x - rowmax), wait again, and write.  The waits are on
// per-row arrival counters.  Workgroups are started in index order and a row's workgroups are consecutive, so
// the ones a workgroup waits for are running or about to be started as long as a row has fewer blocks than
// the device has workgroup slots.  Nothing here relies on that for correctness: every wait is bounded, a
// workgroup whose wait runs out marks its row and leaves, and logsoftmax_redo_kernel recomputes marked rows.
// Arithmetic (leaves, block tree, tree over blocks, expf, logf) is that of the three-kernel path: same bits.
constexpr int RR_MAX_COOP_BLOCKS = 256;
// Per row 64 words (a 256-byte line of its own), of which one is used: the give-up flag.
constexpr int RR_SYNC_WORDS = 64;
constexpr int RR_W_GAVE_UP = 32;
constexpr unsigned RR_NOT_YET = 0xffffffffu;     // a NaN pattern: neither a maximum of finite logits nor a sum of exponentials

// One value per workgroup travels through memory, between workgroups that may sit on different chiplets with
// separate L2 caches.  No cache is flushed or invalidated for it (a release/acquire pair at device scope would write
// back and invalidate a chiplet's whole L2 on every call): the value is written with a read-modify-write atomic of
// device scope, which is performed where all chiplets meet, into a word that starts the call as "not yet", and read
// with device-scope atomic loads.  The word is its own arrival flag: there is no counter to order it against.
// The first wavefront reads the n slots of a row (lane l: slots l, l + 64, ...) until every one holds a value, then
// combines them -- the maximum, or T over the slots padded with +0 to n2 = 2^t (SUM) -- and every thread of the
// workgroup gets the result.  Returns false if the wait ran out (or another workgroup of the row has given up).
constexpr int RR_SLOTS_PER_LANE = 4;             // RR_MAX_COOP_BLOCKS / 64

template <bool SUM>
__device__ __forceinline__ bool gather_row(const float *slots, int n, int n2, const unsigned *gave_up, int limit, int sleep_units,
                                           unsigned *lds_word, float *value) {
    if (threadIdx.x < 64) {
        const int lane = threadIdx.x;
        unsigned u[RR_SLOTS_PER_LANE];
        bool complete = false;
        for (int it = 0; it <= limit; ++it) {
            bool mine = true;
#pragma unroll
            for (int j = 0; j < RR_SLOTS_PER_LANE; ++j) {
                const int i = j * 64 + lane;
                u[j] = 0u;
                if (i < n) {
                    u[j] = __hip_atomic_load(reinterpret_cast<const unsigned *>(slots + i), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    mine = mine && (u[j] != RR_NOT_YET);
                }
            }
            if (__all(mine)) { complete = true; break; }
            if ((it & 15) == 15 && __hip_atomic_load(gave_up, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) break;
            for (int z = 0; z < (sleep_units & 255); ++z) __builtin_amdgcn_s_sleep(8);
        }
        float r;
        if (SUM) {
            TreeStash<2> st;                          // up to 4 groups of 64 slots
            r = 0.0f;
            const int nseg = n2 < 64 ? 1 : n2 >> 6;
#pragma unroll
            for (int j = 0; j < RR_SLOTS_PER_LANE; ++j)
                if (j < nseg) r = st.push(wave_tree_sum((j * 64 + lane < n) ? __uint_as_float(u[j]) : 0.0f), (unsigned)j);
        } else {
            float m = -INFINITY;
#pragma unroll
            for (int j = 0; j < RR_SLOTS_PER_LANE; ++j)
                if (j * 64 + lane < n) m = fmaxf(m, __uint_as_float(u[j]));
            r = wave_max(m);
        }
        if (lane == 0) *lds_word = complete ? __float_as_uint(r) : RR_NOT_YET;
    }
    __syncthreads();
    const unsigned v = *lds_word;
    __syncthreads();
    *value = __uint_as_float(v);
    return v != RR_NOT_YET;
}

// BPW: consecutive blocks of the row per workgroup (1, 2 or 4; the first of them a multiple of BPW, so together they
// are one subtree of the row's tree and their block sums combine by T before anything leaves the workgroup: the same
// additions as in the tree over all blocks).  More blocks per workgroup means more of the row held on the chip per
// resident workgroup and fewer exchanges per byte; nwg = ceil(nb / BPW) workgroups per row.
template <int XT, int BPW>
__global__ __launch_bounds__(RR_THREADS) void logsoftmax_coop_kernel(const void *__restrict__ x, int64_t V, int nwg, int nwg2,
                                                                    float *wsmax, float *wssum, unsigned *sync_words,
                                                                    int wait_limit, int sleep_units, float *__restrict__ out) {
    // sleep_units: bits 8 and up, units of s_sleep 32 before the first look at a row's slots; low byte, units of s_sleep 8
    // between looks.
    __shared__ float lds[RR_SEGS * 4];
    __shared__ unsigned lds_word;
    constexpr int EPL = Elem<XT>::EPL;
    const int row = (int)(blockIdx.x / (unsigned)nwg), w = (int)(blockIdx.x % (unsigned)nwg);
    const int64_t nleaves = V / EPL;
    const char *rowp = reinterpret_cast<const char *>(x) + (int64_t)row * V * Elem<XT>::BYTES;
    float *orow = out + (int64_t)row * V;
    unsigned *words = sync_words + (int64_t)row * RR_SYNC_WORDS, *gave_up = words + RR_W_GAVE_UP;

    float f[BPW][RR_SEGS][8];
    float mx = -INFINITY;
#pragma unroll
    for (int k = 0; k < BPW; ++k)
#pragma unroll
        for (int seg = 0; seg < RR_SEGS; ++seg) {
            const int64_t leaf = (int64_t)(w * BPW + k) * RR_BLOCK_LEAVES + seg * RR_THREADS + threadIdx.x;
            if (leaf < nleaves) {
                Elem<XT>::load(rowp, leaf, f[k][seg]);
#pragma unroll
                for (int e = 0; e < EPL; ++e) mx = fmaxf(mx, f[k][seg][e]);
            }
        }
    // Hand-off: the workgroup puts its block's value into its own slot of the row (one read-modify-write atomic, performed
    // where all chiplets meet; nobody waits for its return) and its first wavefront then reads the row's slots, all of
    // them side by side in its lanes, until none holds the "not yet" pattern the call started them with.  A slot is flag
    // and datum in one word, so a reader that is served an old copy only reads again; the values it ends up with are
    // final, and every workgroup of the row combines the same values in the same order.
    const float bm = block_max(mx, lds);
    if (threadIdx.x == 0)
        __hip_atomic_exchange(reinterpret_cast<unsigned *>(wsmax + (int64_t)row * nwg + w), __float_as_uint(bm), __ATOMIC_RELAXED,
                              __HIP_MEMORY_SCOPE_AGENT);
    for (int z = 0; z < (sleep_units >> 8); ++z) __builtin_amdgcn_s_sleep(32);
    float rowmax;
    if (!gather_row<false>(wsmax + (int64_t)row * nwg, nwg, nwg2, gave_up, wait_limit, sleep_units, &lds_word, &rowmax)) {
        if (threadIdx.x == 0) __hip_atomic_store(gave_up, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return;
    }

    float bsum[BPW];
#pragma unroll
    for (int k = 0; k < BPW; ++k) {
        float L[RR_SEGS];
#pragma unroll
        for (int seg = 0; seg < RR_SEGS; ++seg) {
            const int64_t leaf = (int64_t)(w * BPW + k) * RR_BLOCK_LEAVES + seg * RR_THREADS + threadIdx.x;
            float acc = 0.0f;
            if (leaf < nleaves) {
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc = acc + expf(f[k][seg][e] - rowmax);
            }
            L[seg] = acc;
            __builtin_amdgcn_sched_barrier(0);     // one chunk's exponentials at a time: registers, not latency, bound this kernel
        }
        bsum[k] = block_tree_sum(L, lds);          // a block past the end of the row sums to +0
    }
    const float bs = tree_of(bsum);                // T over this workgroup's blocks
    if (threadIdx.x == 0)
        __hip_atomic_exchange(reinterpret_cast<unsigned *>(wssum + (int64_t)row * nwg + w), __float_as_uint(bs), __ATOMIC_RELAXED,
                              __HIP_MEMORY_SCOPE_AGENT);
    for (int z = 0; z < (sleep_units >> 8); ++z) __builtin_amdgcn_s_sleep(32);
    float S;
    if (!gather_row<true>(wssum + (int64_t)row * nwg, nwg, nwg2, gave_up, wait_limit, sleep_units, &lds_word, &S)) {
        if (threadIdx.x == 0) __hip_atomic_store(gave_up, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return;
    }
    const float lg = logf(S);
#pragma unroll
    for (int k = 0; k < BPW; ++k)
#pragma unroll
        for (int seg = 0; seg < RR_SEGS; ++seg) {
            const int64_t leaf = (int64_t)(w * BPW + k) * RR_BLOCK_LEAVES + seg * RR_THREADS + threadIdx.x;
            if (leaf < nleaves) {
                float o[8];
#pragma unroll
                for (int e = 0; e < EPL; ++e) o[e] = (f[k][seg][e] - rowmax) - lg;
                float4 *dst = reinterpret_cast<float4 *>(orow + leaf * EPL);
                dst[0] = make_float4(o[0], o[1], o[2], o[3]);
                if (EPL == 8) dst[1] = make_float4(o[4], o[5], o[6], o[7]);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
}

// Recomputes the rows that logsoftmax_coop_kernel marked (normally none): one workgroup walks all blocks of its row
// three times.  Same leaves, block trees and tree over blocks, hence the same bits.
template <int XT>
__global__ __launch_bounds__(RR_THREADS) void logsoftmax_redo_kernel(const void *__restrict__ x, int64_t V, int nb, int nb2,
                                                                    const unsigned *__restrict__ sync_words,
                                                                    float *__restrict__ out) {
    __shared__ float lds[RR_SEGS * 4];
    __shared__ float per_block[RR_MAX_COOP_BLOCKS];
    const int row = blockIdx.x;
    if (sync_words[(int64_t)row * RR_SYNC_WORDS + RR_W_GAVE_UP] == 0u) return;   // uniform over the workgroup
    constexpr int EPL = Elem<XT>::EPL;
    const int lane = threadIdx.x & 63;
    const int64_t nleaves = V / EPL;
    const char *rowp = reinterpret_cast<const char *>(x) + (int64_t)row * V * Elem<XT>::BYTES;
    float *orow = out + (int64_t)row * V;

    for (int b = 0; b < nb; ++b) {
        float mx = -INFINITY;
#pragma unroll
        for (int seg = 0; seg < RR_SEGS; ++seg) {
            const int64_t leaf = (int64_t)b * RR_BLOCK_LEAVES + seg * RR_THREADS + threadIdx.x;
            if (leaf < nleaves) {
                float f[8];
                Elem<XT>::load(rowp, leaf, f);
#pragma unroll
                for (int e = 0; e < EPL; ++e) mx = fmaxf(mx, f[e]);
            }
        }
        const float bm = block_max(mx, lds);
        if (threadIdx.x == 0) per_block[b] = bm;
    }
    __syncthreads();
    const float rowmax = wave_max_of_array(per_block, nb, lane);
    __syncthreads();
    for (int b = 0; b < nb; ++b) {
        float L[RR_SEGS];
#pragma unroll
        for (int seg = 0; seg < RR_SEGS; ++seg) {
            const int64_t leaf = (int64_t)b * RR_BLOCK_LEAVES + seg * RR_THREADS + threadIdx.x;
            float acc = 0.0f;
            if (leaf < nleaves) {
                float f[8];
                Elem<XT>::load(rowp, leaf, f);
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc = acc + expf(f[e] - rowmax);
            }
            L[seg] = acc;
        }
        const float bs = block_tree_sum(L, lds);
        if (threadIdx.x == 0) per_block[b] = bs;
    }
    __syncthreads();
    const float S = wave_tree_of_array(per_block, nb, nb2, lane);
    const float lg = logf(S);
    for (int b = 0; b < nb; ++b) {
#pragma unroll
        for (int seg = 0; seg < RR_SEGS; ++seg) {
            const int64_t leaf = (int64_t)b * RR_BLOCK_LEAVES + seg * RR_THREADS + threadIdx.x;
            if (leaf < nleaves) {
                float f[8], o[8];
                Elem<XT>::load(rowp, leaf, f);
#pragma unroll
                for (int e = 0; e < EPL; ++e) o[e] = (f[e] - rowmax) - lg;
                float4 *dst = reinterpret_cast<float4 *>(orow + leaf * EPL);
                dst[0] = make_float4(o[0], o[1], o[2], o[3]);
                if (EPL == 8) dst[1] = make_float4(o[4], o[5], o[6], o[7]);
            }
        }
    }
}

// Before every call: the slots of both hand-offs to "not yet", the rows' flags to zero.
__global__ __launch_bounds__(256) void reset_sync_words_kernel(unsigned *slots_max, unsigned *slots_sum, int64_t nslots,
                                                                unsigned *words, int64_t nwords) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < nslots) {
        slots_max[i] = RR_NOT_YET;
        slots_sum[i] = RR_NOT_YET;
    }
    if (i < nwords) words[i] = 0u;
}

static std::atomic<int> g_wait_limit{1 << 14};   // polls per wait: tens of milliseconds at most
int set_row_wait_limit(int limit) { return g_wait_limit.exchange(limit < 0 ? 0 : limit); }

static int blocks_of(int64_t V, int x_dtype) {
    const int epl = (x_dtype == TBIK_F32) ? 4 : 8;
    const int64_t nleaves = V / epl;
    return (int)((nleaves + RR_BLOCK_LEAVES - 1) / RR_BLOCK_LEAVES);
}

size_t row_reduce_workspace(int M, int64_t V, int x_dtype, int op) {
    if (M <= 0 || V <= 0) return 0;
    const size_t per = (size_t)M * blocks_of(V, x_dtype) * sizeof(float);
    // log-softmax: block maxima, block sums, two arrival counters and one flag per row
    return (op == TBIK_LOGSOFTMAX) ? 2 * per + (size_t)M * RR_SYNC_WORDS * sizeof(unsigned) : per;
}

template <int XT>
static hipError_t run(const void *x, void *out, int op, int M, int64_t V, void *ws, hipStream_t s) {
    const int nb = blocks_of(V, XT);
    int nb2 = 1;
    while (nb2 < nb) nb2 *= 2;
    float *ws0 = reinterpret_cast<float *>(ws);
    float *ws1 = ws0 + (size_t)M * nb;
    float *o = reinterpret_cast<float *>(out);
    // gridDim.y is limited to 65535 rows per launch.
    const int64_t group = 65535;
    for (int64_t m0 = 0; m0 < M; m0 += group) {
        const int mc = (int)((M - m0) < group ? (M - m0) : group);
        const char *xp = reinterpret_cast<const char *>(x) + m0 * V * Elem<XT>::BYTES;
        float *w0 = ws0 + (size_t)m0 * nb, *w1 = ws1 + (size_t)m0 * nb;
        dim3 grid(nb, mc), block(RR_THREADS);
        if (op == TBIK_SUM) {
            hipLaunchKernelGGL((row_block_kernel<XT, MODE_SUM>), grid, block, 0, s, xp, V, nb, (const float *)nullptr, w0);
            hipLaunchKernelGGL((row_finish_kernel<MODE_SUM>), dim3(mc), dim3(64), 0, s, w0, nb, nb2, o + m0);
        } else if (op == TBIK_MAX) {
            hipLaunchKernelGGL((row_block_kernel<XT, MODE_MAX>), grid, block, 0, s, xp, V, nb, (const float *)nullptr, w0);
            hipLaunchKernelGGL((row_finish_kernel<MODE_MAX>), dim3(mc), dim3(64), 0, s, w0, nb, nb2, o + m0);
        } else if (nb == 1) {
            hipLaunchKernelGGL((logsoftmax_one_block_kernel<XT>), dim3(mc), block, 0, s, xp, V, o + m0 * V);
        } else if (nb <= RR_MAX_COOP_BLOCKS && (int64_t)mc * nb <= 0x7fffffff) {
            unsigned *words = reinterpret_cast<unsigned *>(ws1 + (size_t)M * nb) + (size_t)m0 * RR_SYNC_WORDS;
            const int64_t nwords = (int64_t)mc * RR_SYNC_WORDS;
            const int64_t nslots = (int64_t)mc * nb, nreset = nslots > nwords ? nslots : nwords;
            hipLaunchKernelGGL(reset_sync_words_kernel, dim3((unsigned)((nreset + 255) / 256)), dim3(256), 0, s,
                               reinterpret_cast<unsigned *>(w0), reinterpret_cast<unsigned *>(w1), nslots, words, nwords);
            // two blocks per workgroup for fp32 rows once the launch has more workgroups than the device holds at a time
            // (more of the row on the chip per resident workgroup); the choice cannot change a bit
            // Waiting costs the others bandwidth: a wavefront that polls takes issue slots and memory requests from the
            // workgroups that stream.  When the launch fills the device, a workgroup sleeps about 2 us (2 x s_sleep 32)
            // before its first look -- no hand-off completes sooner -- and about 0.5 us between looks (measured at
            // 512 x 151936: 200 us without the first sleep, 171 us with it, 191 us with twice as long; M = 1 loses 3 us
            // with it, so small launches look at once).
            const int sleep_units = (((int64_t)mc * nb >= 256 ? 2 : 0) << 8) | 2;
            const bool two = false;   // measured: 195 -> 282 us at 512 x 151936 (170 registers, three workgroups per compute unit)
            const int nwg = two ? (nb + 1) / 2 : nb, nwg2 = two ? (nb2 + 1) / 2 : nb2;
            if (two)
                hipLaunchKernelGGL((logsoftmax_coop_kernel<XT, (XT == TBIK_F32 ? 2 : 1)>), dim3((unsigned)((int64_t)mc * nwg)), block, 0, s,
                                   xp, V, nwg, nwg2, w0, w1, words, g_wait_limit.load(), sleep_units, o + m0 * V);
            else
                hipLaunchKernelGGL((logsoftmax_coop_kernel<XT, 1>), dim3((unsigned)((int64_t)mc * nwg)), block, 0, s,
                                   xp, V, nwg, nwg2, w0, w1, words, g_wait_limit.load(), sleep_units, o + m0 * V);
            hipLaunchKernelGGL((logsoftmax_redo_kernel<XT>), dim3(mc), block, 0, s, xp, V, nb, nb2,
                               (const unsigned *)words, o + m0 * V);
        } else {
            hipLaunchKernelGGL((row_block_kernel<XT, MODE_MAX>), grid, block, 0, s, xp, V, nb, (const float *)nullptr, w0);
            hipLaunchKernelGGL((row_block_kernel<XT, MODE_EXPSUM>), grid, block, 0, s, xp, V, nb, (const float *)w0, w1);
            hipLaunchKernelGGL((logsoftmax_write_kernel<XT>), grid, block, 0, s, xp, V, nb, nb2, (const float *)w0,
                               (const float *)w1, o + m0 * V);
        }
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_row_reduce(const void *x, int x_dtype, void *out, int op, int M, int64_t V, void *ws, hipStream_t s) {
    if (M <= 0) return hipSuccess;
    if (x_dtype == TBIK_BF16) return run<TBIK_BF16>(x, out, op, M, V, ws, s);
    if (x_dtype == TBIK_F16) return run<TBIK_F16>(x, out, op, M, V, ws, s);
    return run<TBIK_F32>(x, out, op, M, V, ws, s);
}

// ---------------------------------------------------------------------------------------------------------
// Scratch of the library's own for callers that cannot allocate: a fixed array in device memory, one copy per
// GPU, held until the process ends.  In host code the array's name is only a handle for the runtime; the
// address the kernels get is looked up once per device with that device current.
static __device__ __align__(256) unsigned char scratch[TBIK_STATIC_SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
static std::atomic<void *> g_scratch_of_device[MAX_DEVICES];

hipError_t static_scratch(void **ptr) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
    void *p = g_scratch_of_device[dev].load(std::memory_order_acquire);
    if (p == nullptr) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (p == nullptr) return hipErrorInvalidSymbol;
        g_scratch_of_device[dev].store(p, std::memory_order_release);   // two first calls at once look up the same address
    }
    *ptr = p;
    return hipSuccess;
}

hipError_t launch_row_reduce_static(const void *x, int x_dtype, void *out, int op, int M, int64_t V, hipStream_t s) {
    void *ws = nullptr;
    hipError_t e = static_scratch(&ws);
    if (e != hipSuccess) return e;
    if (M <= 0) return hipSuccess;
    if (row_reduce_workspace(M, V, x_dtype, op) > (size_t)TBIK_STATIC_SCRATCH_BYTES) return hipErrorInvalidValue;
    return launch_row_reduce(x, x_dtype, out, op, M, V, ws, s);
}

}  // namespace tbik
