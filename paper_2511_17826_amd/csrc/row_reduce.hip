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
// (bounded waits; a workgroup whose wait runs out finishes its block alone, from memory), so a row is read once.
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
    __device__ static __forceinline__ void unpack(const uint4 &raw, float (&f)[8]) {
        if constexpr (XT == TBIK_F16) {                 // element by element (the conversions are exact either way)
            const unsigned w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
            for (int e = 0; e < 8; ++e)
                f[e] = (float)__builtin_bit_cast(_Float16, (unsigned short)((e & 1) ? w[e >> 1] >> 16 : w[e >> 1] & 0xffffu));
        } else {
            unpack8<false>(raw, f);
        }
    }
};
template <> struct Elem<TBIK_F32> {
    static constexpr int EPL = 4;
    static constexpr int BYTES = 4;
    __device__ static __forceinline__ void load(const void *row, int64_t leaf, float (&f)[8]) {
        const float4 v = reinterpret_cast<const float4 *>(row)[leaf];
        f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
    }
    __device__ static __forceinline__ void unpack(const uint4 &raw, float (&f)[8]) {
        f[0] = __uint_as_float(raw.x); f[1] = __uint_as_float(raw.y); f[2] = __uint_as_float(raw.z); f[3] = __uint_as_float(raw.w);
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

// The same for n2 <= 256 (up to four groups of 64 values), without a loop: the stash stays in registers.
__device__ __forceinline__ float wave_tree_of_256(const float *p, int n, int n2, int lane) {
    TreeStash<2> st;
    float tot = 0.0f;
    const int nseg = n2 < 64 ? 1 : n2 >> 6;
#pragma unroll
    for (int seg = 0; seg < 4; ++seg)
        if (seg < nseg) tot = st.push(wave_tree_sum((seg * 64 + lane < n) ? p[seg * 64 + lane] : 0.0f), (unsigned)seg);
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

// 16 bytes written around the caches (an output that is written once and not read back soon).
__device__ __forceinline__ void stream_store_16B(float4 *dst, float a, float b, float c, float d) {
    typedef float nt_f32x4 __attribute__((ext_vector_type(4)));
    __builtin_nontemporal_store(nt_f32x4{a, b, c, d}, reinterpret_cast<nt_f32x4 *>(dst));
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
            stream_store_16B(dst, o[0], o[1], o[2], o[3]);              // rows this long: written once, around the caches
            if (EPL == 8) stream_store_16B(dst + 1, o[4], o[5], o[6], o[7]);
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
            dst[0] = make_float4(o[0], o[1], o[2], o[3]);             // short rows: ordinary stores (a reader of the whole
            if (EPL == 8) dst[1] = make_float4(o[4], o[5], o[6], o[7]);   // output may follow; streaming gained 4 % here)
        }
    }
}

// What a workgroup does for block b of a row whose hand-off ran out (normally never): it computes the row's maximum
// and the row's sum by itself, walking all blocks of the row twice, and writes its own block.  Same leaves, block
// trees and tree over blocks as the exchange, hence the same bits.  Called by all threads of the workgroup (256, the
// data wavefronts), convergently; per_block holds RR_MAX_COOP_BLOCKS floats and lds RR_SEGS * 4.
template <int XT>
__device__ __forceinline__ void logsoftmax_block_alone(const void *__restrict__ x, int64_t V, int nb, int nb2, int row, int b,
                                                    float *lds, float *per_block, float *__restrict__ out) {
    constexpr int EPL = Elem<XT>::EPL;
    const int lane = threadIdx.x & 63;
    const int64_t nleaves = V / EPL;
    const char *rowp = reinterpret_cast<const char *>(x) + (int64_t)row * V * Elem<XT>::BYTES;
    float *orow = out + (int64_t)row * V;
    __syncthreads();                                                      // per_block and lds may still be in use
    for (int k = 0; k < nb; ++k) {
        float mx = -INFINITY;
#pragma unroll
        for (int seg = 0; seg < RR_SEGS; ++seg) {
            const int64_t leaf = (int64_t)k * RR_BLOCK_LEAVES + seg * RR_THREADS + threadIdx.x;
            if (leaf < nleaves) {
                float f[8];
                Elem<XT>::load(rowp, leaf, f);
#pragma unroll
                for (int e = 0; e < EPL; ++e) mx = fmaxf(mx, f[e]);
            }
        }
        const float bm = block_max(mx, lds);
        if (threadIdx.x == 0) per_block[k] = bm;
    }
    __syncthreads();
    const float rowmax = wave_max_of_array(per_block, nb, lane);
    __syncthreads();
    for (int k = 0; k < nb; ++k) {
        float L[RR_SEGS];
#pragma unroll
        for (int seg = 0; seg < RR_SEGS; ++seg) {
            const int64_t leaf = (int64_t)k * RR_BLOCK_LEAVES + seg * RR_THREADS + threadIdx.x;
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
        if (threadIdx.x == 0) per_block[k] = bs;
    }
    __syncthreads();
    const float S = wave_tree_of_256(per_block, nb, nb2, lane);      // nb <= RR_MAX_COOP_BLOCKS = 256
    const float lg = logf(S);
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
    __syncthreads();
}

// ---------------------------------------------------------------------------------------------------------
// Log-softmax of rows of 2..RR_MAX_COOP_BLOCKS blocks, one launch, one workgroup per (row, block), block index
// fastest.  Each workgroup loads its block once and keeps it in registers; the blocks of a row publish their
// maxima, wait for each other, publish their sums of exp(x - rowmax), wait again, and write.  Workgroups are
// started in index order and a row's workgroups are consecutive, so the ones a workgroup waits for are running or
// about to be started as long as a row has fewer blocks than the device has workgroup slots.  Nothing here relies
// on that for correctness: every wait is bounded, and a workgroup whose wait runs out finishes its block alone
// (logsoftmax_block_alone) after raising the row's flag, which lets the row's other workgroups stop waiting for
// what it will not publish any more; they do the same.
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

// The wavefront's part: lane = 0..63 of the calling wavefront.  Returns the combined value, or the "not yet" pattern
// if the wait ran out.
template <bool SUM>
__device__ __forceinline__ unsigned wave_gather_row(const float *slots, int n, int n2, const unsigned *gave_up, int limit, int sleep_units,
                                                    int lane) {
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
    return complete ? __float_as_uint(r) : RR_NOT_YET;
}

template <bool SUM>
__device__ __forceinline__ bool gather_row(const float *slots, int n, int n2, const unsigned *gave_up, int limit, int sleep_units,
                                           unsigned *lds_word, float *value) {
    if (threadIdx.x < 64) {
        const unsigned r = wave_gather_row<SUM>(slots, n, n2, gave_up, limit, sleep_units, (int)threadIdx.x);
        if (threadIdx.x == 0) *lds_word = r;
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
    __shared__ float per_block[RR_MAX_COOP_BLOCKS];                       // only for a block that has to be finished alone
    constexpr int EPL = Elem<XT>::EPL;
    static_assert(BPW == 1, "a workgroup that finishes alone writes one block");
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
    bool arrived = gather_row<false>(wsmax + (int64_t)row * nwg, nwg, nwg2, gave_up, wait_limit, sleep_units, &lds_word, &rowmax);
    if (arrived) {

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
    arrived = gather_row<true>(wssum + (int64_t)row * nwg, nwg, nwg2, gave_up, wait_limit, sleep_units, &lds_word, &S);
    if (arrived) {
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
                // streaming stores, as in the pipelined kernel (64 x 151936 cold: 26.3 -> 21.2 us)
                stream_store_16B(dst, o[0], o[1], o[2], o[3]);
                if (EPL == 8) stream_store_16B(dst + 1, o[4], o[5], o[6], o[7]);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }   // the sums arrived
    }   // the maxima arrived
    if (!arrived) {                                                       // uniform; the block's registers are free by now
        if (threadIdx.x == 0) __hip_atomic_store(gave_up, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        logsoftmax_block_alone<XT>(x, V, nwg, nwg2, row, w, lds, per_block, out);
    }
}

// ---------------------------------------------------------------------------------------------------------
// The same exchange for launches of more (row, block) items than the device holds workgroups: a fixed number of
// resident workgroups walks the items (item t = row * nb + block; workgroup g takes t = g, g + G, g + 2G, ...) as a
// software pipeline over THREE blocks, two in registers and one parked in LDS.  With one block per workgroup the device alternates between
// everybody loading, everybody waiting and everybody storing, and a workgroup that takes its items one after the
// other waits, at every hand-off, for the slowest of its row.  Here a workgroup's step s is
//     the sum of item s's row and the maximum of item s + 1's row arrive (one wait for both);
//     write item s, start the loads of item s + 3 into the freed registers;
//     sum of exponentials of item s + 1, published;
//     the loads of item s + 3 have landed meanwhile: its maximum, published;
// so a sum is asked for most of a step after it was published and a maximum more than a step after, and a
// workgroup that lags its row by less than that delays nobody.  The first wavefront polls at the start of a step,
// when it has nothing else in flight that its polls would queue behind (a wavefront's memory results come back in
// issue order); the other waits are plain barriers, which do not wait for outstanding loads.
// Every workgroup publishes a block's maximum without waiting for anything of that block or of a later one, so
// with all G workgroups resident no wait is circular; the waits are bounded all the same, and a row whose wait
// runs out is finished alone as above.  Leaves, block tree, tree over blocks and the elementwise arithmetic are
// those of logsoftmax_coop_kernel.
__device__ __forceinline__ void lds_then_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

struct PipeLds {
    float part[RR_SEGS * 4];   // the wavefronts' partial sums of a block
    float max4[4];             // the wavefronts' maxima of a block
    unsigned row_sum;          // T over the block sums of item s's row, or "not yet" if the wait ran out
    unsigned row_max;          // the maximum of item s + 1's row, or "not yet"
};

// All eight loads of a block are issued by every thread in every step -- a leaf past the end of the row re-reads the
// row's last leaf, and a step past the workgroup's last item (real = false) re-reads the first leaf of the tensor;
// such values are never used -- so that the loads sit in straight-line code: the compiler's bookkeeping of
// outstanding loads is then exact and nothing that works on one block waits for another block's loads or stores.
template <int XT>
__device__ __forceinline__ void pipe_load_block(const void *__restrict__ x, int64_t V, unsigned nleaves, int nb, int item, bool real,
                                                uint4 (&raw)[RR_SEGS]) {
    const int row = real ? item / nb : 0;
    const unsigned b = real ? (unsigned)(item - row * nb) : 0u;
    const char *rowp = reinterpret_cast<const char *>(x) + (int64_t)row * V * Elem<XT>::BYTES;     // wave-uniform
#pragma unroll
    for (int seg = 0; seg < RR_SEGS; ++seg) {
        const unsigned leaf = b * RR_BLOCK_LEAVES + seg * RR_THREADS + threadIdx.x;      // a row here has < 2^20 leaves
        const unsigned at = real ? (leaf < nleaves ? leaf : nleaves - 1u) * 16u : 0u;
        raw[seg] = *reinterpret_cast<const uint4 *>(rowp + at);
    }
}

constexpr int RR_PIPE_SLOTS_PER_LANE = 1;         // rows of up to 64 blocks: one slot per lane and hand-off
constexpr int RR_MAX_PIPE_BLOCKS = 64 * RR_PIPE_SLOTS_PER_LANE;

// The first wavefront's wait at the start of a step: the block sums of one row (want_sum) and the block maxima of
// another (want_max), looked at together until both sets are complete.  Results go to LDS; a set that is not
// complete when the looks run out is reported as "not yet" and its row's flag raised.
__device__ __forceinline__ void pipe_gather(bool want_sum, const float *sum_slots, unsigned *sum_gave_up, bool want_max,
                                            const float *max_slots, unsigned *max_gave_up, int n, int n2, int limit, int sleep_units,
                                            int lane, PipeLds *lds) {
    unsigned us[RR_PIPE_SLOTS_PER_LANE], um[RR_PIPE_SLOTS_PER_LANE];
    bool sum_done = !want_sum, max_done = !want_max;
    for (int it = 0; it <= limit; ++it) {
        bool s_ok = true, m_ok = true;
#pragma unroll
        for (int j = 0; j < RR_PIPE_SLOTS_PER_LANE; ++j) {
            const int i = j * 64 + lane;
            us[j] = 0u;
            um[j] = 0u;
            if (i < n) {
                if (!sum_done) {
                    us[j] = __hip_atomic_load(reinterpret_cast<const unsigned *>(sum_slots + i), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    s_ok = s_ok && (us[j] != RR_NOT_YET);
                }
                if (!max_done) {
                    um[j] = __hip_atomic_load(reinterpret_cast<const unsigned *>(max_slots + i), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    m_ok = m_ok && (um[j] != RR_NOT_YET);
                }
            }
        }
        if (!sum_done && __all(s_ok)) {
            sum_done = true;
            TreeStash<2> st;                          // up to 4 groups of 64 slots
            float r = 0.0f;
            const int nseg = n2 < 64 ? 1 : n2 >> 6;
#pragma unroll
            for (int j = 0; j < RR_PIPE_SLOTS_PER_LANE; ++j)
                if (j < nseg) r = st.push(wave_tree_sum((j * 64 + lane < n) ? __uint_as_float(us[j]) : 0.0f), (unsigned)j);
            if (lane == 0) lds->row_sum = __float_as_uint(r);
        }
        if (!max_done && __all(m_ok)) {
            max_done = true;
            float m = -INFINITY;
#pragma unroll
            for (int j = 0; j < RR_PIPE_SLOTS_PER_LANE; ++j)
                if (j * 64 + lane < n) m = fmaxf(m, __uint_as_float(um[j]));
            m = wave_max(m);
            if (lane == 0) lds->row_max = __float_as_uint(m);
        }
        if (sum_done && max_done) return;
        if ((it & 15) == 15) {
            if (!sum_done && __hip_atomic_load(sum_gave_up, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) break;
            if (!max_done && __hip_atomic_load(max_gave_up, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) break;
        }
        for (int z = 0; z < (sleep_units & 255); ++z) __builtin_amdgcn_s_sleep(8);
    }
    if (lane == 0) {
        if (!sum_done) {
            lds->row_sum = RR_NOT_YET;
            __hip_atomic_store(sum_gave_up, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        if (!max_done) {
            lds->row_max = RR_NOT_YET;
            __hip_atomic_store(max_gave_up, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

// One step.  The workgroup's own items are numbered 0..n-1 (item j is global item g + j G) and step s works on items
// s .. s + 3: P holds item s and then item s + 1, Q holds item s + 2 and then item s + 3, parked is this thread's part
// of the block in LDS (leaf seg at parked[seg * RR_THREADS]; nobody else touches it), which holds item s + 1 and
// then item s + 2.
// rowmax: in, the maximum of item s's row as bits ("not yet" if that wait ran out); out, the same for item s + 1.
template <int XT>
__device__ __forceinline__ void pipe_step(const void *__restrict__ x, int64_t V, unsigned nleaves, int nb, int nb2, int g, int G,
                                          int s, int n, uint4 (&P)[RR_SEGS], uint4 (&Q)[RR_SEGS], uint4 *parked, unsigned &rowmax,
                                          float *wsmax, float *wssum, unsigned *sync_words, int wait_limit, int sleep_units,
                                          PipeLds *lds, float *per_block, float *__restrict__ out) {
    constexpr int EPL = Elem<XT>::EPL;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const bool has0 = s >= 0 && s < n, has1 = s + 1 >= 0 && s + 1 < n, has2 = s + 2 >= 0 && s + 2 < n, has3 = s + 3 < n;
    const int item0 = g + s * G, item1 = g + (s + 1) * G, item3 = g + (s + 3) * G;     // the host keeps items below 2^31
    const bool want_sum = has0 && rowmax != RR_NOT_YET;
    if (wave == 0 && (want_sum || has1)) {
        const int64_t row0 = want_sum ? item0 / nb : 0, row1 = has1 ? item1 / nb : 0;
        pipe_gather(want_sum, wssum + row0 * nb, sync_words + row0 * RR_SYNC_WORDS + RR_W_GAVE_UP, has1, wsmax + row1 * nb,
                    sync_words + row1 * RR_SYNC_WORDS + RR_W_GAVE_UP, nb, nb2, wait_limit, sleep_units, lane, lds);
    }
    lds_then_barrier();                                                   // 0: row_sum (item s) and row_max (item s + 1) are in LDS
    const unsigned us = lds->row_sum, um = lds->row_max;
    if (has0 && !(want_sum && us != RR_NOT_YET)) {                        // uniform: a wait for this item's row ran out
        const int row = item0 / nb;
        logsoftmax_block_alone<XT>(x, V, nb, nb2, row, item0 - row * nb, lds->part, per_block, out);
    }
    if (want_sum && us != RR_NOT_YET) {                                   // uniform
        const int row = item0 / nb;
        const unsigned leaf0 = (unsigned)(item0 - row * nb) * RR_BLOCK_LEAVES + threadIdx.x;
        const float rm = __uint_as_float(rowmax), lg = logf(__uint_as_float(us));
        char *orow = reinterpret_cast<char *>(out + (int64_t)row * V);    // wave-uniform
#pragma unroll
        for (int seg = 0; seg < RR_SEGS; ++seg) {
            const unsigned leaf = leaf0 + seg * RR_THREADS;
            float f[8], o[8];
            Elem<XT>::unpack(P[seg], f);
#pragma unroll
            for (int e = 0; e < EPL; ++e) o[e] = (f[e] - rm) - lg;
            if (leaf < nleaves) {
                float4 *dst = reinterpret_cast<float4 *>(orow + leaf * (unsigned)(EPL * 4));
                // Streaming stores: the output of a launch this size is written once and is larger than what the caches
                // would keep for a reader (512 x 151936: 136 -> 121 us; the same hint on the loads gains nothing more).
                stream_store_16B(dst, o[0], o[1], o[2], o[3]);
                if (EPL == 8) stream_store_16B(dst + 1, o[4], o[5], o[6], o[7]);
            }
        }
    }
    if (has1) {
#pragma unroll
        for (int seg = 0; seg < RR_SEGS; ++seg) P[seg] = parked[seg * RR_THREADS];
    }
    if (has2) {
#pragma unroll
        for (int seg = 0; seg < RR_SEGS; ++seg) parked[seg * RR_THREADS] = Q[seg];
    }
    pipe_load_block<XT>(x, V, nleaves, nb, item3, has3, Q);
    if (has1) {
        rowmax = um;
        const int row = item1 / nb;
        const unsigned leaf0 = (unsigned)(item1 - row * nb) * RR_BLOCK_LEAVES + threadIdx.x;
        const float rm = __uint_as_float(um);                             // "not yet": the sums are not used
#pragma unroll
        for (int seg = 0; seg < RR_SEGS; ++seg) {
            float f[8];
            Elem<XT>::unpack(P[seg], f);
            float acc = 0.0f;
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc = acc + expf(f[e] - rm);
            const float w = wave_tree_sum(leaf0 + seg * RR_THREADS < nleaves ? acc : 0.0f);   // levels 0..5
            if (lane == 0) lds->part[seg * 4 + wave] = w;
        }
    }
    lds_then_barrier();                                                   // 1: the partial sums of item s + 1 are in LDS
    if (wave == 0 && has1 && um != RR_NOT_YET) {
        float t[RR_SEGS];
#pragma unroll
        for (int seg = 0; seg < RR_SEGS; ++seg)                           // levels 6..7: the four wavefronts
            t[seg] = (lds->part[seg * 4 + 0] + lds->part[seg * 4 + 1]) + (lds->part[seg * 4 + 2] + lds->part[seg * 4 + 3]);
        const float bs = ((t[0] + t[1]) + (t[2] + t[3])) + ((t[4] + t[5]) + (t[6] + t[7]));   // levels 8..10
        if (lane == 0)
            __hip_atomic_exchange(reinterpret_cast<unsigned *>(wssum + item1), __float_as_uint(bs), __ATOMIC_RELAXED,
                                  __HIP_MEMORY_SCOPE_AGENT);
    }
    {                                                                     // (of no consequence if there is no item s + 3)
        const int row = item3 / nb;
        const unsigned leaf0 = (unsigned)(item3 - row * nb) * RR_BLOCK_LEAVES + threadIdx.x;
        float mx = -INFINITY;
#pragma unroll
        for (int seg = 0; seg < RR_SEGS; ++seg) {
            float f[8];
            Elem<XT>::unpack(Q[seg], f);
            float m = f[0];
#pragma unroll
            for (int e = 1; e < EPL; ++e) m = fmaxf(m, f[e]);
            mx = fmaxf(mx, leaf0 + seg * RR_THREADS < nleaves ? m : -INFINITY);
        }
        mx = wave_max(mx);
        if (lane == 0) lds->max4[wave] = mx;
    }
    lds_then_barrier();                                                   // 2: the four maxima of item s + 3 are in LDS
    if (wave == 0 && has3) {
        const float bm = fmaxf(fmaxf(lds->max4[0], lds->max4[1]), fmaxf(lds->max4[2], lds->max4[3]));
        if (lane == 0)
            __hip_atomic_exchange(reinterpret_cast<unsigned *>(wsmax + item3), __float_as_uint(bm), __ATOMIC_RELAXED,
                                  __HIP_MEMORY_SCOPE_AGENT);
    }
}

template <int XT>
__global__ __launch_bounds__(RR_THREADS) __attribute__((amdgpu_waves_per_eu(4, 4))) void logsoftmax_pipe_kernel(
    const void *__restrict__ x, int64_t V, int nb, int nb2, int64_t items, float *wsmax, float *wssum, unsigned *sync_words,
    int wait_limit, int sleep_units, float *__restrict__ out) {
    __shared__ PipeLds lds;
    __shared__ uint4 parked[RR_SEGS * RR_THREADS];                        // one block, each thread its own eight leaves
    __shared__ float per_block[RR_MAX_PIPE_BLOCKS];                       // only for a block that has to be finished alone
    const int G = (int)gridDim.x, g = (int)blockIdx.x;
    const int n = g < items ? (int)((items - g + G - 1) / G) : 0;        // this workgroup's items
    const unsigned nleaves = (unsigned)(V / Elem<XT>::EPL);
    uint4 P[RR_SEGS], Q[RR_SEGS];
    unsigned rowmax = RR_NOT_YET;
    for (int s = -3; s < n; ++s)
        pipe_step<XT>(x, V, nleaves, nb, nb2, g, G, s, n, P, Q, parked + threadIdx.x, rowmax, wsmax, wssum, sync_words, wait_limit,
                      sleep_units, &lds, per_block, out);
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

// How many workgroups of logsoftmax_pipe_kernel the current device holds at a time (asked once per device and
// element type; 0 if the runtime cannot say, and then the kernel is not used).
template <int XT>
static int pipe_resident_workgroups() {
    constexpr int MAXDEV = 64;
    static std::atomic<int> cached[MAXDEV];             // 0: not asked yet, -1: unknown
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAXDEV) return 0;
    int v = cached[dev].load();
    if (v == 0) {
        int per_cu = 0, cus = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, logsoftmax_pipe_kernel<XT>, RR_THREADS, 0) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || per_cu <= 0 || cus <= 0) {
            (void)hipGetLastError();
            v = -1;
        } else {
            v = per_cu * cus;
        }
        cached[dev].store(v);
    }
    return v > 0 ? v : 0;
}

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
            // From two rounds of resident workgroups on, the pipelined kernel: measured at V = 151936, fp32,
            // 512 rows 160 -> 135 us, 128 rows 40.4 -> 38.5 us, 64 rows (1.2 rounds) 23.6 -> 26.8 us.  Its grid is all the
            // device holds (a smaller grid that gives every workgroup the same number of items measured slower:
            // 973 workgroups 138 us, 1024 135 us).
            const int resident = pipe_resident_workgroups<XT>();
            const int64_t items = (int64_t)mc * nb;
            if (resident > 0 && nb <= RR_MAX_PIPE_BLOCKS && items >= 2 * (int64_t)resident) {
                const int pipe_grid = resident;
                hipLaunchKernelGGL((logsoftmax_pipe_kernel<XT>), dim3((unsigned)pipe_grid), block, 0, s, xp, V, nb, nb2, items, w0, w1,
                                   words, g_wait_limit.load(), /* units of s_sleep 8 between looks */ 4, o + m0 * V);
            } else {
                // Waiting costs the others bandwidth: a wavefront that polls takes issue slots and memory requests from
                // the workgroups that stream.  When the launch fills the device, a workgroup sleeps about 2 us
                // (2 x s_sleep 32) before its first look -- no hand-off completes sooner -- and about 0.5 us between
                // looks (measured at 512 x 151936: 200 us without the first sleep, 171 us with it, 191 us with twice as
                // long; M = 1 loses 3 us with it, so small launches look at once).  Two blocks per workgroup measured
                // slower (195 -> 282 us: 170 registers, three workgroups per compute unit).
                const int sleep_units = ((items >= 256 ? 2 : 0) << 8) | 2;
                hipLaunchKernelGGL((logsoftmax_coop_kernel<XT, 1>), dim3((unsigned)items), block, 0, s, xp, V, nb, nb2, w0, w1, words,
                                   g_wait_limit.load(), sleep_units, o + m0 * V);
            }
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
