// Device-side helpers shared by the TBIK kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tbik {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

// bf16 (bit pattern) -> fp32, exact.
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t h) { return __uint_as_float(h << 16); }

// fp32 -> bf16, round to nearest even (the single rounding of an output element), done by the conversion
// instruction of gfx950 (v_cvt_pk_bf16_f32 under the default rounding mode); two values per instruction.
typedef __bf16 tbik_bf16x2 __attribute__((ext_vector_type(2)));
typedef float tbik_f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    const tbik_f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, tbik_bf16x2));
}
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) { return pack_bf16x2(f, 0.0f) & 0xffffu; }

// The same for IEEE binary16 outputs (v_cvt_f16_f32 under the default rounding mode, fp16 denormals kept).
typedef _Float16 tbik_f16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_f16x2(float lo, float hi) {
    const tbik_f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, tbik_f16x2));
}
template <bool F16>
__device__ __forceinline__ uint32_t pack_16x2(float lo, float hi) { return F16 ? pack_f16x2(lo, hi) : pack_bf16x2(lo, hi); }
template <bool F16>
__device__ __forceinline__ uint32_t f32_to_16_bits(float f) { return pack_16x2<F16>(f, 0.0f) & 0xffffu; }

// The value a 16-bit tensor element gets when v is stored to it (one rounding, then the exact widening).
template <bool F16>
__device__ __forceinline__ float through_16_bits(float v) {
    if constexpr (F16) return (float)(_Float16)v;
    else return bf16_bits_to_f32(f32_to_bf16_bits(v));
}

// The gated activation between the two MLP GEMMs (implementation appendix, "other kernels"): SiLU(g) * u with
// SiLU(g) = g / (1 + e^-g), in fp32.  The exponential and the reciprocal are the hardware's approximations
// (v_exp_f32 of g * -log2(e), v_rcp_f32: about one fp32 ulp each), each product is one rounded multiplication.
// Position-wise, and the one definition for every kernel that applies it, so an element's bits do not depend on the
// kernel, the batch or the launch.  For g below about -87 the reciprocal leaves the normal range and the result may
// flush to zero (true magnitude below 1e-36).
__device__ __forceinline__ float silu_mul(float g, float u) {
    const float e = __builtin_amdgcn_exp2f(g * -1.4426950408889634f);
    float act = (g * __builtin_amdgcn_rcpf(1.0f + e)) * u;
    // The fp32 product is a value of its own: without this the compiler may merge the last multiplication with a
    // following conversion to binary16 into one mixed-precision instruction, which rounds once where the definition
    // rounds twice (seen: one element in 10^5 off by a step, and only in the callers where the merge applied).
    asm("" : "+v"(act));
    return act;
}

// Eight 16-bit values (one 16-byte chunk) of either format -> fp32, exact.
template <bool F16>
__device__ __forceinline__ void unpack8(const uint4 &v, float (&f)[8]) {
    if constexpr (F16) {
        typedef _Float16 h8 __attribute__((ext_vector_type(8)));
        typedef float f8 __attribute__((ext_vector_type(8)));
        const f8 r = __builtin_convertvector(__builtin_bit_cast(h8, v), f8);
#pragma unroll
        for (int e = 0; e < 8; ++e) f[e] = r[e];
    } else {
        f[0] = bf16_bits_to_f32(v.x & 0xffffu); f[1] = bf16_bits_to_f32(v.x >> 16);
        f[2] = bf16_bits_to_f32(v.y & 0xffffu); f[3] = bf16_bits_to_f32(v.y >> 16);
        f[4] = bf16_bits_to_f32(v.z & 0xffffu); f[5] = bf16_bits_to_f32(v.z >> 16);
        f[6] = bf16_bits_to_f32(v.w & 0xffffu); f[7] = bf16_bits_to_f32(v.w >> 16);
    }
}

// One MFMA of the GEMM kernels: D = A(32x16) * B(16x32) + C with 16-bit operands of either format held as
// eight 16-bit patterns per lane.  Both opcodes share the operand layout.
typedef _Float16 f16x8 __attribute__((__vector_size__(8 * sizeof(_Float16))));
template <bool F16>
__device__ __forceinline__ f32x16 mfma_32x32x16(bf16x8 a, bf16x8 b, f32x16 c) {
    if constexpr (F16)
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// global_load_lds_dwordx4: every lane fetches 16 bytes from uniform base + its own 32-bit byte offset + OFFSET;
// lane i's bytes land at LDS address m0 + OFFSET + 16*i (the instruction offset moves both addresses).  Written in
// assembly so that the compiler does not see an LDS write it would guard with a full wait before later LDS reads;
// completion is tracked by hand with vmcnt (above).  m0 is an operand, so one value serves all loads of a stage.
// AFTER_M0_WRITE: the instruction may directly follow the write of m0, which needs one wait state.
template <int OFFSET, bool AFTER_M0_WRITE>
__device__ __forceinline__ void load_16B_per_lane_to_lds(const void *uniform_base, unsigned lane_offset, unsigned m0_value) {
    static_assert(OFFSET >= -4096 && OFFSET < 4096, "13-bit signed instruction offset");
    if (AFTER_M0_WRITE)
        asm volatile("s_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 offset:%2"
                     ::"v"(lane_offset), "s"(uniform_base), "n"(OFFSET), "{m0}"(m0_value) : "memory");
    else
        asm volatile("global_load_lds_dwordx4 %0, %1 offset:%2"
                     ::"v"(lane_offset), "s"(uniform_base), "n"(OFFSET), "{m0}"(m0_value) : "memory");
}

// The 4-byte form (global_load_lds_dword): lane i's 4 bytes land at LDS address m0 + OFFSET + 4*i.
template <int OFFSET, bool AFTER_M0_WRITE>
__device__ __forceinline__ void load_4B_per_lane_to_lds(const void *uniform_base, unsigned lane_offset, unsigned m0_value) {
    static_assert(OFFSET >= -4096 && OFFSET < 4096, "13-bit signed instruction offset");
    if (AFTER_M0_WRITE)
        asm volatile("s_nop 0\n\tglobal_load_lds_dword %0, %1 offset:%2"
                     ::"v"(lane_offset), "s"(uniform_base), "n"(OFFSET), "{m0}"(m0_value) : "memory");
    else
        asm volatile("global_load_lds_dword %0, %1 offset:%2"
                     ::"v"(lane_offset), "s"(uniform_base), "n"(OFFSET), "{m0}"(m0_value) : "memory");
}

// Tells the compiler that a pointer is the same in every lane (it then lives in scalar registers).
__device__ __forceinline__ const char *uniform_pointer(const char *p) {
    const uint64_t v = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return reinterpret_cast<const char *>(((uint64_t)hi << 32) | lo);
}

// T over P = 2^t values held in registers, in the order of Alg. 2's reduce phase: at level l, value r
// (r mod 2^(l+1) == 0) receives value r + 2^l.  The array is used as scratch.
template <int P>
__device__ __forceinline__ float tree_of(float (&v)[P]) {
#pragma unroll
    for (int s = 1; s < P; s *= 2) {
#pragma unroll
        for (int r = 0; r < P; r += 2 * s) v[r] = v[r] + v[r + s];
    }
    return v[0];
}

// Streaming evaluation of the tree operator T (App. C) by the carry-over scheme of App. D.1:
// values arrive in index order; slot l holds a finished subtree of 2^l values that waits for its
// right sibling.  push(v, idx) folds value number idx in and returns the running value, which after
// the last value (idx = 2^t - 1) is T of all of them.  `idx` must be wave-uniform so that the
// slots are addressed statically (they stay in registers).
template <int LEVELS>
struct TreeStash {
    float s[LEVELS > 0 ? LEVELS : 1];
    __device__ __forceinline__ float push(float v, unsigned idx) {
        const int t = __builtin_ctz(~idx);          // number of trailing one bits of idx
#pragma unroll
        for (int l = 0; l < LEVELS; ++l)
            if (l < t) v = s[l] + v;                // left sibling (earlier) + right sibling (later)
#pragma unroll
        for (int l = 0; l < LEVELS; ++l)
            if (l == t) s[l] = v;
        return v;
    }
};

// The value of another lane of the same row of 16 lanes, chosen by a data-parallel-primitive control word: no trip
// through the LDS crossbar, the move folds into the instruction that uses it.
// 0xB1: quad_perm [1,0,3,2] (lane ^ 1); 0x4E: quad_perm [2,3,0,1] (lane ^ 2); 0x141: mirror within 8 lanes; 0x140:
// mirror within 16 lanes.
template <int CTRL>
__device__ __forceinline__ float from_lane_in_row(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false));
}
__device__ __forceinline__ float value_of_lane(float v, int lane) {
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}

// T over the 64 lanes of a wavefront (lane index = leaf index): levels 0..5.  Every lane gets the result.  All 64
// lanes must be active.  Levels 0..3 pair a lane with one whose value is the sibling subtree's sum: lane ^ 1,
// lane ^ 2, then the mirror image within 8 and within 16 lanes -- after level l all lanes of an aligned group of
// 2^(l+1) hold the same bits (the additions are the same up to the order of the two operands), so any lane of the
// sibling group will do.  Levels 4 and 5 take the four row sums through scalar registers.
__device__ __forceinline__ float wave_tree_sum(float v) {
    v = v + from_lane_in_row<0xB1>(v);
    v = v + from_lane_in_row<0x4E>(v);
    v = v + from_lane_in_row<0x141>(v);
    v = v + from_lane_in_row<0x140>(v);
    const float r0 = value_of_lane(v, 0), r1 = value_of_lane(v, 16), r2 = value_of_lane(v, 32), r3 = value_of_lane(v, 48);
    return (r0 + r1) + (r2 + r3);
}

__device__ __forceinline__ float wave_max(float v) {
    v = fmaxf(v, from_lane_in_row<0xB1>(v));
    v = fmaxf(v, from_lane_in_row<0x4E>(v));
    v = fmaxf(v, from_lane_in_row<0x141>(v));
    v = fmaxf(v, from_lane_in_row<0x140>(v));
    const float r0 = value_of_lane(v, 0), r1 = value_of_lane(v, 16), r2 = value_of_lane(v, 32), r3 = value_of_lane(v, 48);
    return fmaxf(fmaxf(r0, r1), fmaxf(r2, r3));
}

}  // namespace tbik
